// Neighbourhood encoding with attention coefficients (Sec. 3.3.1, first equation; gfx950).
//
// The paper gives K heads, one weight matrix per head and a coefficient gamma^k_ij per
// neighbour j of node i (i included) without a formula for gamma; this build takes it as
// graph attention networks do:
//     z_j = W e'_j,   u_ij = LeakyReLU_0.2(a_src . z_i + a_dst . z_j)   per head,
//     gamma_ij = softmax over j in N_i,   e_i = ReLU(sum_j gamma_ij z_j + b),
// with N_i = (i, predecessors ascending, successors ascending) and heads being contiguous
// blocks of H / K columns.  z = h W is a dense contraction (update_kernel); here are the
// two kernels that follow it: the score terms per node and head, and the weighted sums.
//
// A row of z is served by LPR = H / 8 lanes, eight columns each (16 bytes in bf16, 32 in
// fp32); a head's Dh = H / K columns sit in Dh / 8 adjacent lanes, so the reductions over a
// head are butterflies over those lanes.  H and K are powers of two, Dh >= 8.
#include "common.h"

namespace dc {
namespace {

typedef unsigned short u16;
typedef unsigned v4u __attribute__((ext_vector_type(4)));

template <bool kBf16>
__device__ __forceinline__ void load8(const void* base, size_t row, int H, int ll, float (&x)[8]) {
  if constexpr (kBf16) {
    const v4u r = reinterpret_cast<const v4u*>(base)[row * (size_t)(H >> 3) + ll];
    x[0] = __uint_as_float(r.x << 16);
    x[1] = __uint_as_float(r.x & 0xFFFF0000u);
    x[2] = __uint_as_float(r.y << 16);
    x[3] = __uint_as_float(r.y & 0xFFFF0000u);
    x[4] = __uint_as_float(r.z << 16);
    x[5] = __uint_as_float(r.z & 0xFFFF0000u);
    x[6] = __uint_as_float(r.w << 16);
    x[7] = __uint_as_float(r.w & 0xFFFF0000u);
  } else {
    const float4* p = reinterpret_cast<const float4*>(base) + row * (size_t)(H >> 2) + 2 * ll;
    const float4 a = p[0], b = p[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}

// s[v][k] = a_src^k . z^k_v and t[v][k] = a_dst^k . z^k_v for every node v and head k.
template <bool kBf16>
__global__ __launch_bounds__(256) void attention_scores_kernel(const void* __restrict__ z, int H, int K,
                                                                const float* __restrict__ att,
                                                                float* __restrict__ sc_src, float* __restrict__ sc_dst,
                                                                const int* __restrict__ node_off, int C,
                                                                const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int ntot = node_off[C];
  const int LPR = H >> 3, LPH = LPR / K;       // lanes per row, lanes per head
  const int lane = threadIdx.x & 63, sg = lane / LPR, ll = lane - sg * LPR;
  const int rows_per_wave = 64 / LPR;
  const long long wave0 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
  float as[8], ad[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    as[i] = att[ll * 8 + i];
    ad[i] = att[H + ll * 8 + i];
  }
  for (long long r0 = wave0 * rows_per_wave; r0 < ntot; r0 += nwaves * rows_per_wave) {
    const long long v = r0 + sg;
    float ps = 0.f, pd = 0.f;
    if (v < ntot) {
      float x[8];
      load8<kBf16>(z, (size_t)v, H, ll, x);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        ps += as[i] * x[i];
        pd += ad[i] * x[i];
      }
    }
    for (int o = 1; o < LPH; o <<= 1) {          // the head's lanes are adjacent and LPH-aligned
      ps += __shfl_xor(ps, o, 64);
      pd += __shfl_xor(pd, o, 64);
    }
    if (v < ntot && (ll % LPH) == 0) {
      sc_src[v * K + ll / LPH] = ps;
      sc_dst[v * K + ll / LPH] = pd;
    }
  }
}

// e_i = ReLU(sum over j in N_i of gamma_ij z_j + b): one group of LPR lanes per node walks
// the list (i, predecessors, successors) once, keeping a running maximum of the scores and
// rescaling the partial sums when it grows (the usual single-pass softmax), fp32 throughout.
// The group's lanes fetch up to LPR neighbour ids in one load and hand them round; rows and
// score terms of four neighbours are in flight at a time.  Held to 64 registers so that eight
// waves share a SIMD: the walk is a chain of dependent loads and only occupancy hides it.
template <bool kBf16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8))) void attention_aggregate_kernel(
    const void* __restrict__ z, int H, int K, const float* __restrict__ sc_src, const float* __restrict__ sc_dst,
    const float* __restrict__ bias, const int* __restrict__ in_rp, const int* __restrict__ in_ci,
    const int* __restrict__ out_rp, const int* __restrict__ out_ci, void* __restrict__ out,
    const int* __restrict__ node_off, int C, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int ntot = node_off[C];
  const int LPR = H >> 3, LPH = LPR / K;
  const int lane = threadIdx.x & 63, sg = lane / LPR, ll = lane - sg * LPR, hb = sg * LPR;
  const int head = ll / LPH;
  const int rows_per_wave = 64 / LPR, rows_per_wg = rows_per_wave * (blockDim.x >> 6);
  // Workgroups are dealt round-robin to the eight XCDs, each with its own L2: every XCD takes
  // one contiguous eighth of the rows, so that the neighbours of its rows (a graph is a few
  // hundred KB of z) are fetched into one L2 only.  The grid is a multiple of 8 workgroups.
  const long long n_chunks = (ntot + rows_per_wg - 1) / rows_per_wg;
  const int xcd = blockIdx.x & 7, jx = blockIdx.x >> 3, per_x = gridDim.x >> 3;
  const long long c_begin = n_chunks * xcd / 8, c_end = n_chunks * (xcd + 1) / 8;
  for (long long chunk = c_begin + jx; chunk < c_end; chunk += per_x) {
    const long long v = chunk * rows_per_wg + (threadIdx.x >> 6) * rows_per_wave + sg;
    if (v >= ntot) continue;                     // whole lane groups drop out together
    const int is = in_rp[v], din = in_rp[v + 1] - is;
    const int os = out_rp[v], dout = out_rp[v + 1] - os;
    const int n = 1 + din + dout;
    const float si = sc_src[v * K + head];
    float m = -INFINITY, den = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int b0 = 0; b0 < n; b0 += LPR) {
      const int nb = min(LPR, n - b0);
      int mine = 0;
      {
        const int q = b0 + ll;                    // position in N_i
        if (ll < nb) mine = q == 0 ? (int)v : (q <= din ? in_ci[is + q - 1] : out_ci[os + q - 1 - din]);
      }
      for (int k = 0; k < nb; k += 4) {
        int id[4];
        float tj[4], x[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          id[u] = __shfl(mine, hb + min(k + u, nb - 1), 64);       // past the end: repeats the last one, unused
          tj[u] = sc_dst[(size_t)id[u] * K + head];
          load8<kBf16>(z, (size_t)id[u], H, ll, x[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (k + u < nb) {
            float e = si + tj[u];
            e = e > 0.f ? e : 0.2f * e;
            const float mn = fmaxf(m, e);
            const float scale = __expf(m - mn);   // 0 at the first neighbour (m = -inf)
            const float p = __expf(e - mn);
            den = den * scale + p;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = acc[i] * scale + p * x[u][i];
            m = mn;
          }
        }
      }
    }
    const float inv = 1.0f / den;                 // N_i holds at least i itself
    float y[8];
    {
      const float4 b0 = *reinterpret_cast<const float4*>(bias + ll * 8);        // read here, not kept across
      const float4 b1 = *reinterpret_cast<const float4*>(bias + ll * 8 + 4);    // the walk: registers are scarce
      y[0] = fmaxf(acc[0] * inv + b0.x, 0.f);
      y[1] = fmaxf(acc[1] * inv + b0.y, 0.f);
      y[2] = fmaxf(acc[2] * inv + b0.z, 0.f);
      y[3] = fmaxf(acc[3] * inv + b0.w, 0.f);
      y[4] = fmaxf(acc[4] * inv + b1.x, 0.f);
      y[5] = fmaxf(acc[5] * inv + b1.y, 0.f);
      y[6] = fmaxf(acc[6] * inv + b1.z, 0.f);
      y[7] = fmaxf(acc[7] * inv + b1.w, 0.f);
    }
    if constexpr (kBf16) {
      v4u o;
      o.x = pack_bf16x2(y[0], y[1]);
      o.y = pack_bf16x2(y[2], y[3]);
      o.z = pack_bf16x2(y[4], y[5]);
      o.w = pack_bf16x2(y[6], y[7]);
      reinterpret_cast<v4u*>(out)[(size_t)v * LPR + ll] = o;
    } else {
      float4* p = reinterpret_cast<float4*>(out) + (size_t)v * (H >> 2) + 2 * ll;
      p[0] = make_float4(y[0], y[1], y[2], y[3]);
      p[1] = make_float4(y[4], y[5], y[6], y[7]);
    }
  }
}

}  // namespace

bool attention_shape_supported(int H, int heads) {
  const bool pow2_h = H >= 32 && H <= 512 && (H & (H - 1)) == 0;
  const bool pow2_k = heads >= 1 && (heads & (heads - 1)) == 0;
  return pow2_h && pow2_k && H / heads >= 8;
}

hipError_t launch_attention_scores(const GnnArgs& a, const void* z, const float* att_l, hipStream_t s) {
  const dim3 grid(a.n_cu * 8), block(256);
  if (a.bf16)
    hipLaunchKernelGGL(attention_scores_kernel<true>, grid, block, 0, s, z, a.H, a.heads, att_l, a.score[0],
                       a.score[1], a.node_off, a.n_cand, a.status);
  else
    hipLaunchKernelGGL(attention_scores_kernel<false>, grid, block, 0, s, z, a.H, a.heads, att_l, a.score[0],
                       a.score[1], a.node_off, a.n_cand, a.status);
  return hipGetLastError();
}

hipError_t launch_attention_aggregate(const GnnArgs& a, const void* z, const float* bias, void* out, hipStream_t s) {
  const dim3 grid(a.n_cu * 8), block(256);      // 8 waves per SIMD: every workgroup resident from the start
  if (a.bf16)
    hipLaunchKernelGGL(attention_aggregate_kernel<true>, grid, block, 0, s, z, a.H, a.heads, a.score[0], a.score[1],
                       bias, a.in_rowptr, a.in_col, a.out_rowptr, a.out_col, out, a.node_off, a.n_cand, a.status);
  else
    hipLaunchKernelGGL(attention_aggregate_kernel<false>, grid, block, 0, s, z, a.H, a.heads, a.score[0], a.score[1],
                       bias, a.in_rowptr, a.in_col, a.out_rowptr, a.out_col, out, a.node_off, a.n_cand, a.status);
  return hipGetLastError();
}

}  // namespace dc

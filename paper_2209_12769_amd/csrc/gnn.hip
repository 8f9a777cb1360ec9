// Estimator forward pass over a block-diagonal batch of contracted graphs (gfx950).
//
// Per layer (neighbourhood encoding, Sec. 3.3.1, with uniform coefficients and
// one weight block each for the node itself, its predecessors and successors):
//     h_in[v]  = mean over predecessors u of h[u]      (0 if none)
//     h_out[v] = mean over successors  w of h[w]       (0 if none)
//     h'[v]    = ReLU([h[v] | h_in[v] | h_out[v]] W + b)
// then a sum over the nodes of each graph (Sec. 3.3.1, second equation) and a
// head of fully connected layers with ReLU and a scalar output (Sec. 3.3.2).
//
// Kernels: aggregate (HBM/L2-bound gather), update (the dense contraction, on
// MFMA: bf16 32x32x16 with fp32 accumulation, or fp32 32x32x2), readout_head.
// All grids are sized from the device-resident node total, so no host
// synchronisation is needed between contraction and forward pass.
#include <string.h>

#include "common.h"

namespace dc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16;

__device__ __forceinline__ float bf2f(u16 x) { return __uint_as_float((unsigned)x << 16); }

// ---------------------------------------------------------------------------
// aggregate: one 16-byte column chunk of one (node, direction) per lane group
// ---------------------------------------------------------------------------
template <bool kBf16>
__global__ __launch_bounds__(256) void aggregate_kernel(const void* __restrict__ h, int d,
                                                         const int* __restrict__ in_rp, const int* __restrict__ in_ci,
                                                         const int* __restrict__ out_rp,
                                                         const int* __restrict__ out_ci, void* __restrict__ h_in,
                                                         void* __restrict__ h_out, const int* __restrict__ node_off,
                                                         int C, const int* __restrict__ status) {
  if (status[0] != 0) return;
  constexpr int kPer = kBf16 ? 8 : 4;          // elements per 16-byte chunk
  const int cpr = d / kPer;                    // chunks per row
  const long long ntot = node_off[C];
  const long long total = 2 * ntot * cpr;
  const uint4* __restrict__ h4 = reinterpret_cast<const uint4*>(h);
  const unsigned one = bf16_one_reg();
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const long long item = idx / cpr;
    const int ch = (int)(idx - item * cpr);
    const long long v = item >> 1;
    const int dir = (int)(item & 1);
    const int* rp = dir ? out_rp : in_rp;
    const int* ci = dir ? out_ci : in_ci;
    const int s = rp[v], e = rp[v + 1];
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (kBf16) {
      // first neighbour unpacked exactly, the others added in ascending order
      if (e > s) {
        const uint4 x = h4[(size_t)ci[s] * cpr + ch];
        acc[0] = __uint_as_float(x.x << 16);
        acc[1] = __uint_as_float(x.x & 0xFFFF0000u);
        acc[2] = __uint_as_float(x.y << 16);
        acc[3] = __uint_as_float(x.y & 0xFFFF0000u);
        acc[4] = __uint_as_float(x.z << 16);
        acc[5] = __uint_as_float(x.z & 0xFFFF0000u);
        acc[6] = __uint_as_float(x.w << 16);
        acc[7] = __uint_as_float(x.w & 0xFFFF0000u);
      }
      for (int k = s + 1; k < e; ++k) {
        const uint4 x = h4[(size_t)ci[k] * cpr + ch];
        bf16_pair_add(acc[0], acc[1], x.x, one);
        bf16_pair_add(acc[2], acc[3], x.y, one);
        bf16_pair_add(acc[4], acc[5], x.z, one);
        bf16_pair_add(acc[6], acc[7], x.w, one);
      }
    } else {
      for (int k = s; k < e; ++k) {
        const uint4 x = h4[(size_t)ci[k] * cpr + ch];
        acc[0] += __uint_as_float(x.x);
        acc[1] += __uint_as_float(x.y);
        acc[2] += __uint_as_float(x.z);
        acc[3] += __uint_as_float(x.w);
      }
    }
    const float sc = (e > s) ? 1.0f / (float)(e - s) : 0.0f;
    uint4 o;
    if (kBf16) {
      o.x = pack_bf16x2(acc[0] * sc, acc[1] * sc);
      o.y = pack_bf16x2(acc[2] * sc, acc[3] * sc);
      o.z = pack_bf16x2(acc[4] * sc, acc[5] * sc);
      o.w = pack_bf16x2(acc[6] * sc, acc[7] * sc);
    } else {
      o.x = __float_as_uint(acc[0] * sc);
      o.y = __float_as_uint(acc[1] * sc);
      o.z = __float_as_uint(acc[2] * sc);
      o.w = __float_as_uint(acc[3] * sc);
    }
    uint4* dst = reinterpret_cast<uint4*>(dir ? h_out : h_in);
    dst[(size_t)v * cpr + ch] = o;
  }
}

// ---------------------------------------------------------------------------
// update: h' = ReLU([h | h_in | h_out] W + b) on MFMA
// ---------------------------------------------------------------------------
// Tile BM x BN per workgroup, WM x WN per wave, K advanced in steps of BK that
// never straddle the three operand segments (BK divides d).
//   bf16: A tile in LDS row-major with a 16-byte pad per row (conflict-free
//         16-byte fragment reads); W is stored [k/8][H][8] so that the B tile is a
//         straight copy and fragment reads are contiguous across lanes.
//   fp32: A rows padded by one float, B rows padded to an odd multiple of 32.
template <bool kBf16, int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void update_kernel(
    const void* __restrict__ A0, const void* __restrict__ A1, const void* __restrict__ A2, int d, int nseg,
    const void* __restrict__ Wl, const float* __restrict__ bias, void* __restrict__ out, int H,
    const int* __restrict__ node_off, int C, int interleave, const int* __restrict__ status) {
  // nseg = 3: out = ReLU([A0 | A1 | A2] W + bias); nseg = 1 (bias == nullptr): out = A0 W.
  // interleave: the K chunks in the order of the sixteen-wave layer kernel (chunk c of A0, of A1, of A2, then
  // chunk c + 1 ...) instead of segment by segment, so that both add their products in the same order.
  if (status[0] != 0) return;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int ASTR = kBf16 ? (BK + 8) : (BK + 1);                     // elements per A row in LDS
  constexpr int BSTR = kBf16 ? BN * 8 : (BN + ((BN % 64 == 0) ? 32 : 0));  // elements per B "row"
  constexpr int A_BYTES = BM * ASTR * (kBf16 ? 2 : 4);
  constexpr int B_BYTES = (kBf16 ? (BK / 8) : BK) * BSTR * (kBf16 ? 2 : 4);
  __shared__ __attribute__((aligned(16))) char smem[A_BYTES + B_BYTES];
  u16* As16 = reinterpret_cast<u16*>(smem);
  u16* Bs16 = reinterpret_cast<u16*>(smem + A_BYTES);
  float* As32 = reinterpret_cast<float*>(smem);
  float* Bs32 = reinterpret_cast<float*>(smem + A_BYTES);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / (BN / WN), wn = wave % (BN / WN);
  const int l32 = lane & 31, lh = lane >> 5;
  const int ntot = node_off[C];
  const int nct = H / BN;
  const int ntiles = ((ntot + BM - 1) / BM) * nct;

  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int m0 = (tile / nct) * BM;
    const int n0 = (tile % nct) * BN;
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nch = d / BK;                   // chunks per segment
    for (int jc = 0; jc < nseg * nch; ++jc) {
      const int seg = interleave ? jc % nseg : jc / nch;
      const int koff = (interleave ? jc / nseg : jc - seg * nch) * BK;
      const int k0 = seg * d + koff;          // row of W
      const void* Aseg = seg == 0 ? A0 : (seg == 1 ? A1 : A2);
      if (kBf16) {
        constexpr int CH = BK / 8;   // 16-byte chunks per A row
        for (int i = t; i < BM * CH; i += NT) {
          const int r = i / CH, ch = i - r * CH;
          const int gr = m0 + r;
          uint4 x = make_uint4(0u, 0u, 0u, 0u);
          if (gr < ntot) x = *reinterpret_cast<const uint4*>(reinterpret_cast<const u16*>(Aseg) + (size_t)gr * d + koff + ch * 8);
          *reinterpret_cast<uint4*>(As16 + r * ASTR + ch * 8) = x;
        }
        const u16* Wp = reinterpret_cast<const u16*>(Wl);
        for (int i = t; i < CH * BN; i += NT) {
          const int k8 = i / BN, n = i - k8 * BN;
          const uint4 x = *reinterpret_cast<const uint4*>(Wp + ((size_t)(k0 / 8 + k8) * H + n0 + n) * 8);
          *reinterpret_cast<uint4*>(Bs16 + k8 * BSTR + n * 8) = x;
        }
      } else {
        constexpr int CH = BK / 4;   // float4 chunks per A row
        for (int i = t; i < BM * CH; i += NT) {
          const int r = i / CH, ch = i - r * CH;
          const int gr = m0 + r;
          float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
          if (gr < ntot) x = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(Aseg) + (size_t)gr * d + koff + ch * 4);
          float* p = As32 + r * ASTR + ch * 4;
          p[0] = x.x; p[1] = x.y; p[2] = x.z; p[3] = x.w;
        }
        const float* Wf = reinterpret_cast<const float*>(Wl);
        constexpr int CB = BN / 4;
        for (int i = t; i < BK * CB; i += NT) {
          const int kk = i / CB, c4 = i - kk * CB;
          const float4 x = *reinterpret_cast<const float4*>(Wf + (size_t)(k0 + kk) * H + n0 + c4 * 4);
          float* p = Bs32 + kk * BSTR + c4 * 4;
          p[0] = x.x; p[1] = x.y; p[2] = x.z; p[3] = x.w;
        }
      }
      __syncthreads();
      if (kBf16) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
          bf16x8 a[TM], b[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i)
            a[i] = *reinterpret_cast<const bf16x8*>(As16 + (wm * WM + i * 32 + l32) * ASTR + ks * 16 + lh * 8);
#pragma unroll
          for (int j = 0; j < TN; ++j)
            b[j] = *reinterpret_cast<const bf16x8*>(Bs16 + (ks * 2 + lh) * BSTR + (wn * WN + j * 32 + l32) * 8);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < BK / 2; ++ks) {
          float a[TM], b[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i) a[i] = As32[(wm * WM + i * 32 + l32) * ASTR + ks * 2 + lh];
#pragma unroll
          for (int j = 0; j < TN; ++j) b[j] = Bs32[(ks * 2 + lh) * BSTR + wn * WN + j * 32 + l32];
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
      }
      __syncthreads();
    }
    // epilogue: accumulator register v of lane (l32, lh) holds row 8*(v/4)+4*lh+(v%4), column l32
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WN + j * 32 + l32;
      const float bj = bias ? bias[col] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
          if (row < ntot) {
            const float y = bias ? fmaxf(acc[i][j][v] + bj, 0.f) : acc[i][j][v];
            if (kBf16) reinterpret_cast<u16*>(out)[(size_t)row * H + col] = to_bf16(y);
            else reinterpret_cast<float*>(out)[(size_t)row * H + col] = y;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// update, fp32, H a multiple of 128: the same product with the K loop software-pipelined
// ---------------------------------------------------------------------------
// Chunks of 16 along K, double-buffered in LDS: while a chunk multiplies, the next one's global loads
// are in flight and are stored to the other buffer afterwards (one barrier per chunk).  A in LDS
// row-major with a row stride of 17 floats (conflict-free 4-byte fragment reads), W rows as they lie
// in memory; MFMA block j of a wave takes columns 2l + j of its 64 (l = lane mod 32), so one 8-byte
// LDS read feeds both of a lane's B operands and results leave as 8-byte stores.
template <int BN, int WM>
__global__ __launch_bounds__(512) void update32_kernel(const float* __restrict__ A0, const float* __restrict__ A1,
                                                       const float* __restrict__ A2, int d, int nseg,
                                                       const float* __restrict__ Wf, const float* __restrict__ bias,
                                                       float* __restrict__ out, int H,
                                                       const int* __restrict__ node_off, int C,
                                                       const int* __restrict__ status) {
  if (status[0] != 0) return;
  constexpr int BM = 128, BK = 16, WN = 64, NT = 512;
  constexpr int TM = WM / 32;                         // 2 (BN = 256) or 1 (BN = 128)
  constexpr int ASTR = BK + 1, BSTR = BN + 32;
  constexpr int B_PER = (BK * BN / 4) / NT;           // 16-byte loads of W per thread and chunk
  static_assert((BM / WM) * (BN / WN) == 8 && (B_PER == 1 || B_PER == 2), "eight waves, one or two pieces of W each");
  __shared__ float As[2][BM * ASTR];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK * BSTR];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / (BN / WN), wn = wave % (BN / WN);
  const int l32 = lane & 31, lh = lane >> 5;
  const int ntot = node_off[C];
  const int nct = H / BN;
  const int ntiles = ((ntot + BM - 1) / BM) * nct;
  const int K = nseg * d, nk = K / BK;
  const int ar = t >> 2, ach = t & 3;                 // loader: one 16-byte piece of A per thread and chunk

  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int m0 = (tile / nct) * BM;
    const int n0 = (tile % nct) * BN;
    const bool arow_ok = m0 + ar < ntot;
    // per-thread pieces of a chunk: one 16-byte piece of A, B_PER of W (kk = row of the chunk, c4 = piece of the row)
    const size_t arow_off = (size_t)(m0 + ar) * d + ach * 4;
    int bkk[B_PER], bc4[B_PER];
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      bkk[u] = (t + u * NT) / (BN / 4);
      bc4[u] = (t + u * NT) % (BN / 4);
    }
    float4 ra = make_float4(0.f, 0.f, 0.f, 0.f), rb0, rb1 = make_float4(0.f, 0.f, 0.f, 0.f);
#define DC_UPDATE32_FETCH(c_)                                                                              \
    {                                                                                                      \
      const int k0_ = (c_) * BK;                                                                           \
      const int seg_ = k0_ / d;                                                                            \
      const float* Aseg_ = seg_ == 0 ? A0 : (seg_ == 1 ? A1 : A2);                                         \
      if (arow_ok) ra = *reinterpret_cast<const float4*>(Aseg_ + arow_off + (k0_ - seg_ * d));             \
      rb0 = *reinterpret_cast<const float4*>(Wf + (size_t)(k0_ + bkk[0]) * H + n0 + bc4[0] * 4);           \
      if constexpr (B_PER > 1)                                                                             \
        rb1 = *reinterpret_cast<const float4*>(Wf + (size_t)(k0_ + bkk[B_PER - 1]) * H + n0 + bc4[B_PER - 1] * 4); \
    }
#define DC_UPDATE32_STASH(buf_)                                                                            \
    {                                                                                                      \
      float* p_ = &As[buf_][ar * ASTR + ach * 4];                                                          \
      p_[0] = ra.x; p_[1] = ra.y; p_[2] = ra.z; p_[3] = ra.w;                                              \
      *reinterpret_cast<float4*>(&Bs[buf_][bkk[0] * BSTR + bc4[0] * 4]) = rb0;                             \
      if constexpr (B_PER > 1)                                                                             \
        *reinterpret_cast<float4*>(&Bs[buf_][bkk[B_PER - 1] * BSTR + bc4[B_PER - 1] * 4]) = rb1;           \
    }
    f32x16 acc[TM][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    DC_UPDATE32_FETCH(0)
    DC_UPDATE32_STASH(0)
    __syncthreads();
    for (int c = 0; c < nk; ++c) {
      const int buf = c & 1;
      if (c + 1 < nk) DC_UPDATE32_FETCH(c + 1)
      __builtin_amdgcn_sched_barrier(0);     // keep the global loads ahead of this chunk's products
#pragma unroll
      for (int ks = 0; ks < BK / 2; ++ks) {
        float a[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = As[buf][(wm * WM + i * 32 + l32) * ASTR + ks * 2 + lh];
        const float2 b2 = *reinterpret_cast<const float2*>(&Bs[buf][(ks * 2 + lh) * BSTR + wn * WN + l32 * 2]);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b2.x, acc[i][0], 0, 0, 0);
          acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b2.y, acc[i][1], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (c + 1 < nk) DC_UPDATE32_STASH(buf ^ 1)   // last read one chunk ago, before that chunk's barrier
      __syncthreads();
    }
#undef DC_UPDATE32_FETCH
#undef DC_UPDATE32_STASH
    // accumulator register v of lane (l32, lh) holds row 8*(v/4)+4*lh+(v%4) of its block; block j's
    // column l32 is column 2*l32 + j of the wave's 64
    const int col = n0 + wn * WN + l32 * 2;
    const float bj0 = bias ? bias[col] : 0.f, bj1 = bias ? bias[col + 1] : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
        if (row < ntot) {
          float2 y = make_float2(acc[i][0][v], acc[i][1][v]);
          if (bias) y = make_float2(fmaxf(y.x + bj0, 0.f), fmaxf(y.y + bj1, 0.f));
          *reinterpret_cast<float2*>(out + (size_t)row * H + col) = y;
        }
      }
  }
}

// ---------------------------------------------------------------------------
// readout + head: one workgroup per candidate; sums in fp64, fixed order.
//
// kOrder = 0: every column is summed over the graph's rows in fp64 (eight or four interleaved row
// sequences, then those in order).
// kOrder = 1, 2 (bf16, H = 256: the shapes of the bulk layer kernel, which can form the sums itself):
// the rows are taken in chunks of 64 consecutive global row numbers (chunk k = rows 64k .. 64k+63).
// Per chunk and column the 64 places -- a place holds the row's value if the row belongs to the
// graph, else +0 -- are summed in fp32 in one fixed tree (the one the bulk kernel's lane exchanges give):
//   u_l = place l + place l+32 (l < 32), A_l = u_l + u_{l+16} (l < 16), B_l = A_l + A_{15-l} (l < 8),
//   C_l = B_l + B_{7-l} (l < 4), sum = (C_0 + C_2) + (C_1 + C_3);
// the chunk sums of a graph are added in fp64 in ascending chunk order.  1 forms the chunk sums here from h; 2 reads them from `part`,
// where the last layer's kernel left them (the sum of chunk k for graph c at row k + c: both grow
// along the rows, so the place is unique).  The same tree on both routes: the same bits.
// ---------------------------------------------------------------------------
template <bool kBf16, int kOrder>
__global__ __launch_bounds__(256) void readout_head_kernel(const void* __restrict__ h, int H,
                                                            const int* __restrict__ node_off, int C,
                                                            const float* __restrict__ head, float* __restrict__ pred,
                                                            const float* __restrict__ part,
                                                            const int* __restrict__ status) {
  if (status[0] != 0) return;
  constexpr int kPer = kBf16 ? 8 : 4;
  __shared__ double red[kOrder == 0 ? 256 * kPer : 1];   // [row group][H] partial sums
  __shared__ float sub[kOrder == 1 ? 2 * 8 * 256 : 1];   // [buffer][row lane m][column]: B_m
  __shared__ float r[512], z[512];
  __shared__ double wred[4];
  const int c = blockIdx.x, t = threadIdx.x;
  const int n0 = node_off[c], n1 = node_off[c + 1];
  if constexpr (kOrder == 2) {
    // H = 256: thread t has column t
    double acc = 0.0;
    if (n1 > n0)
      for (int k = n0 >> 6; k <= (n1 - 1) >> 6; ++k) acc += (double)part[(size_t)(k + c) * 256 + t];
    r[t] = (float)acc;
  } else if constexpr (kOrder == 1) {
    // thread (row lane m = t / 32, 16-byte piece t % 32) forms B_m from its eight places; then thread t column t
    const int m = t >> 5, ch = t & 31;
    const uint4* h4 = reinterpret_cast<const uint4*>(h);
    double acc = 0.0;
    int buf = 0;
    if (n1 > n0)
      for (int k = n0 >> 6; k <= (n1 - 1) >> 6; ++k, buf ^= 1) {
        uint4 x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          // places m, m+32, m+16, m+48 (A_m), then 15-m, 47-m, 31-m, 63-m (A_{15-m})
          const int place = (i < 4 ? m : 15 - m) + 32 * (i & 1) + 16 * ((i >> 1) & 1);
          const int row = 64 * k + place;
          x[i] = (row >= n0 && row < n1) ? h4[(size_t)row * 32 + ch] : make_uint4(0u, 0u, 0u, 0u);
        }
        float* dst = sub + (buf * 8 + m) * 256 + ch * 8;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float lo[8], hi[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const unsigned v = w == 0 ? x[i].x : (w == 1 ? x[i].y : (w == 2 ? x[i].z : x[i].w));
            lo[i] = __uint_as_float(v << 16);
            hi[i] = __uint_as_float(v & 0xFFFF0000u);
          }
          dst[2 * w] = ((lo[0] + lo[1]) + (lo[2] + lo[3])) + ((lo[4] + lo[5]) + (lo[6] + lo[7]));
          dst[2 * w + 1] = ((hi[0] + hi[1]) + (hi[2] + hi[3])) + ((hi[4] + hi[5]) + (hi[6] + hi[7]));
        }
        __syncthreads();                    // two buffers: the next chunk's sums go to the other one
        const float* q = sub + buf * 8 * 256 + t;
        // B_0 .. B_7 at q[0], q[256], ...: ((B0 + B7) + (B2 + B5)) + ((B1 + B6) + (B3 + B4))
        acc += (double)(((q[0] + q[1792]) + (q[512] + q[1280])) + ((q[256] + q[1536]) + (q[768] + q[1024])));
      }
    r[t] = (float)acc;
  }
  if constexpr (kOrder == 0) {
  const int cpr = H / kPer;            // 16-byte chunks per row (<= 256 for H <= 1024)
  const int rg = 256 / cpr;            // rows handled in parallel
  const int myr = t / cpr, ch = t - myr * cpr;
  double acc[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) acc[i] = 0.0;
  if (myr < rg) {
    const uint4* h4 = reinterpret_cast<const uint4*>(h);
    for (int v = n0 + myr; v < n1; v += rg) {
      const uint4 x = h4[(size_t)v * cpr + ch];
      if constexpr (kBf16) {
        acc[0] += (double)__uint_as_float(x.x << 16);
        acc[1] += (double)__uint_as_float(x.x & 0xFFFF0000u);
        acc[2] += (double)__uint_as_float(x.y << 16);
        acc[3] += (double)__uint_as_float(x.y & 0xFFFF0000u);
        acc[4] += (double)__uint_as_float(x.z << 16);
        acc[5] += (double)__uint_as_float(x.z & 0xFFFF0000u);
        acc[6] += (double)__uint_as_float(x.w << 16);
        acc[7] += (double)__uint_as_float(x.w & 0xFFFF0000u);
      } else {
        acc[0] += (double)__uint_as_float(x.x);
        acc[1] += (double)__uint_as_float(x.y);
        acc[2] += (double)__uint_as_float(x.z);
        acc[3] += (double)__uint_as_float(x.w);
      }
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i) red[myr * H + ch * kPer + i] = acc[i];
  }
  __syncthreads();
  for (int j = t; j < H; j += 256) {
    double s = 0.0;
    for (int g = 0; g < rg; ++g) s += red[g * H + j];
    r[j] = (float)s;
  }
  }
  __syncthreads();
  const float* W1 = head;
  const float* b1 = W1 + (size_t)H * H;
  const float* W2 = b1 + H;
  const float* b2 = W2 + (size_t)H * H;
  const float* w3 = b2 + H;
  const float* b3 = w3 + H;
  for (int j = t; j < H; j += 256) {
    double s = b1[j];
    for (int k = 0; k < H; ++k) s += (double)r[k] * (double)W1[(size_t)k * H + j];
    z[j] = (float)(s > 0.0 ? s : 0.0);
  }
  __syncthreads();
  for (int j = t; j < H; j += 256) {
    double s = b2[j];
    for (int k = 0; k < H; ++k) s += (double)z[k] * (double)W2[(size_t)k * H + j];
    r[j] = (float)(s > 0.0 ? s : 0.0);     // r now holds z2
  }
  __syncthreads();
  double p = 0.0;
  for (int j = t; j < H; j += 256) p += (double)r[j] * (double)w3[j];
  for (int o = 32; o > 0; o >>= 1) p += __shfl_down(p, o, 64);
  if ((t & 63) == 0) wred[t >> 6] = p;
  __syncthreads();
  if (t == 0) pred[c] = (float)((double)b3[0] + wred[0] + wred[1] + wred[2] + wred[3]);
}

template <bool kBf16, int BM, int BN, int BK, int WM, int WN>
void launch_update(const GnnArgs& a, const void* A0, const void* A1, const void* A2, int d, int nseg, const void* Wl,
                   const float* bias, void* out, int interleave, hipStream_t s) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  hipLaunchKernelGGL((update_kernel<kBf16, BM, BN, BK, WM, WN>), dim3(a.n_cu * (kBf16 ? 2 : 4)), dim3(NT), 0, s, A0, A1, A2, d, nseg,
                     Wl, bias, out, a.H, a.node_off, a.n_cand, interleave, a.status);
}

template <bool kBf16, int BK>
void dispatch_update(const GnnArgs& a, const void* A0, const void* A1, const void* A2, int d, int nseg, const void* Wl,
                     const float* bias, void* out, int interleave, hipStream_t s) {
  const int H = a.H;
  if (H % 256 == 0) launch_update<kBf16, 128, 256, BK, 64, 64>(a, A0, A1, A2, d, nseg, Wl, bias, out, interleave, s);
  else if (H % 128 == 0) launch_update<kBf16, 128, 128, BK, 32, 64>(a, A0, A1, A2, d, nseg, Wl, bias, out, interleave, s);
  else if (H % 64 == 0) launch_update<kBf16, 128, 64, BK, 32, 32>(a, A0, A1, A2, d, nseg, Wl, bias, out, interleave, s);
  else launch_update<kBf16, 128, 32, BK, 32, 32>(a, A0, A1, A2, d, nseg, Wl, bias, out, interleave, s);
}

// [A0 | A1 | A2] W (nseg = 3) or A0 W (nseg = 1) with the chunk width the input width allows
void run_update(const GnnArgs& a, const void* A0, const void* A1, const void* A2, int d, int nseg, const void* Wl,
                const float* bias, void* out, hipStream_t s) {
  if (a.bf16) {
    // the shapes the sixteen-wave layer kernel serves add their K chunks in its order
    const int interleave = nseg == 3 && layer256_supported(d, a.H, a.bf16);
    if (d % 64 == 0) dispatch_update<true, 64>(a, A0, A1, A2, d, nseg, Wl, bias, out, interleave, s);
    else dispatch_update<true, 16>(a, A0, A1, A2, d, nseg, Wl, bias, out, 0, s);
  } else {
    const float* f0 = static_cast<const float*>(A0);
    const float* f1 = static_cast<const float*>(A1);
    const float* f2 = static_cast<const float*>(A2);
    if (a.H % 256 == 0)
      hipLaunchKernelGGL((update32_kernel<256, 64>), dim3(a.n_cu * 2), dim3(512), 0, s, f0, f1, f2, d, nseg,
                         static_cast<const float*>(Wl), bias, static_cast<float*>(out), a.H, a.node_off, a.n_cand,
                         a.status);
    else if (a.H % 128 == 0)
      hipLaunchKernelGGL((update32_kernel<128, 32>), dim3(a.n_cu * 2), dim3(512), 0, s, f0, f1, f2, d, nseg,
                         static_cast<const float*>(Wl), bias, static_cast<float*>(out), a.H, a.node_off, a.n_cand,
                         a.status);
    else
      dispatch_update<false, 16>(a, A0, A1, A2, d, nseg, Wl, bias, out, 0, s);
  }
}

}  // namespace

bool gnn_shape_supported(int F, int H, int L) {
  return F > 0 && H > 0 && L > 0 && F % 16 == 0 && H % 32 == 0 && H <= 512 && F <= 512;
}

size_t packed_weight_elems(int F, int H, int L, int nseg) {
  size_t n = 0;
  for (int l = 0; l < L; ++l) n += (size_t)nseg * (l == 0 ? F : H) * H;
  return n;
}

static unsigned short host_f2bf(float x) {
  unsigned u;
  memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) return (unsigned short)(u >> 16);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

void pack_weights_host(const float* W_layers, int F, int H, int L, int nseg, int bf16, void* dst) {
  if (!bf16) {
    memcpy(dst, W_layers, packed_weight_elems(F, H, L, nseg) * sizeof(float));
    return;
  }
  unsigned short* o = static_cast<unsigned short*>(dst);
  const float* w = W_layers;
  for (int l = 0; l < L; ++l) {
    const int K = nseg * (l == 0 ? F : H);
    for (int k = 0; k < K; ++k)
      for (int n = 0; n < H; ++n) o[((size_t)(k / 8) * H + n) * 8 + (k % 8)] = host_f2bf(w[(size_t)k * H + n]);
    o += (size_t)K * H;
    w += (size_t)K * H;
  }
}

namespace {

// Layers with attention coefficients: z = h W (dense), the two score terms per node and
// head, then the softmax-weighted sum over N_i with bias and ReLU.
hipError_t attention_layers(const GnnArgs& a, Profiler* prof, hipStream_t s, const void** h_last) {
  const void* hcur = a.Xc;
  int d = a.F;
  const size_t esz = a.bf16 ? 2 : 4;
  const char* Wl = static_cast<const char*>(a.W);
  const float* bl = a.b;
  const float* al = a.att;
  void* z = a.agg[0];
  for (int l = 0; l < a.L; ++l) {
    void* hnext = a.act[l & 1];
    if (prof) prof->begin(kFamAttProject, s);
    if (a.allow_fused && layer256_supported(d, a.H, a.bf16)) {
      hipError_t e = launch_dense256(hcur, d, a, Wl, nullptr, z, s);
      if (e != hipSuccess) return e;
    } else {
      run_update(a, hcur, nullptr, nullptr, d, 1, Wl, nullptr, z, s);
    }
    if (prof) prof->end(s);
    if (prof) prof->begin(kFamAttScores, s);
    hipError_t e = launch_attention_scores(a, z, al, s);
    if (prof) prof->end(s);
    if (e != hipSuccess) return e;
    if (prof) prof->begin(kFamAttAggregate, s);
    e = launch_attention_aggregate(a, z, bl, hnext, s);
    if (prof) prof->end(s);
    if (e != hipSuccess) return e;
    Wl += (size_t)d * a.H * esz;
    bl += a.H;
    al += 2 * a.H;
    hcur = hnext;
    d = a.H;
  }
  *h_last = hcur;
  return hipGetLastError();
}

// The sum readout follows chunks of 64 rows (see readout_head_kernel) where the last layer is one the bulk
// kernel takes, whichever kernels run it; that kernel can then leave the chunk sums instead of its rows.
bool chunked_readout(const GnnArgs& a) {
  return a.heads == 0 && layer256_supported(a.L > 1 ? a.H : a.F, a.H, a.bf16);
}
bool readout_in_last_layer(const GnnArgs& a) {
  return a.fuse_readout && a.allow_fused && chunked_readout(a) && a.ro_part && a.ro_first;
}

// Layers with uniform coefficients: mean over predecessors, mean over successors, dense update.
hipError_t mean_layers(const GnnArgs& a, Profiler* prof, hipStream_t s, const void** h_last) {
  const void* hcur = a.Xc;
  int d = a.F;
  const size_t esz = a.bf16 ? 2 : 4;
  const char* Wl = static_cast<const char*>(a.W);
  const float* bl = a.b;
  const int agg_grid = a.n_cu * 8;
  if (a.allow_fused && (layer256_supported(a.F, a.H, a.bf16) || (a.L > 1 && layer256_supported(a.H, a.H, a.bf16)))) {
    // neighbour descriptors depend on the graphs only: built once, used by every layer that gathers through them
    if (prof) prof->begin(kFamDesc, s);
    hipError_t e = launch_build_desc(a, s);
    if (e == hipSuccess && readout_in_last_layer(a)) e = launch_chunk_first(a, s);
    if (prof) prof->end(s);
    if (e != hipSuccess) return e;
  }
  for (int l = 0; l < a.L; ++l) {
    void* hnext = a.act[l & 1];
    if (a.allow_fused && layer256_supported(d, a.H, a.bf16)) {
      const bool readout = l == a.L - 1 && readout_in_last_layer(a);   // then hnext is not written
      hipError_t e = launch_layer256(hcur, d, a, Wl, bl, hnext, readout, prof, s);
      if (e != hipSuccess) return e;
    } else if (a.allow_fused && fused_layer_supported(d, a.H, a.bf16)) {
      if (prof) prof->begin(kFamFused, s);
      hipError_t e = launch_fused_layer(hcur, d, a, Wl, bl, hnext, s);
      if (prof) prof->end(s);
      if (e != hipSuccess) return e;
    } else {
      if (prof) prof->begin(kFamAggregate, s);
      if (a.bf16)
        hipLaunchKernelGGL(aggregate_kernel<true>, dim3(agg_grid), dim3(256), 0, s, hcur, d, a.in_rowptr, a.in_col,
                           a.out_rowptr, a.out_col, a.agg[0], a.agg[1], a.node_off, a.n_cand, a.status);
      else
        hipLaunchKernelGGL(aggregate_kernel<false>, dim3(agg_grid), dim3(256), 0, s, hcur, d, a.in_rowptr, a.in_col,
                           a.out_rowptr, a.out_col, a.agg[0], a.agg[1], a.node_off, a.n_cand, a.status);
      if (prof) prof->end(s);
      if (prof) prof->begin(kFamUpdate, s);
      run_update(a, hcur, a.agg[0], a.agg[1], d, 3, Wl, bl, hnext, s);
      if (prof) prof->end(s);
    }
    Wl += (size_t)3 * d * a.H * esz;
    bl += a.H;
    hcur = hnext;
    d = a.H;
  }
  *h_last = hcur;
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gnn_layers(const GnnArgs& a, Profiler* prof, hipStream_t s, const void** h_last) {
  return a.heads > 0 ? attention_layers(a, prof, s, h_last) : mean_layers(a, prof, s, h_last);
}

void launch_mean_aggregate(const GnnArgs& a, const void* h, int d, void* h_in, void* h_out, hipStream_t s) {
  if (a.bf16)
    hipLaunchKernelGGL(aggregate_kernel<true>, dim3(a.n_cu * 8), dim3(256), 0, s, h, d, a.in_rowptr, a.in_col,
                       a.out_rowptr, a.out_col, h_in, h_out, a.node_off, a.n_cand, a.status);
  else
    hipLaunchKernelGGL(aggregate_kernel<false>, dim3(a.n_cu * 8), dim3(256), 0, s, h, d, a.in_rowptr, a.in_col,
                       a.out_rowptr, a.out_col, h_in, h_out, a.node_off, a.n_cand, a.status);
}

void launch_dense_update(const GnnArgs& a, const void* A0, const void* A1, const void* A2, int d, int nseg,
                         const void* Wl, const float* bias, void* out, hipStream_t s) {
  run_update(a, A0, A1, A2, d, nseg, Wl, bias, out, s);
}

void launch_dense_bias_relu(const GnnArgs& a, const void* A, int d, const void* Wp, const float* bias, void* out,
                            hipStream_t s) {
  if (a.allow_fused && layer256_supported(d, a.H, a.bf16) && launch_dense256(A, d, a, Wp, bias, out, s) == hipSuccess)
    return;
  run_update(a, A, nullptr, nullptr, d, 1, Wp, bias, out, s);
}

hipError_t launch_gnn_forward(const GnnArgs& a, Profiler* prof, hipStream_t s) {
  if (a.n_cand <= 0) return hipSuccess;
  const void* hcur = nullptr;
  hipError_t e = launch_gnn_layers(a, prof, s, &hcur);
  if (e != hipSuccess) return e;
  if (prof) prof->begin(kFamReadout, s);
  if (a.bf16 && chunked_readout(a)) {
    if (readout_in_last_layer(a))
      hipLaunchKernelGGL((readout_head_kernel<true, 2>), dim3(a.n_cand), dim3(256), 0, s, hcur, a.H, a.node_off, a.n_cand,
                         a.head, a.pred, a.ro_part, a.status);
    else
      hipLaunchKernelGGL((readout_head_kernel<true, 1>), dim3(a.n_cand), dim3(256), 0, s, hcur, a.H, a.node_off, a.n_cand,
                         a.head, a.pred, static_cast<const float*>(nullptr), a.status);
  } else if (a.bf16) {
    hipLaunchKernelGGL((readout_head_kernel<true, 0>), dim3(a.n_cand), dim3(256), 0, s, hcur, a.H, a.node_off, a.n_cand,
                       a.head, a.pred, static_cast<const float*>(nullptr), a.status);
  } else {
    hipLaunchKernelGGL((readout_head_kernel<false, 0>), dim3(a.n_cand), dim3(256), 0, s, hcur, a.H, a.node_off, a.n_cand,
                       a.head, a.pred, static_cast<const float*>(nullptr), a.status);
  }
  if (prof) prof->end(s);
  return hipGetLastError();
}

}  // namespace dc

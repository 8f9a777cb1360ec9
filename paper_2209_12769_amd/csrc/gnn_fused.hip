// Fused message-passing layer for the bf16 path (gfx950):
//     h'[v] = ReLU([h[v] | mean_pred(h)[v] | mean_succ(h)[v]] W + b)
// with the two neighbour means (Sec. 3.3.1, neighbourhood encoding with uniform
// coefficients) computed while the A tile of the MFMA contraction is loaded, so
// neither mean is ever written to HBM: a layer reads h (gathers hit L2) and
// writes h'.
//
// Workgroup = 4 waves, tile 128 rows x BN (= H) columns, K = 3d in chunks of 64
// that never straddle the self / predecessor / successor segments.  Per chunk:
// the loads of the next chunk (B tile; A rows or the first two neighbours of each
// gathered row) are issued, the MFMAs of the current chunk run, then the gathered
// rows are reduced in fp32 (ascending neighbour order), scaled by 1/deg, rounded
// to bf16 and written to the other A buffer.  Two workgroups share a CU so one
// computes while the other loads.  The output tile goes through LDS so that
// global stores are full 16-byte, row-contiguous.
#include "common.h"

namespace dc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16;
typedef unsigned v4u __attribute__((ext_vector_type(4)));   // native 16-byte vector (plain loads, no struct copies)

constexpr int kBM = 128;
constexpr int kBK = 64;
constexpr int kNT = 256;
constexpr int kASTR = kBK + 8;   // A row stride in LDS (elements): 144 B, conflict-free 16-byte reads
constexpr int kCiCap = 1024;     // neighbour ids of one tile and direction staged in LDS
constexpr int kAItems = kBM * (kBK / 8) / kNT;   // 16-byte A chunks per thread and K chunk (4)

template <int BN>
struct Lds {
  static constexpr int A_BYTES = kBM * kASTR * 2;
  static constexpr int B_BYTES = (kBK / 8) * BN * 8 * 2;
  static constexpr int OSTR = BN + 8;
  static constexpr int O_BYTES = kBM * OSTR * 2;
  static constexpr int MAIN = (2 * A_BYTES + B_BYTES) > O_BYTES ? (2 * A_BYTES + B_BYTES) : O_BYTES;
  static constexpr int RP_OFF = MAIN;
  static constexpr int CI_OFF = RP_OFF + ((2 * (kBM + 1) * 4 + 15) & ~15);
  static constexpr int TOTAL = CI_OFF + 2 * kCiCap * 4;
};

__device__ __forceinline__ unsigned pack2(float a, float b) { return pack_bf16x2(a, b); }

__device__ __forceinline__ void set8(float* acc, const v4u x) {   // first neighbour: exact unpack
  acc[0] = __uint_as_float(x.x << 16);
  acc[1] = __uint_as_float(x.x & 0xFFFF0000u);
  acc[2] = __uint_as_float(x.y << 16);
  acc[3] = __uint_as_float(x.y & 0xFFFF0000u);
  acc[4] = __uint_as_float(x.z << 16);
  acc[5] = __uint_as_float(x.z & 0xFFFF0000u);
  acc[6] = __uint_as_float(x.w << 16);
  acc[7] = __uint_as_float(x.w & 0xFFFF0000u);
}
__device__ __forceinline__ void add8(float* acc, const v4u x, unsigned one) {   // further neighbours
  bf16_pair_add(acc[0], acc[1], x.x, one);
  bf16_pair_add(acc[2], acc[3], x.y, one);
  bf16_pair_add(acc[4], acc[5], x.z, one);
  bf16_pair_add(acc[6], acc[7], x.w, one);
}

extern __shared__ __attribute__((aligned(16))) char dc_fused_smem[];

template <int BN, int WM, int WN>
__global__ __launch_bounds__(kNT, 2) void fused_layer_kernel(
    const u16* __restrict__ h, int d, const int* __restrict__ in_rp, const int* __restrict__ in_ci,
    const int* __restrict__ out_rp, const int* __restrict__ out_ci, const u16* __restrict__ Wp,
    const float* __restrict__ bias, u16* __restrict__ out, const int* __restrict__ node_off, int C,
    const int* __restrict__ status) {
  using L = Lds<BN>;
  constexpr int WAVES_N = BN / WN;
  static_assert((kBM / WM) * WAVES_N * 64 == kNT, "wave grid must cover the tile");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kBItems = (kBK / 8) * BN / kNT;     // 16-byte B chunks per thread and K chunk
  if (status[0] != 0) return;

  char* smem = dc_fused_smem;
  u16* As0 = reinterpret_cast<u16*>(smem);
  u16* Bs = reinterpret_cast<u16*>(smem + 2 * L::A_BYTES);
  u16* Os = reinterpret_cast<u16*>(smem);
  int* s_rp = reinterpret_cast<int*>(smem + L::RP_OFF);   // [2][kBM+1]
  int* s_ci = reinterpret_cast<int*>(smem + L::CI_OFF);   // [2][kCiCap]

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  const int H = BN;
  const int cpr = d >> 3;                 // 16-byte chunks per row of h
  const int nk = 3 * d / kBK;
  const v4u* __restrict__ h4 = reinterpret_cast<const v4u*>(h);
  const int ar = t >> 3, ach = t & 7;     // this thread's A rows are ar + 32*i, 16-byte column ach
  const unsigned one = bf16_one_reg();

  // Each XCD (workgroups are dealt round-robin over the 8 XCDs) sweeps one contiguous
  // range of tiles, so the rows a tile gathers were written / read through the same L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per = gridDim.x >> 3;
  const int tpx = (ntiles + 7) >> 3;

  for (int it = slot; it < tpx; it += per) {
    const int tile = xcd * tpx + it;
    if (tile >= ntiles) break;
    const int m0 = tile * kBM;

    // ---- stage row pointers and neighbour ids of the tile ---------------------------
    for (int i = t; i <= kBM; i += kNT) {
      const int r = min(m0 + i, ntot);
      s_rp[i] = in_rp[r];
      s_rp[(kBM + 1) + i] = out_rp[r];
    }
    __syncthreads();
    const int e0_in = s_rp[0], e0_out = s_rp[kBM + 1];
    const int ne_in = s_rp[kBM] - e0_in, ne_out = s_rp[(kBM + 1) + kBM] - e0_out;
    const bool staged_in = ne_in <= kCiCap, staged_out = ne_out <= kCiCap;
    if (staged_in)
      for (int i = t; i < ne_in; i += kNT) s_ci[i] = in_ci[e0_in + i];
    if (staged_out)
      for (int i = t; i < ne_out; i += kNT) s_ci[kCiCap + i] = out_ci[e0_out + i];
    __syncthreads();

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    v4u ax[kAItems][2];
    int adeg[kAItems], ast[kAItems];

    // issue the global loads of K chunk kc
    auto issue = [&](int kc) __attribute__((always_inline)) {
      const int k0 = kc * kBK;
      const int seg = k0 / d;
      const int cc = ((k0 - seg * d) >> 3) + ach;      // 16-byte column inside a row of h
      if (seg == 0) {
#pragma unroll
        for (int i = 0; i < kAItems; ++i) {
          const int gr = m0 + ar + 32 * i;
          ax[i][0] = v4u{0u, 0u, 0u, 0u};
          if (gr < ntot) ax[i][0] = h4[(size_t)gr * cpr + cc];
        }
      } else {
        const int dir = seg - 1;
        const int* rp = s_rp + dir * (kBM + 1);
        const int e0d = dir ? e0_out : e0_in;
        const bool stg = dir ? staged_out : staged_in;
        const int* gci = (dir ? out_ci : in_ci) + e0d;
        const int* sci = s_ci + dir * kCiCap;
#pragma unroll
        for (int i = 0; i < kAItems; ++i) {
          const int r = ar + 32 * i;
          const int s = rp[r] - e0d;
          const int dg = rp[r + 1] - rp[r];
          ast[i] = s;
          adeg[i] = dg;
          ax[i][0] = v4u{0u, 0u, 0u, 0u};
          ax[i][1] = v4u{0u, 0u, 0u, 0u};
          if (dg > 0) {
            const int u0 = stg ? sci[s] : gci[s];
            ax[i][0] = h4[(size_t)u0 * cpr + cc];
          }
          if (dg > 1) {
            const int u1 = stg ? sci[s + 1] : gci[s + 1];
            ax[i][1] = h4[(size_t)u1 * cpr + cc];
          }
        }
      }
    };
    // finish the A rows of chunk kc (reduce gathered rows) and write them to LDS buffer dst
    auto finish_a = [&](int kc, u16* dst) __attribute__((always_inline)) {
      const int k0 = kc * kBK;
      const int seg = k0 / d;
      if (seg == 0) {
#pragma unroll
        for (int i = 0; i < kAItems; ++i)
          *reinterpret_cast<v4u*>(dst + (ar + 32 * i) * kASTR + ach * 8) = ax[i][0];
      } else {
        const int dir = seg - 1;
        const int cc = ((k0 - seg * d) >> 3) + ach;
        const bool stg = dir ? staged_out : staged_in;
        const int* gci = (dir ? out_ci : in_ci) + (dir ? e0_out : e0_in);
        const int* sci = s_ci + dir * kCiCap;
#pragma unroll
        for (int i = 0; i < kAItems; ++i) {
          float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          const int dg = adeg[i], s = ast[i];
          if (dg > 0) set8(a8, ax[i][0]);
          if (dg > 1) add8(a8, ax[i][1], one);
          for (int u = 2; u < dg; ++u) {
            const int un = stg ? sci[s + u] : gci[s + u];
            const v4u x = h4[(size_t)un * cpr + cc];
            add8(a8, x, one);
          }
          const float sc = dg > 0 ? 1.0f / (float)dg : 0.0f;
          v4u o;
          o.x = pack2(a8[0] * sc, a8[1] * sc);
          o.y = pack2(a8[2] * sc, a8[3] * sc);
          o.z = pack2(a8[4] * sc, a8[5] * sc);
          o.w = pack2(a8[6] * sc, a8[7] * sc);
          *reinterpret_cast<v4u*>(dst + (ar + 32 * i) * kASTR + ach * 8) = o;
        }
      }
    };
    // kc = -1 is the prologue: it only loads chunk 0
    for (int kc = -1; kc < nk; ++kc) {
      const u16* Acur = As0 + (kc & 1) * (L::A_BYTES / 2);
      u16* Anext = As0 + ((kc + 1) & 1) * (L::A_BYTES / 2);
      const bool more = kc + 1 < nk;
      v4u bx[kBItems];
      {
        // W is stored [k/8][H][8]: the B tile of a chunk is one contiguous run
        // (the last iteration reloads the last chunk and drops it)
        const int kn = more ? kc + 1 : kc;
        const v4u* wsrc = reinterpret_cast<const v4u*>(Wp) + (size_t)(kn * (kBK / 8)) * H;
#pragma unroll
        for (int i = 0; i < kBItems; ++i) bx[i] = wsrc[t + i * kNT];
      }
      if (more) issue(kc + 1);
      if (kc >= 0) {
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
          bf16x8 a[TM], b[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i)
            a[i] = *reinterpret_cast<const bf16x8*>(Acur + (wm * WM + i * 32 + l32) * kASTR + ks * 16 + lh * 8);
#pragma unroll
          for (int j = 0; j < TN; ++j)
            b[j] = *reinterpret_cast<const bf16x8*>(Bs + ((ks * 2 + lh) * BN + wn * WN + j * 32 + l32) * 8);
          // operands swapped: the accumulator tile is (column, row), so a lane owns one
          // output row and four consecutive columns per register quad
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        }
      }
      if (more) finish_a(kc + 1, Anext);
      __syncthreads();                 // everyone is done with Bs and Acur
      if (more) {
#pragma unroll
        for (int i = 0; i < kBItems; ++i) reinterpret_cast<v4u*>(Bs)[t + i * kNT] = bx[i];
        __syncthreads();
      }
    }

    // ---- epilogue: bias, ReLU, bf16, stage in LDS, coalesced stores -------------------
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c0 = wn * WN + j * 32 + 8 * q + 4 * lh;
        const float4 bq = *reinterpret_cast<const float4*>(bias + c0);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int r = wm * WM + i * 32 + l32;
          uint2 p;
          p.x = pack2(fmaxf(acc[i][j][4 * q + 0] + bq.x, 0.f), fmaxf(acc[i][j][4 * q + 1] + bq.y, 0.f));
          p.y = pack2(fmaxf(acc[i][j][4 * q + 2] + bq.z, 0.f), fmaxf(acc[i][j][4 * q + 3] + bq.w, 0.f));
          *reinterpret_cast<uint2*>(Os + r * L::OSTR + c0) = p;
        }
      }
    }
    __syncthreads();
    constexpr int OC = BN / 8;   // 16-byte chunks per output row
    for (int idx = t; idx < kBM * OC; idx += kNT) {
      const int r = idx / OC, c = idx - r * OC;
      if (m0 + r < ntot)
        *reinterpret_cast<v4u*>(out + (size_t)(m0 + r) * H + c * 8) = *reinterpret_cast<const v4u*>(Os + r * L::OSTR + c * 8);
    }
    __syncthreads();
  }
}

template <int BN, int WM, int WN>
hipError_t launch(const u16* h, int d, const GnnArgs& a, const u16* Wp, const float* bias, u16* out, hipStream_t s) {
  using L = Lds<BN>;
  static bool attr_done = false;
  auto kern = fused_layer_kernel<BN, WM, WN>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       L::TOTAL);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(((a.n_cu * 2 + 7) / 8) * 8), dim3(kNT), L::TOTAL, s, h, d, a.in_rowptr, a.in_col, a.out_rowptr,
                     a.out_col, Wp, bias, out, a.node_off, a.n_cand, a.status);
  return hipGetLastError();
}

}  // namespace

bool fused_layer_supported(int d, int H, int bf16) { return bf16 && (H == 256 || H == 128) && d % kBK == 0; }

hipError_t launch_fused_layer(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                              hipStream_t s) {
  const u16* hh = static_cast<const u16*>(h);
  const u16* Wp = static_cast<const u16*>(Wl);
  u16* o = static_cast<u16*>(out);
  if (a.H == 256) return launch<256, 64, 128>(hh, d, a, Wp, bias, o, s);
  return launch<128, 64, 64>(hh, d, a, Wp, bias, o, s);
}

}  // namespace dc

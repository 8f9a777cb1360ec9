// The plain product out = h W (or ReLU(h W + b)) for output width H = 256 and input width d = 256 or
// 64, bf16 (gfx950): z = W e' of the attention variant, the hidden layers of the regression network over
// many fused ops.  Four waves each own a 64 x 128 block of a 128 x 256 output tile and read their
// fragments from LDS rings that are filled from global memory by direct copies (no registers), with one
// barrier per K chunk of 64 columns (mfma_step).  The message-passing layer for these shapes is the
// sixteen-wave kernel of gnn_layer256w.hip; this file also holds the launchers of both.
#include <type_traits>

#include "common.h"

namespace dc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kBM = 128, kBN = 256, kBK = 64;
constexpr int kNT = 512;
// Shape constants for input width D = 64 * DCH: K = D in DCH chunks of 64 columns, every one the
// row's own columns (DENSE; the flag is kept so that the step below reads like the layer's).
template <int DCH, bool DENSE = true>
struct Shape {
  static_assert(DCH == 4 || DCH == 1, "input widths 256 and 64");
  static_assert(DENSE, "the message-passing layer is the sixteen-wave kernel");
  static constexpr int D = 64 * DCH;
  static constexpr int NK = DCH;
  static constexpr unsigned ROWB = D * 2;     // bytes per row of h
};
// LDS: a ring of three A chunks (128 rows x 64 columns, no padding: the 16-byte pieces of a row
// are XOR-swizzled so that fragment reads stay conflict free and a row-contiguous DMA piece of
// 1 KB is eight whole rows), a ring of three B chunks, and one 32 x 64 staging area per MFMA wave.
constexpr int kARow = kBK * 2;              // 128 bytes per A row
constexpr int kABytes = kBM * kARow;        // 16384
constexpr int kBBytes = (kBK / 8) * kBN * 8 * 2;   // 32768
constexpr int kBOff = 3 * kABytes;
constexpr int kStageBytes = 32 * kARow;     // 4096 per MFMA wave: 32 rows x 64 columns per pass, same swizzle
constexpr int kStageOff = kBOff + 3 * kBBytes;
constexpr int kLdsTotal = kStageOff + 4 * kStageBytes;
static_assert(kLdsTotal <= 160 * 1024, "one workgroup per CU owns the whole LDS");
// byte offset of 16-byte piece c (0..7) of row r in a swizzled 128-byte-row area
__device__ __forceinline__ int swz(int r, int c) { return r * kARow + ((c ^ ((r >> 1) & 7)) << 4); }
typedef __attribute__((address_space(3))) char lds_char;

__device__ __forceinline__ unsigned pack2(float a, float b) { return pack_bf16x2(a, b); }

extern __shared__ __attribute__((aligned(16))) char dc_l256_smem[];

// 16 bytes per lane from global memory straight into LDS (no registers): lane l of the wave
// writes lds_base + 16*l.  Not tracked by the compiler: waited for by hand (wait_vm_times4).  Loads
// return in issue order, so "at most N newer loads outstanding" is what s_waitcnt vmcnt(N) waits for.
__device__ __forceinline__ void load16_to_lds(const void* gaddr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gaddr), "s"(lds_base) : "memory");
}
// s_waitcnt vmcnt(4 * n4), n4 in 0..5 (wave-uniform), as one statement: separate wait sites in
// an if/else around the tile epilogue made the register allocator spill.
__device__ __forceinline__ void wait_vm_times4(int n4) {
  asm volatile(
      "s_cmp_eq_u32 %0, 5\n\t"
      "s_cbranch_scc1 .Ldc_w20_%=\n\t"
      "s_cmp_eq_u32 %0, 4\n\t"
      "s_cbranch_scc1 .Ldc_w16_%=\n\t"
      "s_cmp_eq_u32 %0, 3\n\t"
      "s_cbranch_scc1 .Ldc_w12_%=\n\t"
      "s_cmp_eq_u32 %0, 2\n\t"
      "s_cbranch_scc1 .Ldc_w8_%=\n\t"
      "s_cmp_eq_u32 %0, 1\n\t"
      "s_cbranch_scc1 .Ldc_w4_%=\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_branch .Ldc_wend_%=\n"
      ".Ldc_w4_%=:\n\t"
      "s_waitcnt vmcnt(4)\n\t"
      "s_branch .Ldc_wend_%=\n"
      ".Ldc_w8_%=:\n\t"
      "s_waitcnt vmcnt(8)\n\t"
      "s_branch .Ldc_wend_%=\n"
      ".Ldc_w12_%=:\n\t"
      "s_waitcnt vmcnt(12)\n\t"
      "s_branch .Ldc_wend_%=\n"
      ".Ldc_w16_%=:\n\t"
      "s_waitcnt vmcnt(16)\n\t"
      "s_branch .Ldc_wend_%=\n"
      ".Ldc_w20_%=:\n\t"
      "s_waitcnt vmcnt(20)\n"
      ".Ldc_wend_%=:"
      :
      : "s"(n4)
      : "scc", "memory");
}
// One step of an MFMA wave: request the B chunk of job s+2 and, if that job is one of the
// node's own chunks, its A chunk as well (both straight into their LDS ring slots), run the
// MFMAs of job s, make sure everything requested one step ago has landed and, at the end of
// a tile, write the tile out.
struct MfmaConst {
  const u16* Wp;
  const char* h;
  const float* bias;
  u16* out;
  char* smem;
  char* stage;
  unsigned lds0;        // LDS byte address of smem
  int ntot, tile0, per, wm, wn, l32, lh, lane, wave, sw;
};

template <int DCH, bool DENSE>
__device__ __forceinline__ void mfma_step(int s, int S, f32x16 (&acc)[2][4], const MfmaConst c) {
  constexpr int NK = Shape<DCH, DENSE>::NK;
  int n_req = 0;                            // requests of this step, in fours
  if (s + 2 >= 0) {
    const int J = s + 2;
    const int ti = J / NK, kc = J - ti * NK;
    if (J < S && kc < DCH) {
      // the node's own rows need no arithmetic: 128 rows x 128 bytes = sixteen 1 KB pieces of
      // eight rows, four per wave; lane l fills position l&7 of row l>>3 of its piece, which
      // under the swizzle holds column piece (l&7) ^ ((row>>1)&7).  Rows past the end are
      // clamped to the last row (read, never stored).
      n_req += 1;
      const int m0 = (c.tile0 + ti * c.per) * kBM;
      const unsigned aring = c.lds0 + (unsigned)(J % 3) * kABytes;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int piece = c.wave * 4 + i;
        const int r = piece * 8 + (c.lane >> 3);
        const int col = (c.lane & 7) ^ ((r >> 1) & 7);
        const int row = min(m0 + r, c.ntot - 1);
        load16_to_lds(c.h + (size_t)row * Shape<DCH>::ROWB + kc * kARow + col * 16, aring + piece * 1024);
      }
    }
    // W is [k/8][H][8]: the B tile of a chunk is one contiguous 32 KB run; each wave moves
    // eight 1 KB pieces of it (chunk index clamped at the end: the count of loads is fixed).
    // With at most three chunks in all chunk k always lands in ring slot k: the ring then
    // holds the whole of W and only the first tile loads it.
    if (NK > 3 || J < NK) {
      n_req += 2;
      const int jn = min(J, S - 1);
      const char* wsrc = reinterpret_cast<const char*>(c.Wp) + (size_t)(jn % NK) * kBBytes;
      const unsigned ring = c.lds0 + kBOff + (unsigned)(NK > 3 ? J % 3 : kc) * kBBytes;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int piece = c.wave * 8 + i;   // c.wave is wave-uniform by construction (readfirstlane)
        load16_to_lds(wsrc + piece * 1024 + c.lane * 16, ring + piece * 1024);
      }
    }
  }
  if (s >= 0) {
    const char* As = c.smem + (s % 3) * kABytes;
    const u16* Bs = reinterpret_cast<const u16*>(c.smem + kBOff + (NK > 3 ? s % 3 : s % NK) * kBBytes);
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8 a[2], b[4];
#pragma unroll
      for (int i = 0; i < 2; ++i)          // rows wm*64 + i*32 + l32 all share the swizzle of row l32
        a[i] = *reinterpret_cast<const bf16x8*>(As + (c.wm * 64 + i * 32 + c.l32) * kARow +
                                                (((ks * 2 + c.lh) ^ c.sw) << 4));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(Bs + ((ks * 2 + c.lh) * kBN + c.wn * 128 + j * 32 + c.l32) * 8);
      // operands swapped: accumulator tile is (column, row); a lane owns one output row
      // and four consecutive columns per register quad
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
  }
  // All but this step's requests (eight W pieces and/or, for one of the node's own chunks, four
  // A pieces): everything requested one step ago, which job s+1 needs, is in LDS.  Loads
  // complete in issue order, so this holds whatever stores of an earlier tile are still
  // on their way; placed before the tile's stores so that it never waits for those.
  wait_vm_times4(__builtin_amdgcn_readfirstlane(n_req));
  const bool tile_end = s >= 0 && (s % NK) == NK - 1;
  if (tile_end) {
    // ---- tile finished.  First bias and ReLU in place, one group of 32 columns at a time,
    // with the next group's bias in flight; no load follows a store, so nothing here waits
    // for a store to be acknowledged.
    const int ti = s / NK;
    const int m0 = (c.tile0 + ti * c.per) * kBM;
    if (!DENSE || c.bias != nullptr) {     // the plain product takes a bias (then also the ReLU) or none
    float4 bq[4];
    {
      int cb = c.wn * 128 + 4 * c.lh;
      asm volatile("" : "+v"(cb));         // opaque: keeps the bias loads out of the step loop's live set
#pragma unroll
      for (int q = 0; q < 4; ++q) bq[q] = *reinterpret_cast<const float4*>(c.bias + cb + 8 * q);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float4 cur[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) cur[q] = bq[q];
      if (j < 3) {
        int cb = c.wn * 128 + (j + 1) * 32 + 4 * c.lh;
        asm volatile("" : "+v"(cb));
#pragma unroll
        for (int q = 0; q < 4; ++q) bq[q] = *reinterpret_cast<const float4*>(c.bias + cb + 8 * q);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          acc[i][j][4 * q + 0] = fmaxf(acc[i][j][4 * q + 0] + cur[q].x, 0.f);
          acc[i][j][4 * q + 1] = fmaxf(acc[i][j][4 * q + 1] + cur[q].y, 0.f);
          acc[i][j][4 * q + 2] = fmaxf(acc[i][j][4 * q + 2] + cur[q].z, 0.f);
          acc[i][j][4 * q + 3] = fmaxf(acc[i][j][4 * q + 3] + cur[q].w, 0.f);
        }
    }
    // keep the whole of that phase ahead of the first store (the optimiser would otherwise
    // sink the second half of it below the first pass's stores, and its waits with it)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(acc[i][j]));
    }
    // ---- then bf16, wave-local staging, 16-byte row-contiguous stores
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int jh = 0; jh < 2; ++jh) {      // 32 rows x 64 columns per pass through the staging area
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const int j = 2 * jh + jj;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            v2u p;
            p.x = pack2(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]);
            p.y = pack2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            // 16-byte piece jj*4 + q of staging row l32, half lh of the piece
            *reinterpret_cast<v2u*>(c.stage + c.l32 * kARow + (((jj * 4 + q) ^ c.sw) << 4) + 8 * c.lh) = p;
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][4 * q + v] = 0.f;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int idx = c.lane + 64 * k;
          const int r = idx >> 3, cc = idx & 7;
          const int gr = m0 + c.wm * 64 + i * 32 + r;
          const v4u val = *reinterpret_cast<const v4u*>(c.stage + swz(r, cc));
          if (gr < c.ntot) *reinterpret_cast<v4u*>(c.out + (size_t)gr * kBN + c.wn * 128 + jh * 64 + cc * 8) = val;
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
  }
}

// The plain product out = h W (bias == nullptr) or ReLU(h W + bias): K = d, every chunk comes from global
// memory by direct copy.  Waves 0-3 run the multiplying steps; waves 4-7 have nothing to move and only
// keep step with the barriers (the workgroup keeps the shape of the layer kernel, whose LDS plan it shares).
template <int DCH>
__global__ __launch_bounds__(kNT) void layer256_dense_kernel(
    const u16* __restrict__ h, const u16* __restrict__ Wp, const float* __restrict__ bias, u16* __restrict__ out,
    const int* __restrict__ node_off, int C, const int* __restrict__ status) {
  constexpr int NK = Shape<DCH, true>::NK;
  if (status[0] != 0) return;
  char* smem = dc_l256_smem;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  // XCD-contiguous tile ranges (workgroups are dealt round-robin over the 8 XCDs)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per = gridDim.x >> 3;
  const int tpx = (ntiles + 7) >> 3;
  const int lim = min(tpx, ntiles - xcd * tpx);
  const int nt_wg = lim > slot ? (lim - slot + per - 1) / per : 0;
  const int S = nt_wg * NK;                 // steps of this workgroup
  if (S == 0) return;                       // no tile for this workgroup (uniform)
  // All waves pass S + 3 barriers (steps -3 .. S-1).
  const int role_wave = wave & 3;
  if (wave < 4) {
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    MfmaConst mc;
    mc.Wp = Wp;
    mc.bias = bias;
    mc.out = out;
    mc.smem = smem;
    mc.h = reinterpret_cast<const char*>(h);
    mc.stage = smem + kStageOff + role_wave * kStageBytes;
    mc.lds0 = (unsigned)(size_t)((lds_char*)dc_l256_smem);
    mc.ntot = ntot;
    mc.tile0 = xcd * tpx + slot;
    mc.per = per;
    mc.wm = role_wave >> 1;
    mc.wn = role_wave & 1;
    mc.l32 = lane & 31;
    mc.lh = lane >> 5;
    mc.lane = lane;
    mc.sw = ((lane & 31) >> 1) & 7;
    mc.wave = __builtin_amdgcn_readfirstlane(role_wave);   // scalar: the LDS base of a direct copy must be uniform
    __syncthreads();                          // step -3
    for (int s = -2; s < S; ++s) {
      mfma_step<DCH, true>(s, S, acc, mc);
      __syncthreads();
    }
  } else {
    for (int s = -3; s < S; ++s) __syncthreads();
  }
}

}  // namespace

bool layer256_supported(int d, int H, int bf16) { return bf16 && H == kBN && (d == 256 || d == 64); }

// the sixteen-wave layer kernel takes its descriptors sorted per tile
hipError_t launch_build_desc(const GnnArgs& a, hipStream_t s) { return launch_build_desc_sorted(a, s); }

namespace {

template <int DCH>
hipError_t launch_dense_shape(const void* h, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                              hipStream_t s) {
  static bool attr_done = false;
  auto kern = layer256_dense_kernel<DCH>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int grid = ((a.n_cu + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), kLdsTotal, s, static_cast<const u16*>(h),
                     static_cast<const u16*>(Wl), bias, static_cast<u16*>(out), a.node_off, a.n_cand, a.status);
  return hipGetLastError();
}

}  // namespace

// out = h W (bias == nullptr) or ReLU(h W + bias) for H = 256, d = 256 or 64, bf16
hipError_t launch_dense256(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                           hipStream_t s) {
  if (d == 256) return launch_dense_shape<4>(h, a, Wl, bias, out, s);
  if (d == 64) return launch_dense_shape<1>(h, a, Wl, bias, out, s);
  return hipErrorInvalidValue;
}

// One layer for H = 256, d = 256 or 64, bf16, after launch_build_desc: the pre-pass over the listed long rows,
// then the sixteen-wave kernel.
hipError_t launch_layer256(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                           bool readout, Profiler* prof, hipStream_t s) {
  if (d != 256 && d != 64) return hipErrorInvalidValue;
  if (prof) prof->begin(kFamHeavy, s);
  hipError_t e = launch_heavy_means(h, d, a, s);
  if (prof) prof->end(s);
  if (e != hipSuccess) return e;
  if (prof) prof->begin(d == 256 ? kFamLayer256 : kFamLayer64, s);
  e = launch_layer256w(h, d, a, Wl, bias, out, readout, s);
  if (prof) prof->end(s);
  return e;
}

}  // namespace dc

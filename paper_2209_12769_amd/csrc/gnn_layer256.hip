// Eight-wave kernels for output width H = 256 and input width d = 256 or 64, bf16 (gfx950), built
// around one multiplying step (mfma_step): four waves that each own a 64 x 128 block of a 128 x 256
// output tile and read their fragments from LDS rings that are filled from global memory by direct
// copies (no registers), with one barrier per K chunk of 64 columns.
//   layer256_dense_kernel: the plain product out = h W (or ReLU(h W + b)), K = d: z = W e' of the
//     attention variant, the hidden layers of the regression network over many fused ops.
//   layer256_dma1_kernel: the layer h' = ReLU([h | mean_pred(h) | mean_succ(h)] W + b) (neighbourhood
//     encoding of Sec. 3.3.1 with uniform coefficients) for batches whose rows have at most one
//     neighbour per direction in-kernel (fused-op subgraphs): the mean of such a row is a row that
//     already lies in memory, so four further waves copy it into the A ring as well.
// The layer with three gather slots (candidate modules) is the sixteen-wave kernel of its own file.
// Also here: the descriptor builder and the pre-pass (means of rows with longer lists) of the one-slot
// layer.
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
constexpr int kU = 3;                       // neighbours gathered in-kernel per row and direction, at most
// The kernels are built for U = 3 slots (candidate modules: 2.4 neighbours per row and
// direction on average) and for U = 1 (batches of small sparse graphs such as fused-op
// subgraphs, where almost every list has at most one entry): a slot costs a vector-memory
// instruction per eight rows whether it is used or not.
// Shape constants for input width D = 64 * DCH: K = 3 D in chunks of 64 columns, the first
// DCH of them the node's own row.  A lane needs eight gather descriptors per tile (two
// directions x four items).  With DCH = 4 each serves four jobs: one is requested per step
// (RQ = 1) and filed, two steps later, into a per-tile table, in time for its first use.
// With DCH = 1 a direction is a single job: that job's four descriptors are requested
// together (RQ = 4) and used directly when its rows are requested (DIRECT).
// DENSE: the plain product h W (K = D, every chunk the node's own row, no bias, no ReLU),
// used for z = W e' of the attention variant; the data-moving waves then only keep step.
template <int DCH, bool DENSE = false>
struct Shape {
  static_assert(DCH == 4 || DCH == 1, "input widths 256 and 64");
  static constexpr int D = 64 * DCH;
  static constexpr int NK = DENSE ? DCH : 3 * DCH;
  static constexpr bool DIRECT = DCH == 1;
  static constexpr int RQ = DIRECT ? 4 : 1;
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

// PF: the LDS fragments of the next 16 columns are requested ahead of the products.  NODMA: the
// data-moving waves issue (and wait for) all DMA requests; this wave only multiplies and stores.
template <int DCH, bool DENSE, bool PF = false, bool NODMA = false>
__device__ __forceinline__ void mfma_step(int s, int S, f32x16 (&acc)[2][4], const MfmaConst c) {
  constexpr int NK = Shape<DCH, DENSE>::NK;
  int n_req = 0;                            // requests of this step, in fours
  if (!NODMA && s + 2 >= 0) {
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
    if constexpr (PF) {
      // The whole chunk is in LDS when the step starts: the fragments of the next 16 columns are
      // requested before this 16's products are issued, so that the one MFMA wave of a SIMD does
      // not wait out an LDS round trip per 16 columns.
      bf16x8 a[2][2], b[2][4];
#define DC_FRAGS(ks_, buf_)                                                                                  \
      {                                                                                                      \
        _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                        \
          a[buf_][i] = *reinterpret_cast<const bf16x8*>(As + (c.wm * 64 + i * 32 + c.l32) * kARow +          \
                                                        ((((ks_) * 2 + c.lh) ^ c.sw) << 4));                 \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                        \
          b[buf_][j] = *reinterpret_cast<const bf16x8*>(Bs + (((ks_) * 2 + c.lh) * kBN + c.wn * 128 + j * 32 + c.l32) * 8); \
      }
      DC_FRAGS(0, 0)
#pragma unroll
      for (int ks = 0; ks < kBK / 16; ++ks) {
        if (ks + 1 < kBK / 16) DC_FRAGS(ks + 1, (ks + 1) & 1)
        __builtin_amdgcn_sched_barrier(0);     // keep these requests ahead of the products below
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks & 1][j], a[ks & 1][i], acc[i][j], 0, 0, 0);
      }
#undef DC_FRAGS
    } else {
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
  }
  // All but this step's requests (eight W pieces and/or, for one of the node's own chunks, four
  // A pieces): everything requested one step ago, which job s+1 needs, is in LDS.  Loads
  // complete in issue order, so this holds whatever stores of an earlier tile are still
  // on their way; placed before the tile's stores so that it never waits for those.
  if constexpr (!NODMA) wait_vm_times4(__builtin_amdgcn_readfirstlane(n_req));
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

// The same layer for batches whose rows have at most one neighbour per direction in-kernel
// (one gather slot; longer lists bring their finished mean from the pre-pass): the mean of such a row
// is a row that already exists in memory -- the neighbour's, the pre-pass's, or a row of zeros for an
// empty list -- so the data-moving waves copy it from global memory straight into the A ring by
// DMA, exactly as the MFMA waves do with the node's own rows, and do no arithmetic at all.  Per
// tile a lane turns the descriptors of its four rows into eight source addresses (requested one
// tile ahead with ordinary loads); a gather step is then four DMA instructions.  The MFMA waves run
// the very same steps as in layer256_kernel.
template <int DCH>
__global__ __launch_bounds__(kNT) void layer256_dma1_kernel(
    const u16* __restrict__ h, const u16* __restrict__ hin_heavy, const u16* __restrict__ hout_heavy,
    const v4i* __restrict__ desc_in, const v4i* __restrict__ desc_out, const u16* __restrict__ zero_row,
    const u16* __restrict__ Wp, const float* __restrict__ bias, u16* __restrict__ out,
    const int* __restrict__ node_off, int C, const int* __restrict__ status) {
  constexpr int NK = Shape<DCH, false>::NK;
  if (status[0] != 0) return;
  char* smem = dc_l256_smem;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per = gridDim.x >> 3;   // as in layer256_kernel
  const int tpx = (ntiles + 7) >> 3;
  const int lim = min(tpx, ntiles - xcd * tpx);
  const int nt_wg = lim > slot ? (lim - slot + per - 1) / per : 0;
  const int S = nt_wg * NK;
  if (S == 0) return;
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
    mc.wave = __builtin_amdgcn_readfirstlane(role_wave);
    __syncthreads();                          // step -3
    for (int s = -2; s < S; ++s) {
      mfma_step<DCH, false, true, true>(s, S, acc, mc);
      __syncthreads();
    }
  } else {
    constexpr unsigned kRowB = Shape<DCH>::ROWB;
    const int mwave = __builtin_amdgcn_readfirstlane(role_wave);
    const unsigned lds0 = (unsigned)(size_t)((lds_char*)dc_l256_smem);
    const char* hb = reinterpret_cast<const char*>(h);
    const char* pb_in = reinterpret_cast<const char*>(hin_heavy);
    const char* pb_out = reinterpret_cast<const char*>(hout_heavy);
    const char* zr = reinterpret_cast<const char*>(zero_row);
    const int tile0 = xcd * tpx + slot;
    // piece mwave*4 + i of a chunk is rows 8*piece .. 8*piece+7; lane l fills position l&7 of row l>>3
    // of the piece, which under the swizzle holds column piece (l&7) ^ ((row>>1)&7)
    const int r0l = mwave * 32 + (lane >> 3);                 // row of item 0 within the tile; item i: + 8 i
    v4i nd0, nd1, nd2, nd3, ne0, ne1, ne2, ne3;               // next tile's descriptors: predecessors, successors
    const char *si0, *si1, *si2, *si3, *so0, *so1, *so2, *so3;   // this tile's source addresses
#define DC_REQUEST(ti_)                                                                      \
    {                                                                                        \
      const int mq_ = (tile0 + (ti_) * per) * kBM + r0l;                                     \
      nd0 = desc_in[min(mq_, ntot - 1)];       ne0 = desc_out[min(mq_, ntot - 1)];           \
      nd1 = desc_in[min(mq_ + 8, ntot - 1)];   ne1 = desc_out[min(mq_ + 8, ntot - 1)];       \
      nd2 = desc_in[min(mq_ + 16, ntot - 1)];  ne2 = desc_out[min(mq_ + 16, ntot - 1)];      \
      nd3 = desc_in[min(mq_ + 24, ntot - 1)];  ne3 = desc_out[min(mq_ + 24, ntot - 1)];      \
    }
    // code 0: empty list (zeros); 1: the neighbour's row of h; above 3: the row's own place in the pre-pass buffer
#define DC_SOURCE(dd_, pb_, i_)                                                              \
    (((dd_).w == 0 ? zr : (((dd_).w > 3 ? (pb_) : hb) + (size_t)(unsigned)(dd_).x * kRowB)) + \
     ((((lane & 7) ^ (((r0l + 8 * (i_)) >> 1) & 7))) << 4))
#define DC_ADOPT()                                                                           \
    {                                                                                        \
      si0 = DC_SOURCE(nd0, pb_in, 0);  so0 = DC_SOURCE(ne0, pb_out, 0);                      \
      si1 = DC_SOURCE(nd1, pb_in, 1);  so1 = DC_SOURCE(ne1, pb_out, 1);                      \
      si2 = DC_SOURCE(nd2, pb_in, 2);  so2 = DC_SOURCE(ne2, pb_out, 2);                      \
      si3 = DC_SOURCE(nd3, pb_in, 3);  so3 = DC_SOURCE(ne3, pb_out, 3);                      \
    }
    DC_REQUEST(0)
    DC_ADOPT()
    DC_REQUEST(min(1, nt_wg - 1))
    for (int s = -3; s < S; ++s) {
      const int J = s + 2;
      int n4 = 0;                              // vector-memory instructions of this step, in fours
      if (J >= 0 && J < S) {
        const int ti = J / NK, kc = J - ti * NK;
        if (kc == 0 && ti > 0) {
          DC_ADOPT()
          DC_REQUEST(min(ti + 1, nt_wg - 1))
          n4 += 2;
        }
        // W is [k/8][H][8]: the B tile of a chunk is one contiguous 32 KB run, eight 1 KB pieces per
        // wave.  With at most three chunks in all, chunk k always lands in ring slot k: the ring then
        // holds the whole of W and only the first tile loads it.
        if (NK > 3 || J < NK) {
          const char* wsrc = reinterpret_cast<const char*>(Wp) + (size_t)kc * kBBytes + (size_t)mwave * 8192u + lane * 16;
          const unsigned wring = lds0 + kBOff + (unsigned)(NK > 3 ? J % 3 : kc) * kBBytes + (unsigned)mwave * 8192u;
#pragma unroll
          for (int i = 0; i < 8; ++i) load16_to_lds(wsrc + i * 1024, wring + i * 1024u);
          n4 += 2;
        }
        if (kc < DCH) {
          // the node's own rows: rows past the end are clamped to the last row (read, never stored)
          const int m0 = (tile0 + ti * per) * kBM;
          const unsigned ring = lds0 + (unsigned)(J % 3) * kABytes + (unsigned)mwave * 4096u;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int r = r0l + 8 * i;
            const int col = (lane & 7) ^ ((r >> 1) & 7);
            const int row = min(m0 + r, ntot - 1);
            load16_to_lds(hb + (size_t)row * kRowB + kc * kARow + col * 16, ring + i * 1024u);
          }
          n4 += 1;
        }
        if (kc >= DCH) {
          const bool succ = kc / DCH == 2;
          const unsigned q = (unsigned)(kc % DCH) * (unsigned)kARow;      // 64 columns = 128 bytes
          const unsigned ring = lds0 + (unsigned)(J % 3) * kABytes + (unsigned)mwave * 4096u;
          load16_to_lds((succ ? so0 : si0) + q, ring);
          load16_to_lds((succ ? so1 : si1) + q, ring + 1024u);
          load16_to_lds((succ ? so2 : si2) + q, ring + 2048u);
          load16_to_lds((succ ? so3 : si3) + q, ring + 3072u);
          n4 += 1;
        }
      }
      // everything but this step's requests has landed: the rows of job s+1, which the MFMA waves
      // read after the barrier, were requested one step ago
      wait_vm_times4(__builtin_amdgcn_readfirstlane(n4));
      __syncthreads();
    }
#undef DC_REQUEST
#undef DC_SOURCE
#undef DC_ADOPT
  }
}

// One gather descriptor per node and direction: the first `slots` neighbours (unused slots
// and rows left to the pre-pass point at the node itself, always a valid row) and a code:
// the number of slots that count, or 5 for a row left to the pre-pass.  Depends only on the
// graphs, so it is built once per forward pass.
__global__ __launch_bounds__(256) void build_desc_kernel(const int* __restrict__ in_rp, const int* __restrict__ in_ci,
                                                          const int* __restrict__ out_rp,
                                                          const int* __restrict__ out_ci, v4i* __restrict__ desc_in,
                                                          v4i* __restrict__ desc_out,
                                                          const int* __restrict__ node_off, int C, int slots,
                                                          const int* __restrict__ status) {
  if (status[0] != 0) return;
  const long long ntot = node_off[C];
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < 2 * ntot;
       idx += (long long)gridDim.x * blockDim.x) {
    const int dir = idx >= ntot;
    const int v = (int)(dir ? idx - ntot : idx);
    const int* rp = dir ? out_rp : in_rp;
    const int* ci = dir ? out_ci : in_ci;
    const int s = rp[v], dg = rp[v + 1] - s;
    // last word: the number of slots that count (0..3), plus 4 for a row left to the pre-pass (which
    // has one slot: its finished mean); such rows and empty lists point at the row itself
    v4i d = v4i{v, v, v, dg > slots ? 5 : dg};
    if (dg <= slots && dg > 0) {
      d.x = ci[s];                     // unused slots repeat the first neighbour: same cache line, never summed
      d.y = dg > 1 ? ci[s + 1] : d.x;
      d.z = dg > 2 ? ci[s + 2] : d.x;
    }
    (dir ? desc_out : desc_in)[v] = d;
  }
}

// Means of rows with more than `slots` neighbours (both directions), written at the rows'
// own positions in h_in / h_out; all other rows are left untouched.  Each thread tests
// one (row, direction) pair; the pairs that qualify are then served by the wave, 64 / LPR
// at a time, LPR = D / 8 lanes (16 bytes each) per row.  The grid must be a multiple of
// 8 workgroups.
template <int LPR>
__global__ __launch_bounds__(256) void aggregate_heavy_kernel(const u16* __restrict__ h,
                                                               const int* __restrict__ in_rp,
                                                               const int* __restrict__ in_ci,
                                                               const int* __restrict__ out_rp,
                                                               const int* __restrict__ out_ci, u16* __restrict__ h_in,
                                                               u16* __restrict__ h_out,
                                                               const int* __restrict__ node_off, int C, int slots,
                                                               const int* __restrict__ status) {
  constexpr int NSG = 64 / LPR;              // pairs served at a time
  if (status[0] != 0) return;
  const int ntot = node_off[C];
  const long long total = 2LL * ntot;
  const v4u* __restrict__ h4 = reinterpret_cast<const v4u*>(h);
  const int lane = threadIdx.x & 63, sg = lane / LPR, ll = lane % LPR, hb = sg * LPR;
  const unsigned one = bf16_one_reg();
  // Chunks of 128 rows x 2 directions.  Workgroups are dealt round-robin to the eight
  // XCDs, each with its own L2: every XCD takes one contiguous eighth of the chunks, so
  // a row that serves several long lists (they lie close together) is fetched once.
  const long long n_chunks = (total + blockDim.x - 1) / blockDim.x;
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, per_x = gridDim.x >> 3;
  const long long c_begin = n_chunks * xcd / 8, c_end = n_chunks * (xcd + 1) / 8;
  for (long long chunk = c_begin + j; chunk < c_end; chunk += per_x) {
    const long long p = chunk * blockDim.x + threadIdx.x;
    int v = 0, dir = 0, s = 0, e = 0;
    if (p < total) {
      dir = (int)(p & 1);
      v = (int)(p >> 1);
      const int* rp = dir ? out_rp : in_rp;
      s = rp[v];
      e = rp[v + 1];
    }
    unsigned long long todo = __ballot(e - s > slots);
    while (todo) {
      // lane group g takes the g-th lowest pending pair (if there is one)
      int src = -1;
#pragma unroll
      for (int g = 0; g < NSG; ++g) {
        const int b = todo ? __ffsll((long long)todo) - 1 : -1;
        todo = todo ? (todo & (todo - 1)) : 0ull;
        if (sg == g) src = b;
      }
      const int sl = src < 0 ? 0 : src;
      const int mv = __shfl(v, sl, 64), md = __shfl(dir, sl, 64), ms = __shfl(s, sl, 64), me = __shfl(e, sl, 64);
      if (src >= 0) {
        const int* ci = md ? out_ci : in_ci;
        const int deg = me - ms;
        float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // the group's lanes first fetch up to LPR neighbour ids in one coalesced load and
        // then hand them round, so that no row load waits for an index load of its own;
        // rows are added in ascending list order, four in flight
        for (int b0 = 0; b0 < deg; b0 += LPR) {
          const int nb = min(LPR, deg - b0);
          const int mine = ll < nb ? ci[ms + b0 + ll] : 0;
          int k = 0;
          if (b0 == 0) {                        // a pair here has more than slots >= 1 neighbours
            set8(a8, h4[(size_t)__shfl(mine, hb, 64) * LPR + ll]);
            k = 1;
          }
          for (; k + 3 < nb; k += 4) {
            const v4u x0 = h4[(size_t)__shfl(mine, hb + k, 64) * LPR + ll];
            const v4u x1 = h4[(size_t)__shfl(mine, hb + k + 1, 64) * LPR + ll];
            const v4u x2 = h4[(size_t)__shfl(mine, hb + k + 2, 64) * LPR + ll];
            const v4u x3 = h4[(size_t)__shfl(mine, hb + k + 3, 64) * LPR + ll];
            add8(a8, x0, one);
            add8(a8, x1, one);
            add8(a8, x2, one);
            add8(a8, x3, one);
          }
          for (; k < nb; ++k) add8(a8, h4[(size_t)__shfl(mine, hb + k, 64) * LPR + ll], one);
        }
        const float sc = 1.0f / (float)deg;
        v4u o;
        o.x = pack2(a8[0] * sc, a8[1] * sc);
        o.y = pack2(a8[2] * sc, a8[3] * sc);
        o.z = pack2(a8[4] * sc, a8[5] * sc);
        o.w = pack2(a8[6] * sc, a8[7] * sc);
        reinterpret_cast<v4u*>(md ? h_out : h_in)[(size_t)mv * LPR + ll] = o;
      }
    }
  }
}

}  // namespace

bool layer256_supported(int d, int H, int bf16) { return bf16 && H == kBN && (d == 256 || d == 64); }

static_assert(kU == 3, "a descriptor holds three neighbour ids and the degree");
static int slots_of(const GnnArgs& a) { return a.gather_slots == 1 ? 1 : kU; }

hipError_t launch_build_desc(const GnnArgs& a, hipStream_t s) {
  // the sixteen-wave layer kernel (three slots) takes its descriptors sorted per tile
  if (slots_of(a) == kU) return launch_build_desc_sorted(a, s);
  hipLaunchKernelGGL(build_desc_kernel, dim3(a.n_cu * 8), dim3(256), 0, s, a.in_rowptr, a.in_col, a.out_rowptr,
                     a.out_col, static_cast<v4i*>(a.desc[0]), static_cast<v4i*>(a.desc[1]), a.node_off, a.n_cand,
                     slots_of(a), a.status);
  return hipGetLastError();
}

namespace {

// One layer with one gather slot: the pre-pass for rows with two or more neighbours, then the kernel whose
// data-moving waves copy every mean row into LDS.
template <int DCH>
hipError_t launch_one_slot(const void* h, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                           Profiler* prof, hipStream_t s) {
  static bool attr_done = false;
  auto kern = layer256_dma1_kernel<DCH>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if (!a.zero_row) return hipErrorInvalidValue;
  const u16* hh = static_cast<const u16*>(h);
  if (prof) prof->begin(kFamHeavy, s);
  hipLaunchKernelGGL(aggregate_heavy_kernel<8 * DCH>, dim3(a.n_cu * 8), dim3(256), 0, s, hh, a.in_rowptr, a.in_col,
                     a.out_rowptr, a.out_col, static_cast<u16*>(a.agg[0]), static_cast<u16*>(a.agg[1]), a.node_off,
                     a.n_cand, 1, a.status);
  if (prof) prof->end(s);
  if (prof) prof->begin(DCH == 4 ? kFamLayer256 : kFamLayer64, s);
  const int grid = ((a.n_cu + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), kLdsTotal, s, hh, static_cast<const u16*>(a.agg[0]),
                     static_cast<const u16*>(a.agg[1]), static_cast<const v4i*>(a.desc[0]),
                     static_cast<const v4i*>(a.desc[1]), static_cast<const u16*>(a.zero_row),
                     static_cast<const u16*>(Wl), bias, static_cast<u16*>(out), a.node_off, a.n_cand, a.status);
  if (prof) prof->end(s);
  return hipGetLastError();
}

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

// One layer for H = 256, d = 256 or 64, bf16, after launch_build_desc: three gather slots (candidate modules: the
// pre-pass over the listed long rows, then the sixteen-wave kernel) or one (batches of fused-op subgraphs).
hipError_t launch_layer256(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                           Profiler* prof, hipStream_t s) {
  if (d != 256 && d != 64) return hipErrorInvalidValue;
  if (slots_of(a) == 1)
    return d == 256 ? launch_one_slot<4>(h, a, Wl, bias, out, prof, s) : launch_one_slot<1>(h, a, Wl, bias, out, prof, s);
  if (prof) prof->begin(kFamHeavy, s);
  hipError_t e = launch_heavy_means(h, d, a, s);
  if (prof) prof->end(s);
  if (e != hipSuccess) return e;
  if (prof) prof->begin(d == 256 ? kFamLayer256 : kFamLayer64, s);
  e = launch_layer256w(h, d, a, Wl, bias, out, s);
  if (prof) prof->end(s);
  return e;
}

}  // namespace dc

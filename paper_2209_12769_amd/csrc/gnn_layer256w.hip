// Sixteen-wave form of the fused layer for output width H = 256 and input width d = 256 or 64,
// bf16 (gfx950):
//     h'[v] = ReLU([h[v] | mean_pred(h)[v] | mean_succ(h)[v]] W + b)
// (neighbourhood encoding of Sec. 3.3.1 with uniform coefficients), both means formed on the
// fly, so that a layer reads h once and writes h' once (the last layer of a forward pass with a sum
// readout can leave the readout's sums instead of h': write_tile_readout).
//
// One workgroup of 16 waves per CU; every SIMD hosts two waves of each kind, so that one wave's
// waits are covered by its twin's work.
//   Waves 0-7 multiply: each owns a 64 x 64 block of the 128 x 256 output tile (64 accumulator
//   registers), reads its fragments from LDS, and requests the copies that need no arithmetic
//   (the chunks of W and the node's own K chunks) from global memory straight into the LDS rings,
//   two steps ahead.  They have no other loads, so their hand-placed waits count exactly these.
//   Waves 8-15 form the means: a lane owns two (row, 16-byte column) items per K chunk of 64
//   columns; it loads up to five neighbour pieces per item one step ahead, adds them in fp32 in
//   ascending neighbour order, scales by 1/deg, rounds to bf16 and writes the piece into the A
//   ring.  These are ordinary loads that the compiler tracks: no register is touched while a
//   load into it is in flight, and the waits are the compiler's.  The steps of a tile are
//   unrolled, so chunk offsets, ring slots and the direction are constants of each step.
//   The K chunks take turns (64 columns of the own row, of the predecessors' mean, of the successors'
//   mean, then the next 64): a mean-forming wave has two chunks to deliver in every three steps.
// Rows with more than five neighbours take their mean from a pre-pass (one slot: the finished
// mean), so that no lane walks a long list here.  The descriptors of a tile come sorted by the
// number of slots that count, separately per direction: a lane may form the mean of any row of the
// tile (it writes the piece to that row's place in the A chunk), so the eight rows that share a load
// instruction are chosen to need the same slots, and slots and arithmetic that none of them needs
// are skipped (a single slot is a plain copy).  All waves meet at one barrier per step that
// waits for LDS traffic only: global loads stay in flight across it.
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
constexpr int kNT = 1024;
constexpr int kMfmaWaves = 8;
constexpr int kSlots = 5;   // neighbours gathered in the layer kernel per row and direction, at most (up to 6 fit a descriptor)
// LDS: a ring of three A chunks (128 rows x 64 columns, the 16-byte pieces of a row XOR-swizzled so
// that fragment reads are conflict free and a 1 KB copy is eight whole rows), a ring of three
// B chunks (64 k x 256 columns of W), the bias vector.
constexpr int kARow = kBK * 2;                       // 128 bytes
constexpr int kABytes = kBM * kARow;                 // 16384
constexpr int kBBytes = (kBK / 8) * kBN * 8 * 2;     // 32768
constexpr int kBOff = 3 * kABytes;
constexpr int kBiasOff = kBOff + 3 * kBBytes;
constexpr int kLdsTotal = kBiasOff + kBN * 4;
static_assert(kLdsTotal <= 160 * 1024, "one workgroup per CU owns the whole LDS");

template <int DCH>
struct Shape {
  static_assert(DCH == 4 || DCH == 1, "input widths 256 and 64");
  static constexpr int D = 64 * DCH;
  static constexpr int NK = 3 * DCH;                 // K chunks per tile: own, predecessors' mean, successors' mean, taking turns
  static constexpr unsigned ROWB = D * 2;            // bytes per row of h
};

// byte offset of 16-byte piece c (0..7) of row r in a swizzled 128-byte-row area
__device__ __forceinline__ int swz(int r, int c) { return r * kARow + ((c ^ ((r >> 1) & 7)) << 4); }
typedef __attribute__((address_space(3))) char lds_char;

extern __shared__ __attribute__((aligned(16))) char dc_l256w_smem[];

// Workgroup barrier that orders LDS traffic only: this wave's LDS reads have returned and its LDS
// writes have landed, global loads and copies stay in flight.  One statement with a memory
// clobber, so that the compiler moves no memory access across it, between two scheduling fences, so
// that it moves no arithmetic across it either (the arithmetic of the next step, pulled up in front
// of the barrier, would wait there for loads that were meant to stay in flight for a step).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// 16 bytes per lane from global memory straight into LDS (no registers): lane l of the wave reads
// base + off (a wave-uniform 64-bit address plus the lane's unsigned 32-bit byte offset) and
// writes lds_base + 16 l.  Not tracked by the compiler; waited for with wait_copies().
__device__ __forceinline__ void copy16_to_lds(const char* base, unsigned off, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(base), "s"(lds_base) : "memory");
}
// A pointer the compiler may not know to be wave-uniform, as a scalar.
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const char*>(((unsigned long long)hi << 32) | lo);
}
// s_waitcnt vmcnt(n), n in 0 .. 15 (wave-uniform; larger values wait as for 15): at most n newer
// vector-memory operations may still be outstanding.  Loads and stores leave the counter in issue order.
__device__ __forceinline__ void wait_copies(int n) {
  asm volatile(
      "s_cmp_lt_u32 %0, 8\n\t"
      "s_cbranch_scc1 .Ldcw_r0_7_%=\n\t"
      "s_cmp_lt_u32 %0, 12\n\t"
      "s_cbranch_scc1 .Ldcw_r8_11_%=\n\t"
      "s_cmp_lt_u32 %0, 14\n\t"
      "s_cbranch_scc1 .Ldcw_r12_13_%=\n\t"
      "s_cmp_lt_u32 %0, 15\n\t"
      "s_cbranch_scc1 .Ldcw_r14_14_%=\n\t"
      "s_waitcnt vmcnt(15)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r14_14_%=:\n\t"
      "s_waitcnt vmcnt(14)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r12_13_%=:\n\t"
      "s_cmp_lt_u32 %0, 13\n\t"
      "s_cbranch_scc1 .Ldcw_r12_12_%=\n\t"
      "s_waitcnt vmcnt(13)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r12_12_%=:\n\t"
      "s_waitcnt vmcnt(12)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r8_11_%=:\n\t"
      "s_cmp_lt_u32 %0, 10\n\t"
      "s_cbranch_scc1 .Ldcw_r8_9_%=\n\t"
      "s_cmp_lt_u32 %0, 11\n\t"
      "s_cbranch_scc1 .Ldcw_r10_10_%=\n\t"
      "s_waitcnt vmcnt(11)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r10_10_%=:\n\t"
      "s_waitcnt vmcnt(10)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r8_9_%=:\n\t"
      "s_cmp_lt_u32 %0, 9\n\t"
      "s_cbranch_scc1 .Ldcw_r8_8_%=\n\t"
      "s_waitcnt vmcnt(9)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r8_8_%=:\n\t"
      "s_waitcnt vmcnt(8)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r0_7_%=:\n\t"
      "s_cmp_lt_u32 %0, 4\n\t"
      "s_cbranch_scc1 .Ldcw_r0_3_%=\n\t"
      "s_cmp_lt_u32 %0, 6\n\t"
      "s_cbranch_scc1 .Ldcw_r4_5_%=\n\t"
      "s_cmp_lt_u32 %0, 7\n\t"
      "s_cbranch_scc1 .Ldcw_r6_6_%=\n\t"
      "s_waitcnt vmcnt(7)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r6_6_%=:\n\t"
      "s_waitcnt vmcnt(6)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r4_5_%=:\n\t"
      "s_cmp_lt_u32 %0, 5\n\t"
      "s_cbranch_scc1 .Ldcw_r4_4_%=\n\t"
      "s_waitcnt vmcnt(5)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r4_4_%=:\n\t"
      "s_waitcnt vmcnt(4)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r0_3_%=:\n\t"
      "s_cmp_lt_u32 %0, 2\n\t"
      "s_cbranch_scc1 .Ldcw_r0_1_%=\n\t"
      "s_cmp_lt_u32 %0, 3\n\t"
      "s_cbranch_scc1 .Ldcw_r2_2_%=\n\t"
      "s_waitcnt vmcnt(3)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r2_2_%=:\n\t"
      "s_waitcnt vmcnt(2)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r0_1_%=:\n\t"
      "s_cmp_lt_u32 %0, 1\n\t"
      "s_cbranch_scc1 .Ldcw_r0_0_%=\n\t"
      "s_waitcnt vmcnt(1)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_r0_0_%=:\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_branch .Ldcw_end_%=\n"
      ".Ldcw_end_%=:"
      :
      : "s"(n)
      : "scc", "memory");
}

// ------------------------------------------------------------------------------------------
// multiplying waves
// ------------------------------------------------------------------------------------------
struct MulCtx {
  const char* Wp;
  const char* h;
  const float* bias64;  // the 64 bias values of this wave's columns, in LDS
  u16* out;
  float* part;          // readout variant: chunk sums [chunk + graph][256]
  const int* chunk_first;   // readout variant: the graph that holds the first row of a chunk of 64 rows
  const int* node_off;
  int n_graphs;
  char* smem;
  unsigned lds0;        // LDS byte address of smem
  int ntot, tile0, per, wm, wn, l32, lh, lane, wave, sw;
};

// The copies for step J = g + 2 (four 1 KB pieces of the W chunk and, if that step multiplies the node's
// own columns, two pieces of eight rows each); returns how many were requested.
template <int DCH>
__device__ __forceinline__ int request_copies(int g, int S, const MulCtx& c) {
  constexpr int NK = Shape<DCH>::NK;
  int n_req = 0;
  {
    const int J = g + 2;
    if (J < S) {
      // step kc of a tile multiplies column chunk kc / 3 of the node's own row (kc % 3 = 0), of the predecessors'
      // mean (1) or of the successors' mean (2): the three kinds take turns, so that a mean-forming wave has
      // two chunks to deliver in every three steps
      const int ti = J / NK, kc = J - ti * NK;
      const int kind = kc % 3, colc = kc / 3;
      if (kind == 0) {
        // piece p of an A chunk is rows 8p .. 8p+7; lane l fills position l&7 of row l>>3 of the piece,
        // which under the swizzle holds column piece (l&7) ^ ((row>>1)&7).  Rows past the end are
        // clamped to the last row (read, never stored).
        n_req += 2;
        const int m0 = (c.tile0 + ti * c.per) * kBM;
        const unsigned aring = c.lds0 + (unsigned)(J % 3) * kABytes;
        const char* abase = uniform_ptr(c.h + (size_t)m0 * Shape<DCH>::ROWB + colc * kARow);
        const int last = c.ntot - 1 - m0;                  // >= 0: the tile has at least one row
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int piece = c.wave * 2 + i;
          const int r = piece * 8 + (c.lane >> 3);
          const int col = (c.lane & 7) ^ ((r >> 1) & 7);
          copy16_to_lds(abase, (unsigned)min(r, last) * Shape<DCH>::ROWB + (unsigned)col * 16u, aring + piece * 1024);
        }
      }
      // W is [k/8][H][8]: the B tile of a chunk is one contiguous 32 KB run.  With three chunks in
      // all (d = 64) chunk k always lands in ring slot k: the ring holds the whole of W and only the
      // first tile loads it.
      if (NK > 3 || J < NK) {
        n_req += 4;
        const unsigned ring = c.lds0 + kBOff + (unsigned)(J % 3) * kBBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int piece = c.wave * 4 + i;
          copy16_to_lds(uniform_ptr(c.Wp + (size_t)(kind * DCH + colc) * kBBytes + piece * 1024), (unsigned)c.lane * 16u, ring + piece * 1024);
        }
      }
    }
  }
  return n_req;
}

// The products of step g.
template <int DCH>
__device__ __forceinline__ void products(int g, f32x16 (&acc)[2][2], const MulCtx& c) {
  if (g >= 0) {
    const char* As = c.smem + (g % 3) * kABytes;
    const u16* Bs = reinterpret_cast<const u16*>(c.smem + kBOff + (g % 3) * kBBytes);
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)          // rows wm*64 + i*32 + l32 all share the swizzle of row l32
        a[i] = *reinterpret_cast<const bf16x8*>(As + (c.wm * 64 + i * 32 + c.l32) * kARow +
                                                (((ks * 2 + c.lh) ^ c.sw) << 4));
#pragma unroll
      for (int j = 0; j < 2; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(Bs + ((ks * 2 + c.lh) * kBN + c.wn * 64 + j * 32 + c.l32) * 8);
      // operands swapped: the accumulator block is (column, row); a lane owns one output row and four
      // consecutive columns per register quad
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
  }
}

// Tile ti of a multiplying wave is complete: bias, ReLU, bf16, and out; the accumulators start the next
// tile at zero.  A lane holds, of each 32 x 32 block, one row and
// the columns 8q + 4 (lane / 32) .. + 3 for q = 0..3.  Swapping registers between the two halves
// of the wave (v_permlane32_swap: lanes 32..63 of the first operand with lanes 0..31 of the second)
// leaves lanes 0..31 with columns 0..15 of their row and lanes 32..63 with columns 16..31, each as
// two 16-byte pieces.  A second swap between neighbouring groups of 16 lanes (v_permlane16_swap:
// lanes 16..31 and 48..63 of the first operand with lanes 0..15 and 32..47 of the second) gives the
// first piece of every lane to rows 0..15 of the block and the second to rows 16..31, so that one
// store writes 16 rows of 64 contiguous bytes (a store whose lanes spread over 32 rows costs the
// compute unit's memory path twice as long).  No staging through LDS, no waits between the stores.
template <int DCH>
__device__ __forceinline__ void write_tile(int ti, f32x16 (&acc)[2][2], const MulCtx& c) {
  const int m0 = (c.tile0 + ti * c.per) * kBM;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int gr = m0 + c.wm * 64 + i * 32 + (c.l32 & 15);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      unsigned p[4][2];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 bq = *reinterpret_cast<const float4*>(c.bias64 + j * 32 + 8 * q + 4 * c.lh);
        p[q][0] = pack_bf16x2(fmaxf(acc[i][j][4 * q + 0] + bq.x, 0.f), fmaxf(acc[i][j][4 * q + 1] + bq.y, 0.f));
        p[q][1] = pack_bf16x2(fmaxf(acc[i][j][4 * q + 2] + bq.z, 0.f), fmaxf(acc[i][j][4 * q + 3] + bq.w, 0.f));
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[i][j][4 * q + v] = 0.f;
      }
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const v2u sw = __builtin_amdgcn_permlane32_swap(p[q][e], p[q + 2][e], false, false);
          p[q][e] = sw.x;
          p[q + 2][e] = sw.y;
        }
#pragma unroll
      for (int q = 0; q < 4; q += 2)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const v2u sw = __builtin_amdgcn_permlane16_swap(p[q][e], p[q + 1][e], false, false);
          p[q][e] = sw.x;
          p[q + 1][e] = sw.y;
        }
      u16* dst = c.out + (size_t)gr * kBN + c.wn * 64 + j * 32 + 16 * c.lh + 8 * (c.l32 >> 4);
      if (gr < c.ntot) *reinterpret_cast<v4u*>(dst) = v4u{p[0][0], p[0][1], p[2][0], p[2][1]};
      if (gr + 16 < c.ntot) *reinterpret_cast<v4u*>(dst + 16 * kBN) = v4u{p[1][0], p[1][1], p[3][0], p[3][1]};
    }
  }
}

// The last layer of a forward pass with a sum readout need not write its rows at all: what the readout
// needs of tile ti is, per graph and column, the sum over the tile's rows of that graph.  A wave holds
// 64 rows (one chunk of 64 consecutive global row numbers) x 64 columns.  Per graph with rows in the
// chunk: the values (bias, ReLU, rounded to bf16 exactly as they would be stored) of rows outside the
// graph are replaced by +0, then the 64 places are summed in fp32 in the fixed tree the readout kernel
// documents, by exchanges between lanes, and lane l32 ends with the column it stores: 256 bytes per
// wave, graph and tile.  Returns the number of stores issued (wave-uniform).
template <int CTRL>
__device__ __forceinline__ float lanes_get(float x) {       // x of the lane the data-parallel pattern CTRL names
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
template <int DCH>
__device__ __forceinline__ int write_tile_readout(int ti, f32x16 (&acc)[2][2], const MulCtx& c) {
  const int k = 2 * (c.tile0 + ti * c.per) + c.wm;          // chunk number
  const int r0 = 64 * k;
  int n_stores = 0;
  if (r0 < c.ntot) {                                        // else: the second half of a ragged last tile (uniform)
    // the values as they would be stored, kept in the accumulators' registers
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 bq = *reinterpret_cast<const float4*>(c.bias64 + j * 32 + 8 * q + 4 * c.lh);
          const unsigned p0 = pack_bf16x2(fmaxf(acc[i][j][4 * q + 0] + bq.x, 0.f), fmaxf(acc[i][j][4 * q + 1] + bq.y, 0.f));
          const unsigned p1 = pack_bf16x2(fmaxf(acc[i][j][4 * q + 2] + bq.z, 0.f), fmaxf(acc[i][j][4 * q + 3] + bq.w, 0.f));
          acc[i][j][4 * q + 0] = __uint_as_float(p0 << 16);
          acc[i][j][4 * q + 1] = __uint_as_float(p0 & 0xFFFF0000u);
          acc[i][j][4 * q + 2] = __uint_as_float(p1 << 16);
          acc[i][j][4 * q + 3] = __uint_as_float(p1 & 0xFFFF0000u);
        }
    const int r1 = min(r0 + 64, c.ntot);
    const int row0 = r0 + c.l32, row1 = row0 + 32;
    // lane l32 stores column (l32 / 16) * 32 + 8 * ((l32 / 4) % 4) + 4 * (lane / 32) + l32 % 4 of the wave's 64
    const int col = c.wn * 64 + (c.l32 >> 4) * 32 + 8 * ((c.l32 >> 2) & 3) + 4 * c.lh + (c.l32 & 3);
    int g = __builtin_amdgcn_readfirstlane(c.chunk_first[k]);
    for (;;) {
      const int lo = __builtin_amdgcn_readfirstlane(c.node_off[g]);
      const int hi = __builtin_amdgcn_readfirstlane(c.node_off[g + 1]);
      const bool whole = lo <= r0 && hi >= r0 + 64;         // every place of the chunk is a row of this graph
      const bool in0 = row0 >= lo && row0 < hi, in1 = row1 >= lo && row1 < hi;
      // u_n = place l32 + place l32 + 32 of column n (n = 16 j + v).  Then five exchanges, each of which
      // halves what a lane holds: of the pair (n, n + half) a lane keeps the one its lane bit names, adds
      // what its partner sends of it and gives the other away.  Partners: the lane 16 further (rows of 16
      // swapped), then within a row of 16 lanes the mirrored lane, within eight the mirrored lane, lane ^ 2,
      // lane ^ 1.  In the end lane l32 holds column n = l32, summed in the tree the readout kernel documents.
      float y[16];
#pragma unroll
      for (int n = 0; n < 16; ++n) {
        float a0 = acc[0][0][n], a1 = acc[1][0][n], b0 = acc[0][1][n], b1 = acc[1][1][n];
        if (!whole) {
          a0 = in0 ? a0 : 0.f;
          a1 = in1 ? a1 : 0.f;
          b0 = in0 ? b0 : 0.f;
          b1 = in1 ? b1 : 0.f;
        }
        // lanes 0..15 of a half keep column n and get the partner's u_n, lanes 16..31 keep column n + 16
        const v2u sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(a0 + a1), __float_as_uint(b0 + b1), false, false);
        y[n] = __uint_as_float(sw.x) + __uint_as_float(sw.y);
      }
      __builtin_amdgcn_sched_barrier(0);
      const bool b3 = (c.l32 & 8) != 0, b2 = (c.l32 & 4) != 0, b1 = (c.l32 & 2) != 0, b0 = (c.l32 & 1) != 0;
      float z[8], w[4], t2[2];
#pragma unroll
      for (int n = 0; n < 8; ++n) z[n] = (b3 ? y[n + 8] : y[n]) + lanes_get<0x140>(b3 ? y[n] : y[n + 8]);   // row_mirror
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int n = 0; n < 4; ++n) w[n] = (b2 ? z[n + 4] : z[n]) + lanes_get<0x141>(b2 ? z[n] : z[n + 4]);   // row_half_mirror
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int n = 0; n < 2; ++n) t2[n] = (b1 ? w[n + 2] : w[n]) + lanes_get<0x4E>(b1 ? w[n] : w[n + 2]);   // lane ^ 2
      __builtin_amdgcn_sched_barrier(0);
      const float mine = (b0 ? t2[1] : t2[0]) + lanes_get<0xB1>(b0 ? t2[0] : t2[1]);                         // lane ^ 1
      c.part[(size_t)(k + g) * kBN + col] = mine;
      ++n_stores;
      if (hi >= r1 || g + 1 >= c.n_graphs) break;           // the next graph starts behind this chunk (uniform)
      ++g;
    }
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  return n_stores;
}

// Step g of a multiplying wave: request the copies for step g + 2 and run the products of step g --
// the two multiplying waves of a SIMD in opposite order, so that while one stands in the queue of
// the vector-memory unit with its requests the other one multiplies -- then make sure what was
// requested one step ago has landed and, at the end of a tile, write the tile out.  (Writing it out
// behind the barrier, at the next tile's first step, was measured 2 % slower.)
template <int DCH, bool RO>
__device__ __forceinline__ void mul_step(int g, int S, f32x16 (&acc)[2][2], const MulCtx& c, int& tile_stores) {
  constexpr int NK = Shape<DCH>::NK;
  const bool products_first = c.wm == 0;
  if (products_first) products<DCH>(g, acc, c);
  const int n_req = request_copies<DCH>(g, S, c);
  if (!products_first) products<DCH>(g, acc, c);
  // Everything requested one step ago (needed by step g + 1 after the barrier) is older than this
  // step's n_req copies, and older than the eight stores of a tile that ended one step ago (those
  // were issued after that step's copies: they are counted, not waited for); placed before this
  // tile's stores so that it never waits for those.  The last tile of the batch may issue fewer
  // stores; it is the last tile of its workgroup, and nothing is waited for after it.  The readout
  // variant issues one store per graph in the wave's rows: counting fewer than were issued (eight at
  // most) only waits for some of them.
  const int stores_behind = (g >= 1 && ((g - 1) % NK) == NK - 1) ? (RO ? min(tile_stores, 8) : 8) : 0;
  wait_copies(__builtin_amdgcn_readfirstlane(n_req + stores_behind));
  if (g >= 0 && (g % NK) == NK - 1) {
    if constexpr (RO) tile_stores = write_tile_readout<DCH>(g / NK, acc, c);
    else write_tile<DCH>(g / NK, acc, c);
  }
}

// ------------------------------------------------------------------------------------------
// mean-forming waves
// ------------------------------------------------------------------------------------------
struct Dsc {            // one (row, direction) of the tile at hand, decoded for this lane's column piece
  const char* p0;       // first slot: the first neighbour's piece, or the row's finished mean from the pre-pass
  unsigned o[kSlots];   // slot u >= 1: byte offset from the tile's base row of h (o[0] unused)
  int ns_row;           // bits 0-2: slots that count (slot u counts where u < ns); above: the row's place in its tile
  float sc;             // 1 / ns, 0 for an empty list
};
// A descriptor (16 bytes) as a field of bits: the code (0 .. kSlots slots that count, 7 = left to the pre-pass)
// in bits 0-2, the row's place in its tile in bits 3-9, then kSlots neighbours of 18 bits each, as distances
// from the tile's base row (tile * 128 - 65536, at least 0): a graph has fewer than 65536 nodes, so every
// neighbour of a row of the tile lies less than 2^18 rows above that base.
constexpr int kDescHeavy = 7;
__device__ __forceinline__ void desc_put(v4i& d, int f, unsigned v18) {
  const int pos = 10 + 18 * f, w = pos >> 5, sh = pos & 31;
  d[w] |= (int)(v18 << sh);
  if (sh > 14) d[w + 1] |= (int)(v18 >> (32 - sh));
}
__device__ __forceinline__ unsigned desc_get(const v4i& d, int f) {
  const int pos = 10 + 18 * f, w = pos >> 5, sh = pos & 31;
  unsigned v = (unsigned)d[w] >> sh;
  if (sh > 14) v |= (unsigned)d[w + 1] << (32 - sh);
  return v & 0x3FFFFu;
}

struct MeanCtx {
  const char* h;
  const char* hin;      // pre-pass means (rows with long lists): predecessors / successors
  const char* hout;
  const v4i* desc_in;
  const v4i* desc_out;
  char* smem;
  int ntot, tile0, per, nt_wg;
  int pos[2];           // the two sorted positions (0..127) of the tile this lane serves
  int piece;            // its 16-byte piece (0..7) of a 64-column chunk
  unsigned cb;          // = 16 * piece
};

template <int DCH>
struct MeanState {
  Dsc cur[2][2];        // [direction][item]
  v4i raw[2][2];        // the next tile's descriptors as loaded
  v4u ld[2][2][kSlots]; // neighbour pieces in flight: [consuming step & 1][item][slot]
  const char* hb;       // h at the base row of the tile `cur` belongs to (uniform)
  int base_row;
  bool more[2][2][kSlots];   // wave-uniform: some row of the item has more than u slots that count
};

template <int DCH>
__device__ __forceinline__ void request_descriptors(MeanState<DCH>& st, const MeanCtx& c, int t) {
  // descriptors are stored tile by tile in sorted order, 128 per tile also for the last one
  const int m = (c.tile0 + min(t, c.nt_wg - 1) * c.per) * kBM;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    st.raw[0][i] = c.desc_in[m + c.pos[i]];
    st.raw[1][i] = c.desc_out[m + c.pos[i]];
  }
}

// Turns the loaded descriptors of tile t into addresses, slot factors and the scale.  A graph has
// fewer than 65536 nodes, so every neighbour lies within 65536 rows of the tile: offsets from the
// tile's base row fit 32 bits whatever the size of the batch.
template <int DCH>
__device__ __forceinline__ void adopt_descriptors(MeanState<DCH>& st, const MeanCtx& c, int t) {
  constexpr unsigned ROWB = Shape<DCH>::ROWB;
  const int m = (c.tile0 + min(t, c.nt_wg - 1) * c.per) * kBM;
  st.base_row = max(m - 65536, 0);
  st.hb = c.h + (size_t)st.base_row * ROWB;
#pragma unroll
  for (int dir = 0; dir < 2; ++dir)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const v4i d = st.raw[dir][i];
      const int code = d.x & 7, row = (d.x >> 3) & (kBM - 1);
      const int ns = code > kSlots ? 1 : code;   // a row left to the pre-pass has one slot: its finished mean
      Dsc& o = st.cur[dir][i];
      o.ns_row = ns | (row << 3);
#pragma unroll
      for (int u = 1; u < kSlots; ++u) st.more[dir][i][u] = __ballot(ns > u) != 0;
      o.p0 = (code > kSlots ? (dir ? c.hout : c.hin) : c.h) + (size_t)(st.base_row + (int)desc_get(d, 0)) * ROWB + c.cb;
#pragma unroll
      for (int u = 1; u < kSlots; ++u) o.o[u] = desc_get(d, u) * ROWB + c.cb;
      o.sc = ns > 0 ? 1.0f / (float)ns : 0.f;    // the division the other kernels make
    }
}

// Step s (0 .. NK-1) of tile t for a mean-forming wave: reduce the chunk of step s + 1 (requested one step
// ago) into its A ring slot, then request the neighbour pieces of the chunk that step s + 2 multiplies
// (requests last: a wave stands in the vector-memory unit's queue with them, and has nothing left to do).  The last step of a tile first turns to the next tile's descriptors: nothing of this tile is
// requested or reduced from there on.
template <int DCH, int s>
__device__ __forceinline__ void mean_step(int t, MeanState<DCH>& st, const MeanCtx& c) {
  constexpr int NK = Shape<DCH>::NK;
  if constexpr (s == NK - 1) adopt_descriptors<DCH>(st, c, t + 1);
  if constexpr (s == (NK >= 3 ? NK - 2 : 0)) request_descriptors<DCH>(st, c, t + 1);   // one step before they are adopted: not held longer
  constexpr int rq = (s + 1) % NK;                   // the step whose chunk is reduced now
  if constexpr (rq % 3 != 0) {
    constexpr int dir = rq % 3 - 1;
    char* dst = c.smem + (rq % 3) * kABytes;                     // NK is a multiple of 3: ring slot = step % 3
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const Dsc& d = st.cur[dir][i];
      const int ns = d.ns_row & 7, row = d.ns_row >> 3;
      const v4u x0 = st.ld[rq & 1][i][0];
      v4u o;
      if (!st.more[dir][i][1]) {
        // one slot at most in all eight rows: the mean is the neighbour's piece (or the finished mean)
        // as it is, or zero for an empty list
#pragma unroll
        for (int w = 0; w < 4; ++w) o[w] = ns != 0 ? x0[w] : 0u;
      } else {
        float lo[4], hi[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // ascending neighbour order: the first neighbour unpacked exactly, the others added where their
          // slot counts (multiplied by bf16 1.0) and left out where it does not (by 0)
          lo[w] = __uint_as_float(x0[w] << 16);
          hi[w] = __uint_as_float(x0[w] & 0xFFFF0000u);
        }
#pragma unroll
        for (int u = 1; u < kSlots; ++u)
          if (st.more[dir][i][u]) {
            const v4u xu = st.ld[rq & 1][i][u];
            const unsigned ku = ns > u ? 0x3F80u : 0u;
#pragma unroll
            for (int w = 0; w < 4; ++w) bf16_pair_add(lo[w], hi[w], xu[w], ku);
          }
#pragma unroll
        for (int w = 0; w < 4; ++w) o[w] = pack_bf16x2(lo[w] * d.sc, hi[w] * d.sc);   // x * 1.0 repacks to the same bf16 value
      }
      *reinterpret_cast<v4u*>(dst + swz(row, c.piece)) = o;
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  constexpr int lq = (s + 2) % NK;                   // the step whose chunk is requested now
  if constexpr (lq % 3 != 0) {
    constexpr int dir = lq % 3 - 1;
    constexpr unsigned coff = (unsigned)(lq / 3) * kARow;        // 64 columns = 128 bytes
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const Dsc& d = st.cur[dir][i];
      st.ld[lq & 1][i][0] = *reinterpret_cast<const v4u*>(d.p0 + coff);
#pragma unroll
      for (int u = 1; u < kSlots; ++u)
        if (st.more[dir][i][u]) st.ld[lq & 1][i][u] = *reinterpret_cast<const v4u*>(st.hb + d.o[u] + coff);
    }
  }
}

template <int DCH, int s>
__device__ __forceinline__ void mean_tile(int t, MeanState<DCH>& st, const MeanCtx& c) {
  mean_step<DCH, s>(t, st, c);
  lds_barrier();
  if constexpr (s + 1 < Shape<DCH>::NK) mean_tile<DCH, s + 1>(t, st, c);
}

template <int DCH, bool RO>
__global__ __launch_bounds__(kNT) void layer256w_kernel(
    const u16* __restrict__ h, const u16* __restrict__ hin_heavy, const u16* __restrict__ hout_heavy,
    const v4i* __restrict__ desc_in, const v4i* __restrict__ desc_out, const u16* __restrict__ Wp,
    const float* __restrict__ bias, u16* __restrict__ out, float* __restrict__ part,
    const int* __restrict__ chunk_first, const int* __restrict__ node_off, int C,
    const int* __restrict__ status) {
  constexpr int NK = Shape<DCH>::NK;
  if (status[0] != 0) return;
  char* smem = dc_l256w_smem;
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  // XCD-contiguous tile ranges (workgroups are dealt round-robin over the 8 XCDs)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per = gridDim.x >> 3;
  const int tpx = (ntiles + 7) >> 3;
  const int lim = min(tpx, ntiles - xcd * tpx);
  const int nt_wg = lim > slot ? (lim - slot + per - 1) / per : 0;
  const int S = nt_wg * NK;                 // steps of this workgroup
  if (S == 0) return;                       // no tile for this workgroup (uniform)
  if (t < kBN) reinterpret_cast<float*>(smem + kBiasOff)[t] = bias[t];   // read after many barriers, at the first tile's end
  // Both kinds of wave pass S + 2 barriers (steps -2 .. S-1).  Waves are dealt to the four SIMDs
  // round-robin, so every SIMD hosts two waves of each kind.
  if (wave < kMfmaWaves) {
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    MulCtx mc;
    mc.Wp = reinterpret_cast<const char*>(Wp);
    mc.h = reinterpret_cast<const char*>(h);
    mc.wm = wave >> 2;
    mc.wn = wave & 3;
    mc.bias64 = reinterpret_cast<const float*>(smem + kBiasOff) + mc.wn * 64;
    mc.out = out;
    mc.part = part;
    mc.chunk_first = chunk_first;
    mc.node_off = node_off;
    mc.n_graphs = C;
    mc.smem = smem;
    mc.lds0 = (unsigned)(size_t)((lds_char*)dc_l256w_smem);
    mc.ntot = ntot;
    mc.tile0 = xcd * tpx + slot;
    mc.per = per;
    mc.l32 = lane & 31;
    mc.lh = lane >> 5;
    mc.lane = lane;
    mc.sw = ((lane & 31) >> 1) & 7;
    mc.wave = wave;
    int tile_stores = 0;
    for (int g = -2; g < S; ++g) {
      mul_step<DCH, RO>(g, S, acc, mc, tile_stores);
      lds_barrier();
    }
  } else {
    MeanCtx mc;
    mc.h = reinterpret_cast<const char*>(h);
    mc.hin = reinterpret_cast<const char*>(hin_heavy);
    mc.hout = reinterpret_cast<const char*>(hout_heavy);
    mc.desc_in = desc_in;
    mc.desc_out = desc_out;
    mc.smem = smem;
    mc.ntot = ntot;
    mc.tile0 = xcd * tpx + slot;
    mc.per = per;
    mc.nt_wg = nt_wg;
    // A wave serves two groups of eight sorted positions: group w (few slots) and group 15 - w (many)
    mc.pos[0] = (wave - kMfmaWaves) * 8 + (lane >> 3);
    mc.pos[1] = (15 - (wave - kMfmaWaves)) * 8 + (lane >> 3);
    mc.piece = lane & 7;
    mc.cb = (unsigned)(lane & 7) * 16u;
    MeanState<DCH> st;
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int u = 0; u < kSlots; ++u) st.ld[p][i][u] = v4u{0u, 0u, 0u, 0u};
    // steps -2 and -1: the first tile's descriptors; with d = 64 its first chunk of means is
    // requested here, as the last step of a tile does for the tile after it
    request_descriptors<DCH>(st, mc, 0);
    lds_barrier();
    mean_step<DCH, NK - 1>(-1, st, mc);
    lds_barrier();
    for (int tt = 0; tt < nt_wg; ++tt) mean_tile<DCH, 0>(tt, st, mc);
  }
}

// One gather descriptor per node and direction, stored tile by tile (128 per tile, also for the last one)
// and, within a tile, sorted by the number of slots that count: first the rows with at most one (a single
// neighbour, a finished mean from the pre-pass, or none), then two, three, ... kSlots.  The 16 bytes are
// the field of bits desc_put / desc_get describe: code, the row's place in its tile, kSlots neighbours
// (unused slots, empty lists and rows left to the pre-pass name the node itself, always a valid row).
// Places of the last tile past the end of the batch are empty lists.
// Depends only on the graphs: built once per forward pass.  One workgroup of 256 per tile: threads
// 0..127 the predecessors' lists, 128..255 the successors'.
__global__ __launch_bounds__(256) void build_desc_sorted_kernel(
    const int* __restrict__ in_rp, const int* __restrict__ in_ci, const int* __restrict__ out_rp,
    const int* __restrict__ out_ci, v4i* __restrict__ desc_in, v4i* __restrict__ desc_out,
    int* __restrict__ heavy_in, int* __restrict__ heavy_out, int* __restrict__ heavy_cnt,
    const int* __restrict__ node_off, int C, const int* __restrict__ status) {
  if (status[0] != 0) return;
  __shared__ int cnt[2][4][kSlots + 1];      // [parity][wave][class, and the rows left to the pre-pass]
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  const int t = threadIdx.x, wave = t >> 6, lane = t & 63, dir = t >> 7, r = t & 127;
  int par = 0;
  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x, par ^= 1) {
    const int v = tile * kBM + r;
    const bool valid = v < ntot;
    const int vv = valid ? v : ntot - 1;
    const int* rp = dir ? out_rp : in_rp;
    const int* ci = dir ? out_ci : in_ci;
    const int s = rp[vv], dg = valid ? rp[vv + 1] - s : 0;
    const int ns = dg > kSlots ? 1 : dg;
    const int cls = ns <= 1 ? 0 : ns - 1;
    int rank = 0;
#pragma unroll
    for (int k = 0; k < kSlots; ++k) {
      const unsigned long long m = __ballot(cls == k);
      if (cls == k) rank = __popcll(m & ((1ull << lane) - 1ull));
      if (lane == 0) cnt[par][wave][k] = __popcll(m);
    }
    // the rows left to the pre-pass, in ascending order, for the kernel that forms their means
    const unsigned long long mh = __ballot(dg > kSlots);
    const int hrank = __popcll(mh & ((1ull << lane) - 1ull));
    if (lane == 0) cnt[par][wave][kSlots] = __popcll(mh);
    __syncthreads();                           // the next tile writes the other parity: one barrier per tile
    const int w0 = dir * 2;
    int start = 0;
#pragma unroll
    for (int k = 0; k < kSlots; ++k) {
      const int c0 = cnt[par][w0][k], c1 = cnt[par][w0 + 1][k];
      if (k < cls) start += c0 + c1;
      if (k == cls && (wave & 1)) start += c0;
    }
    const int base = max(tile * kBM - 65536, 0);
    v4i d = v4i{(dg > kSlots ? kDescHeavy : dg) | (r << 3), 0, 0, 0};
    // unused slots, empty lists and rows left to the pre-pass name the row itself (always a valid row)
    const unsigned first = (unsigned)((dg <= kSlots && dg > 0 ? ci[s] : vv) - base);
    desc_put(d, 0, first);
#pragma unroll
    for (int u = 1; u < kSlots; ++u) desc_put(d, u, dg <= kSlots && dg > u ? (unsigned)(ci[s + u] - base) : first);
    (dir ? desc_out : desc_in)[(size_t)tile * kBM + start + rank] = d;
    const int h0 = cnt[par][w0][kSlots];
    if (dg > kSlots) (dir ? heavy_out : heavy_in)[(size_t)tile * kBM + ((wave & 1) ? h0 : 0) + hrank] = v;
    if (r == 0) heavy_cnt[2 * tile + dir] = h0 + cnt[par][w0 + 1][kSlots];
  }
}

// The per-tile lists of the rows left to the pre-pass, made one list: an exclusive scan of the per-(tile,
// direction) counts (one workgroup, eight entries per thread and round, the next round's entries loaded
// before this round's barrier; a few hundred thousand entries at most), ...
constexpr int kScanPer = 8;
__global__ __launch_bounds__(1024) void heavy_scan_kernel(const int* __restrict__ heavy_cnt, int* __restrict__ heavy_off,
                                                          const int* __restrict__ node_off, int C,
                                                          const int* __restrict__ status) {
  __shared__ int wsum[2][16];
  if (status[0] != 0) return;
  const int ntot = node_off[C];
  const int n = 2 * ((ntot + kBM - 1) / kBM);
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  auto load = [&](int i, int (&x)[kScanPer]) {   // i is a multiple of 8: whole 16-byte pieces where they lie below n
#pragma unroll
    for (int q = 0; q < kScanPer; q += 4) {
      if (i + q + 3 < n) {
        const v4i p = *reinterpret_cast<const v4i*>(heavy_cnt + i + q);
        x[q] = p.x; x[q + 1] = p.y; x[q + 2] = p.z; x[q + 3] = p.w;
      } else {
#pragma unroll
        for (int k = q; k < q + 4; ++k) x[k] = i + k < n ? heavy_cnt[i + k] : 0;
      }
    }
  };
  int carry = 0, par = 0;                      // the same value in every thread
  int x[kScanPer], xn[kScanPer];
  load(kScanPer * t, x);
  for (int i0 = 0; i0 < n; i0 += 1024 * kScanPer, par ^= 1) {
    const int i = i0 + kScanPer * t;
    load(i + 1024 * kScanPer, xn);
    int mine = 0;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k) mine += x[k];
    int incl = mine;                           // inclusive scan inside the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int y = __shfl_up(incl, d, 64);
      if (lane >= d) incl += y;
    }
    if (lane == 63) wsum[par][wave] = incl;
    __syncthreads();                           // the next round writes the other half of wsum: one barrier per round
    int before = carry, total = carry;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int ws = wsum[par][w];
      if (w < wave) before += ws;
      total += ws;
    }
    int run = before + incl - mine;
#pragma unroll
    for (int q = 0; q < kScanPer; q += 4) {
      int o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        o[k] = run;
        run += x[q + k];
      }
      if (i + q + 3 < n) {
        *reinterpret_cast<v4i*>(heavy_off + i + q) = v4i{o[0], o[1], o[2], o[3]};
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (i + q + k < n) heavy_off[i + q + k] = o[k];
      }
    }
    carry = total;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k) x[k] = xn[k];
  }
  if (t == 0) heavy_off[n] = carry;
}

// ... and the lists copied to their places in it: entry = row number, bit 31 set for the successors' direction;
// a tile's predecessor-side rows first, each side in ascending row order.  A workgroup of 256 takes four
// tiles at a time (thread = direction and place), so that their dependent loads overlap.
__global__ __launch_bounds__(256) void heavy_compact_kernel(const int* __restrict__ heavy_in,
                                                            const int* __restrict__ heavy_out,
                                                            const int* __restrict__ heavy_cnt,
                                                            const int* __restrict__ heavy_off,
                                                            unsigned* __restrict__ heavy_list,
                                                            const int* __restrict__ node_off, int C,
                                                            const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  const int dir = threadIdx.x >> 7, r = threadIdx.x & 127;
  const int* list = dir ? heavy_out : heavy_in;
  for (int tile0 = blockIdx.x * 4; tile0 < ntiles; tile0 += gridDim.x * 4) {
    int cnt[4], off[4], v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) cnt[k] = tile0 + k < ntiles ? heavy_cnt[2 * (tile0 + k) + dir] : 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (r < cnt[k]) {
        off[k] = heavy_off[2 * (tile0 + k) + dir];
        v[k] = list[(size_t)(tile0 + k) * kBM + r];
      }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (r < cnt[k]) heavy_list[off[k] + r] = (unsigned)v[k] | ((unsigned)dir << 31);
  }
}

__global__ __launch_bounds__(256) void clear_heavy_ctr_kernel(int* __restrict__ ctr) {
  if (threadIdx.x < kHeavyCtrInts) ctr[threadIdx.x] = 0;
}

// Means of the rows with more than kSlots neighbours (the pre-pass), from the list the two kernels above
// leave.  LPR = d / 8 lanes (16 bytes each) serve a row: they fetch sixteen neighbour ids (eight at d = 64) with
// one load, hand them round, and keep eight neighbour rows in flight; the rows are added in ascending list order
// in fp32 (first one unpacked exactly), scaled by 1/deg and rounded to bf16: the arithmetic of the layer
// kernel.
// The list is cut into eight contiguous runs of tiles, one per XCD, and a run is handed out in order, in
// batches of kHeavyGroups rows per lane group, through a counter: whatever the rows cost, the rows being
// worked on at any time are neighbours in the list, i.e. rows of one or two graphs per XCD, whose rows
// stay in that XCD's L2 while the graph's other long lists ask for them again.  (Dealing the tiles out by
// a fixed stride lets the workgroups drift apart, and every row then comes from HBM each time it is asked
// for.)  The batch after the next one is claimed while the current one is summed, and what a row needs
// before its neighbour rows can be asked for -- its number, its list's start and length, its first neighbour
// ids -- is fetched while the row before it is summed, also across batches.
constexpr int kHeavyGroups = 2;      // rows per lane group and batch
constexpr int kHeavyThreads = 256;   // four waves share a batch
constexpr int kHeavyWgs = 7;         // workgroups per CU: all that fit the kernel's registers
static_assert(kHeavyThreads % 64 == 0 && kHeavyThreads >= 64 && kHeavyThreads <= 1024, "whole waves");
template <int LPR>
__global__ __launch_bounds__(kHeavyThreads) void heavy_means_kernel(
    const u16* __restrict__ h, const int* __restrict__ in_rp, const int* __restrict__ in_ci,
    const int* __restrict__ out_rp, const int* __restrict__ out_ci, const unsigned* __restrict__ heavy_list,
    const int* __restrict__ heavy_off, u16* __restrict__ h_in, u16* __restrict__ h_out, int* __restrict__ ctr,
    const int* __restrict__ node_off, int C, const int* __restrict__ status) {
  constexpr int NSG = 64 / LPR;              // rows a wave serves at a time
  constexpr int kIds = LPR >= 16 ? 16 : 8;   // neighbour ids a lane group fetches with one load
  __shared__ int claimed[2];
  if (status[0] != 0) return;
  const int ntot = node_off[C];
  const int ntiles = (ntot + kBM - 1) / kBM;
  const v4u* __restrict__ h4 = reinterpret_cast<const v4u*>(h);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), n_waves = (int)(blockDim.x >> 6);
  const int sg = lane / LPR, ll = lane % LPR, hb = sg * LPR;
  const unsigned one = bf16_one_reg();
  const int xcd = blockIdx.x & 7;
  const int t_begin = (int)((long long)ntiles * xcd / 8), t_end = (int)((long long)ntiles * (xcd + 1) / 8);
  const int r0 = heavy_off[2 * t_begin], r1 = heavy_off[2 * t_end];
  const int per_batch = n_waves * NSG * kHeavyGroups;
  const int n_batches = (r1 - r0 + per_batch - 1) / per_batch;
  int* my_ctr = ctr + xcd * 32;
  if (threadIdx.x == 0) {
    claimed[0] = atomicAdd(my_ctr, 1);
    claimed[1] = atomicAdd(my_ctr, 1);
  }
  __syncthreads();
  int cur = __builtin_amdgcn_readfirstlane(claimed[0]), nxt = __builtin_amdgcn_readfirstlane(claimed[1]);
  __syncthreads();
  int par = 0;
  // list position of this lane group's row in group g of batch b
  auto place = [&](int b, int g) { return r0 + b * per_batch + (g * n_waves + wave) * NSG + sg; };
  int v = 0, s = 0, deg = 0, mine = 0, dir = 0;
  bool have = false;
  auto fetch = [&](int r) {
    have = r < r1;
    if (have) {
      const unsigned e = heavy_list[r];
      dir = (int)(e >> 31);
      v = (int)(e & 0x7FFFFFFFu);
      const int* rp = dir ? out_rp : in_rp;
      s = rp[v];
      deg = rp[v + 1] - s;
      mine = (dir ? out_ci : in_ci)[s + (ll < min(kIds, deg) ? ll : 0)];
    }
  };
  if (cur < n_batches) fetch(place(cur, 0));
  while (cur < n_batches) {
    int after = 0;
    if (threadIdx.x == 0) after = atomicAdd(my_ctr, 1);
    for (int g = 0; g < kHeavyGroups; ++g) {
      const bool chave = have;
      const int cv = v, cs = s, cdeg = deg, cdir = dir;
      int cmine = mine;
      // the next row of this lane group: in this batch, or the first one of the next batch
      fetch(g + 1 < kHeavyGroups ? place(cur, g + 1) : (nxt < n_batches ? place(nxt, 0) : r1));
      if (!chave) continue;
      const int* ci = cdir ? out_ci : in_ci;
      float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      // kIds neighbour ids per round, held by the first kIds lanes of the group; eight rows in flight: row
      // q + 8 is asked for as soon as row q has been added (loads return in the order they were issued, so
      // waiting for row q leaves the seven behind it in flight), and a list of up to kIds entries costs one
      // memory round trip instead of one per eight
      for (int b0 = 0; b0 < cdeg; b0 += kIds) {
        const int nb = min(kIds, cdeg - b0);
        if (b0 > 0) cmine = ci[cs + b0 + (ll < nb ? ll : 0)];
        v4u x[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int id = __shfl(cmine, hb + (q < nb ? q : 0), 64);
          if (q < nb) x[q] = h4[(size_t)id * LPR + ll];
        }
#pragma unroll
        for (int q = 0; q < kIds; ++q) {
          if (q < nb) {
            if (b0 == 0 && q == 0) {         // the first neighbour: exact unpack
#pragma unroll
              for (int w = 0; w < 4; ++w) {
                a8[2 * w] = __uint_as_float(x[0][w] << 16);
                a8[2 * w + 1] = __uint_as_float(x[0][w] & 0xFFFF0000u);
              }
            } else {
#pragma unroll
              for (int w = 0; w < 4; ++w) bf16_pair_add(a8[2 * w], a8[2 * w + 1], x[q & 7][w], one);
            }
          }
          if (q + 8 < kIds) {
            const int id = __shfl(cmine, hb + (q + 8 < nb ? q + 8 : 0), 64);
            if (q + 8 < nb) x[q & 7] = h4[(size_t)id * LPR + ll];
          }
        }
      }
      const float sc = 1.0f / (float)cdeg;
      v4u o;
#pragma unroll
      for (int w = 0; w < 4; ++w) o[w] = pack_bf16x2(a8[2 * w] * sc, a8[2 * w + 1] * sc);
      reinterpret_cast<v4u*>(cdir ? h_out : h_in)[(size_t)cv * LPR + ll] = o;
    }
    if (threadIdx.x == 0) claimed[par] = after;
    __syncthreads();
    const int got = __builtin_amdgcn_readfirstlane(claimed[par]);
    par ^= 1;
    cur = nxt;
    nxt = got;
  }
}

template <int DCH, bool RO>
hipError_t launch_w(const void* h, const GnnArgs& a, const void* Wl, const float* bias, void* out, hipStream_t s) {
  static bool attr_done = false;
  auto kern = layer256w_kernel<DCH, RO>;
  if (RO && (!a.ro_part || !a.ro_first)) return hipErrorInvalidValue;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int grid = ((a.n_cu + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), kLdsTotal, s, static_cast<const u16*>(h),
                     static_cast<const u16*>(a.agg[0]), static_cast<const u16*>(a.agg[1]),
                     static_cast<const v4i*>(a.desc[0]), static_cast<const v4i*>(a.desc[1]),
                     static_cast<const u16*>(Wl), bias, static_cast<u16*>(out), a.ro_part, a.ro_first, a.node_off,
                     a.n_cand, a.status);
  return hipGetLastError();
}

// The graph that holds the first row of every chunk of 64 rows: thread c marks the chunks that begin
// inside graph c.
__global__ __launch_bounds__(256) void chunk_first_kernel(const int* __restrict__ node_off, int C,
                                                           int* __restrict__ chunk_first,
                                                           const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  const int n0 = node_off[c], n1 = node_off[c + 1];
  for (int k = (n0 + 63) >> 6; 64 * k < n1; ++k) chunk_first[k] = c;
}

}  // namespace

hipError_t launch_chunk_first(const GnnArgs& a, hipStream_t s) {
  if (!a.ro_first) return hipErrorInvalidValue;
  hipLaunchKernelGGL(chunk_first_kernel, dim3((a.n_cand + 255) / 256), dim3(256), 0, s, a.node_off, a.n_cand, a.ro_first,
                     a.status);
  return hipGetLastError();
}

hipError_t launch_build_desc_sorted(const GnnArgs& a, hipStream_t s) {
  if (!a.heavy_off || !a.heavy_list || !a.heavy_ctr) return hipErrorInvalidValue;
  hipLaunchKernelGGL(build_desc_sorted_kernel, dim3(a.n_cu * 8), dim3(256), 0, s, a.in_rowptr, a.in_col, a.out_rowptr,
                     a.out_col, static_cast<v4i*>(a.desc[0]), static_cast<v4i*>(a.desc[1]), a.heavy[0], a.heavy[1],
                     a.heavy_cnt, a.node_off, a.n_cand, a.status);
  hipLaunchKernelGGL(heavy_scan_kernel, dim3(1), dim3(1024), 0, s, a.heavy_cnt, a.heavy_off, a.node_off, a.n_cand,
                     a.status);
  hipLaunchKernelGGL(heavy_compact_kernel, dim3(a.n_cu * 8), dim3(256), 0, s, a.heavy[0], a.heavy[1], a.heavy_cnt,
                     a.heavy_off, a.heavy_list, a.node_off, a.n_cand, a.status);
  return hipGetLastError();
}

hipError_t launch_heavy_means(const void* h, int d, const GnnArgs& a, hipStream_t s) {
  if (d != 256 && d != 64) return hipErrorInvalidValue;
  const int grid = ((a.n_cu + 7) / 8) * 8 * kHeavyWgs;
  const u16* hh = static_cast<const u16*>(h);
  hipLaunchKernelGGL(clear_heavy_ctr_kernel, dim3(1), dim3(256), 0, s, a.heavy_ctr);
  if (d == 256)
    hipLaunchKernelGGL(heavy_means_kernel<32>, dim3(grid), dim3(kHeavyThreads), 0, s, hh, a.in_rowptr, a.in_col,
                       a.out_rowptr, a.out_col, a.heavy_list, a.heavy_off, static_cast<u16*>(a.agg[0]),
                       static_cast<u16*>(a.agg[1]), a.heavy_ctr, a.node_off, a.n_cand, a.status);
  else
    hipLaunchKernelGGL(heavy_means_kernel<8>, dim3(grid), dim3(kHeavyThreads), 0, s, hh, a.in_rowptr, a.in_col,
                       a.out_rowptr, a.out_col, a.heavy_list, a.heavy_off, static_cast<u16*>(a.agg[0]),
                       static_cast<u16*>(a.agg[1]), a.heavy_ctr, a.node_off, a.n_cand, a.status);
  return hipGetLastError();
}

// The layer kernel alone (sorted descriptors built, pre-pass means in a.agg[]): d = 256 or 64, kSlots gather slots.
hipError_t launch_layer256w(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                            bool readout, hipStream_t s) {
  if (d == 256) return readout ? launch_w<4, true>(h, a, Wl, bias, out, s) : launch_w<4, false>(h, a, Wl, bias, out, s);
  if (d == 64) return readout ? launch_w<1, true>(h, a, Wl, bias, out, s) : launch_w<1, false>(h, a, Wl, bias, out, s);
  return hipErrorInvalidValue;
}

}  // namespace dc

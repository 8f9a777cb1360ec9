// Times of the nodes of a candidate module, as the simulator needs them (gfx950).
//
// The cost model of the paper is a composition (Sec. 3.1, Simulator): profiled data for
// individual ops, the GNN estimator for fused ops, a linear model on the tensor size for
// all-reduce instructions.  A fused op is the subgraph of its original ops with the
// dependencies among them (Sec. 3.3), so the estimator runs on a batch with one small graph
// per fused op.  The kernels here build that batch from what the contraction leaves behind
// (members grouped by contracted node, ascending), and afterwards turn the estimator's
// embeddings into times:
//
//   fo_count_kernel   per candidate: classifies every contracted node (bucket of tensors /
//                     single op / fused op / mixture), writes the times that need no
//                     estimator, counts fused ops, their rows and their internal edges.
//                     Candidates of one batch mostly share their fused ops (a search step mutates
//                     a few groups of a parent): a fused op whose base graph and member list equal
//                     those of one met before (a hash table over the batch, members compared in
//                     full) gets no rows of its own and takes that one's estimate afterwards
//   fo_scan_kernel    offsets of every candidate's share of the fused-op batch
//   fo_fill_kernel    writes the batch: one graph per fused op, rows = members in ascending
//                     base index with their own features, edges = base edges inside the group
//   fo_readout_kernel sum of the final embeddings over the rows of each fused op
//                     (Sec. 3.3.1, second equation), fp64 accumulation in row order
//   (two dense layers with bias and ReLU on those sums run in the layer kernels' GEMM)
//   fo_time_kernel    last layer of the regression network (Sec. 3.3.2), clamped at zero,
//                     scattered to the fused op's node of the module
//   fo_repeat_kernel  the time of every fused op that repeats an earlier one
//
// Per contracted node: all members tensors: size = sum of the members' sizes (Sec. 2.3), fp64
// in ascending member order, rounded once; one op: its profiled time; two or more ops: the
// estimate; ops and tensors mixed: +infinity (no strategy of Sec. 3.2 produces it).
// Base rows must be strictly ascending (no duplicates, no self loops): the count of edges
// inside a group is then exact without sorting.
#include <math.h>

#include "common.h"

namespace dc {
namespace {

typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kMaxProbes = 4096;   // a fused op that finds no place within so many steps simply keeps its own rows

__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Exclusive scans of a[0..n) and b[0..n) in place by a workgroup of 256 threads, in rounds of 1024 entries: a
// thread takes four neighbouring entries of each array, so a wave reads and writes whole cache lines (the
// arrays live in global memory; a contiguous run per thread would touch a line per entry).  One barrier per
// round (the wave sums alternate between two halves of ws), one at the end.  Returns the totals.
__device__ __forceinline__ void block_exscan_pair(int* a, int* b, int n, int (&ws)[2][2][4], int& total_a, int& total_b) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int carry_a = 0, carry_b = 0, par = 0;
  for (int i0 = 0; i0 < n; i0 += 1024, par ^= 1) {
    const int i = i0 + 4 * t;
    int xa[4], xb[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      xa[k] = i + k < n ? a[i + k] : 0;
      xb[k] = i + k < n ? b[i + k] : 0;
    }
    const int sa = xa[0] + xa[1] + xa[2] + xa[3], sb = xb[0] + xb[1] + xb[2] + xb[3];
    const int ia = wave_incl_scan(sa), ib = wave_incl_scan(sb);
    if (lane == 63) {
      ws[par][0][wave] = ia;
      ws[par][1][wave] = ib;
    }
    __syncthreads();
    int before_a = carry_a, before_b = carry_b;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int wa = ws[par][0][w], wb = ws[par][1][w];
      if (w < wave) {
        before_a += wa;
        before_b += wb;
      }
      carry_a += wa;
      carry_b += wb;
    }
    int ra = before_a + ia - sa, rb = before_b + ib - sb;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (i + k < n) {
        a[i + k] = ra;
        b[i + k] = rb;
      }
      ra += xa[k];
      rb += xb[k];
    }
  }
  __syncthreads();
  total_a = carry_a;
  total_b = carry_b;
}

__global__ __launch_bounds__(256) void fo_clear_table_kernel(int* __restrict__ table, unsigned mask, int* totals) {
  const size_t n = (size_t)mask + 1;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) table[i] = -1;
  if (blockIdx.x == 0 && threadIdx.x == 0) totals[5] = 0;
}

// The fused op (candidate c, group g: base graph b, members mem[s .. s + n)) against the table: returns the
// contracted node (global) of an equal fused op entered before, or -1 after entering this one (`me`).
__device__ __forceinline__ int find_or_enter(const FusedOpsArgs& a, int b, const int* mem, int s, int n, int me) {
  unsigned long long h = mix64(0x9E3779B97F4A7C15ull + (unsigned)b);
  for (int i = 0; i < n; ++i) h = mix64(h ^ (unsigned)mem[s + i]);
  unsigned slot = (unsigned)h & a.table_mask;
  for (int probe = 0; probe < kMaxProbes; ++probe) {
    // a place only ever changes from free to taken, so whatever a plain read finds taken is final, and only a
    // place that looks free needs the atomic (thousands of candidates may carry the same fused op)
    int old = a.table[slot];
    if (old == -1) old = atomicCAS(&a.table[slot], -1, me);
    if (old == -1) return -1;
    int lo = 0, hi = a.n_cand;                 // the candidate of node `old`: the last one that starts at or before it
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.c_node_off[mid] <= old) lo = mid; else hi = mid;
    }
    if (a.cand_graph[lo] == b) {
      const int coff2 = a.cand_off[lo];
      const int* ms2 = a.mstart + coff2 + lo;
      const int* mem2 = a.members + coff2;
      const int g2 = old - a.c_node_off[lo];
      const int s2 = ms2[g2];
      bool same = ms2[g2 + 1] - s2 == n;
      for (int i = 0; same && i < n; ++i) same = mem2[s2 + i] == mem[s + i];
      if (same) return old;
    }
    slot = (slot + 1) & a.table_mask;
  }
  return -1;
}

__global__ __launch_bounds__(256) void fo_count_kernel(FusedOpsArgs a) {
  __shared__ int wsum[2][2][4];
  if (a.status[0] != 0) return;
  const int c = blockIdx.x, t = threadIdx.x, T = blockDim.x;
  const int b = a.cand_graph[c];
  const int coff = a.cand_off[c], N = a.cand_off[c + 1] - coff, nslot = coff + c;
  const int G = a.Gc[c], gb = a.bg.gno[b], n0 = a.c_node_off[c];
  const int* ms = a.mstart + nslot;
  const int* mem = a.members + coff;
  const int* nid = a.new_id + coff;
  const float* tb = a.op_time_base + gb;
  const float* xb = a.ar_size_base + gb;
  int* gfm = a.gfm + nslot;
  int* gfk = a.gfk + nslot;
  int n_repeats = 0;
  for (int g = t; g < G; g += T) {
    const int s = ms[g], e = ms[g + 1], n = e - s;
    int n_ar = 0;
    double size = 0.0;
    for (int m = s; m < e; ++m) {
      const float x = xb[mem[m]];
      if (x >= 0.0f) {
        ++n_ar;
        size += (double)x;
      }
    }
    bool fused = n_ar == 0 && n >= 2;
    if (a.table) {
      const int first = fused ? find_or_enter(a, b, mem, s, n, n0 + g) : -1;
      a.dup_of[nslot + g] = first;
      if (first >= 0) {
        fused = false;                         // no rows of its own
        ++n_repeats;
      }
    }
    float ot, as;
    if (n_ar == n) {
      ot = 0.0f;
      as = (float)size;
    } else if (n_ar == 0) {
      ot = n == 1 ? tb[mem[s]] : 0.0f;      // a fused op's time is written by fo_time_kernel / fo_repeat_kernel
      as = -1.0f;
    } else {
      ot = INFINITY;
      as = -1.0f;
    }
    a.op_time[n0 + g] = ot;
    a.ar_size[n0 + g] = as;
    gfm[g] = fused ? n : 0;
    gfk[g] = fused ? 1 : 0;
  }
  if (a.table) {
    for (int o = 32; o > 0; o >>= 1) n_repeats += __shfl_down(n_repeats, o, 64);
    if ((t & 63) == 0 && n_repeats > 0) atomicAdd(&a.totals[5], n_repeats);
  }
  __syncthreads();
  int Mc, Kc;
  block_exscan_pair(gfm, gfk, G, wsum, Mc, Kc);
  if (t == 0) {
    gfm[G] = Mc;
    gfk[G] = Kc;
  }
  __syncthreads();
  // edges inside a group, per member (in member order), both directions
  const int* rp = a.bg.rowptr + gb + b;
  const int* ci = a.bg.col + a.bg.geo[b];
  const int* crp = a.bg.crowptr + gb + b;
  const int* cci = a.bg.ccol + a.bg.geo[b];
  int* dgo = a.dgo + nslot;
  int* dgi = a.dgi + nslot;
  for (int i = t; i < N; i += T) {
    const int u = mem[i], g = nid[u];
    int no = 0, ni = 0;
    if (gfm[g + 1] != gfm[g]) {
      for (int k = rp[u]; k < rp[u + 1]; ++k) no += nid[ci[k]] == g;
      for (int k = crp[u]; k < crp[u + 1]; ++k) ni += nid[cci[k]] == g;
    }
    dgo[i] = no;
    dgi[i] = ni;
  }
  __syncthreads();
  int Eo, Ei;
  block_exscan_pair(dgo, dgi, N, wsum, Eo, Ei);
  if (t == 0) {
    dgo[N] = Eo;
    dgi[N] = Ei;
    a.cnt[c] = Kc;
    a.cnt[a.n_cand + 1 + c] = Mc;
    a.cnt[2 * (a.n_cand + 1) + c] = Eo;
    if (Eo != Ei) set_error(a.status, (int)DC_ERR_BAD_GRAPH);
  }
}

__global__ __launch_bounds__(1024) void fo_scan_kernel(FusedOpsArgs a) {
  __shared__ int wsum[16];
  if (a.status[0] != 0) return;
  const int C = a.n_cand;
  int* cK = a.cnt;
  int* cM = a.cnt + (C + 1);
  int* cE = a.cnt + 2 * (C + 1);
  const int K = block_exscan(cK, cK, C, wsum);
  const int M = block_exscan(cM, cM, C, wsum);
  const int E = block_exscan(cE, cE, C, wsum);
  if (threadIdx.x == 0) {
    cK[C] = K;
    cM[C] = M;
    cE[C] = E;
    if (K > a.cap_ops || M > a.cap_rows || E > a.cap_edges) {
      set_error(a.status, (int)DC_ERR_CAPACITY);
      a.totals[1] = 0;
      a.totals[3] = 0;
      return;
    }
    a.totals[0] = 0;       // {0, rows}: offsets of the whole batch as one graph, for the layer kernels
    a.totals[1] = M;
    a.totals[2] = 0;       // {0, fused ops}: the same for the dense layers of the regression network
    a.totals[3] = K;
    a.totals[4] = E;
    a.fb.node_off[K] = M;
    a.fb.edge_off[K] = E;
    a.fb.out_rowptr[M] = E;
    a.fb.in_rowptr[M] = E;
  }
}

// position of w in the ascending list m[0..n)
__device__ __forceinline__ int rank_in(const int* m, int n, int w) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (m[mid] <= w) lo = mid; else hi = mid;
  }
  return lo;
}

template <bool kBf16>
__global__ __launch_bounds__(256) void fo_fill_kernel(FusedOpsArgs a) {
  if (a.status[0] != 0) return;
  const int c = blockIdx.x, t = threadIdx.x, T = blockDim.x, C = a.n_cand;
  const int b = a.cand_graph[c];
  const int coff = a.cand_off[c], N = a.cand_off[c + 1] - coff, nslot = coff + c;
  const int G = a.Gc[c], gb = a.bg.gno[b], n0 = a.c_node_off[c];
  const int k0 = a.cnt[c], m0 = a.cnt[C + 1 + c], e0 = a.cnt[2 * (C + 1) + c];
  const int Mc = a.cnt[C + 1 + c + 1] - m0;
  const int* ms = a.mstart + nslot;
  const int* mem = a.members + coff;
  const int* nid = a.new_id + coff;
  const int* gfm = a.gfm + nslot;
  const int* gfk = a.gfk + nslot;
  const int* dgo = a.dgo + nslot;
  const int* dgi = a.dgi + nslot;
  for (int g = t; g < G; g += T) {
    if (gfm[g + 1] == gfm[g]) continue;
    const int k = k0 + gfk[g];
    a.fb.node_off[k] = m0 + gfm[g];
    a.fb.edge_off[k] = e0 + dgo[ms[g]];
    a.fo_cnode[k] = n0 + g;
  }
  const int* rp = a.bg.rowptr + gb + b;
  const int* ci = a.bg.col + a.bg.geo[b];
  const int* crp = a.bg.crowptr + gb + b;
  const int* cci = a.bg.ccol + a.bg.geo[b];
  for (int i = t; i < N; i += T) {
    const int u = mem[i], g = nid[u];
    if (gfm[g + 1] == gfm[g]) continue;
    const int s = ms[g], n = ms[g + 1] - s;
    const int first = m0 + gfm[g];            // row of the group's first member
    const int row = first + (i - s);
    a.fb.new_id[row] = u;
    int ko = e0 + dgo[i], ki = e0 + dgi[i];
    a.fb.out_rowptr[row] = ko;
    a.fb.in_rowptr[row] = ki;
    for (int k = rp[u]; k < rp[u + 1]; ++k) {
      const int w = ci[k];
      if (nid[w] == g) a.fb.out_col[ko++] = first + rank_in(mem + s, n, w);
    }
    for (int k = crp[u]; k < crp[u + 1]; ++k) {
      const int w = cci[k];
      if (nid[w] == g) a.fb.in_col[ki++] = first + rank_in(mem + s, n, w);
    }
  }
  __syncthreads();          // fb.new_id of this candidate's rows is complete
  const int q = a.F >> 2;
  const float4* X4 = reinterpret_cast<const float4*>(a.bg.X) + (size_t)gb * q;
  for (int i = t; i < Mc * q; i += T) {
    const int r = i / q, f = i - r * q;
    const size_t row = (size_t)(m0 + r);
    const float4 x = X4[(size_t)a.fb.new_id[row] * q + f];
    if (kBf16) {
      uint2 p;
      p.x = pack_bf16x2(x.x, x.y);
      p.y = pack_bf16x2(x.z, x.w);
      reinterpret_cast<uint2*>(a.fb.Xc)[row * q + f] = p;
    } else {
      reinterpret_cast<float4*>(a.fb.Xc)[row * q + f] = x;
    }
  }
}

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
    const float4 u = p[0], v = p[1];
    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
    x[4] = v.x; x[5] = v.y; x[6] = v.z; x[7] = v.w;
  }
}

// r_k = sum over the rows of fused op k of the final embeddings.  H / 8 lanes per fused op,
// eight columns each; the rows of a fused op are contiguous, two of them in flight.
template <bool kBf16>
__global__ __launch_bounds__(256) void fo_readout_kernel(const void* __restrict__ h, int H,
                                                          const int* __restrict__ node_off,
                                                          const int* __restrict__ totals, void* __restrict__ R,
                                                          const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int K = totals[3];
  const int LPR = H >> 3, per_wave = 64 / LPR;
  const int lane = threadIdx.x & 63, sg = lane / LPR, ll = lane - sg * LPR;
  if (sg >= per_wave) return;
  const long long wave0 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
  for (long long k = wave0 * per_wave + sg; k < K; k += nwaves * per_wave) {
    const int p0 = node_off[k], p1 = node_off[k + 1];
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int p = p0;
    for (; p + 1 < p1; p += 2) {
      float x[8], y[8];
      load8<kBf16>(h, (size_t)p, H, ll, x);
      load8<kBf16>(h, (size_t)p + 1, H, ll, y);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = (acc[i] + (double)x[i]) + (double)y[i];
    }
    if (p < p1) {
      float x[8];
      load8<kBf16>(h, (size_t)p, H, ll, x);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += (double)x[i];
    }
    if constexpr (kBf16) {
      v4u o;
      o.x = pack_bf16x2((float)acc[0], (float)acc[1]);
      o.y = pack_bf16x2((float)acc[2], (float)acc[3]);
      o.z = pack_bf16x2((float)acc[4], (float)acc[5]);
      o.w = pack_bf16x2((float)acc[6], (float)acc[7]);
      reinterpret_cast<v4u*>(R)[(size_t)k * LPR + ll] = o;
    } else {
      float4* o = reinterpret_cast<float4*>(R) + (size_t)k * (H >> 2) + 2 * ll;
      o[0] = make_float4((float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]);
      o[1] = make_float4((float)acc[4], (float)acc[5], (float)acc[6], (float)acc[7]);
    }
  }
}

// t_k = max(0, z2_k . w3 + b3) -> op_time of the fused op's node; the raw value also goes to
// fo_pred when that is not null.  fp64 accumulation in a fixed order.
template <bool kBf16>
__global__ __launch_bounds__(256) void fo_time_kernel(const void* __restrict__ Z, int H,
                                                       const float* __restrict__ w3b3,
                                                       const int* __restrict__ fo_cnode,
                                                       const int* __restrict__ totals, float* __restrict__ op_time,
                                                       float* __restrict__ fo_pred, const int* __restrict__ status) {
  if (status[0] != 0) return;
  const int K = totals[3];
  const int LPR = H >> 3, per_wave = 64 / LPR;
  const int lane = threadIdx.x & 63, sg = lane / LPR, ll = lane - sg * LPR, hb = sg * LPR;
  const bool active = sg < per_wave;
  const long long wave0 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
  float w[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) w[i] = active ? w3b3[ll * 8 + i] : 0.0f;
  const double b3 = (double)w3b3[H];
  for (long long k0 = wave0 * per_wave; k0 < K; k0 += nwaves * per_wave) {      // wave-uniform trip count
    const long long k = k0 + sg;
    double part = 0.0;
    if (active && k < K) {
      float x[8];
      load8<kBf16>(Z, (size_t)k, H, ll, x);
#pragma unroll
      for (int i = 0; i < 8; ++i) part += (double)x[i] * (double)w[i];
    }
    double sum = b3;
    if ((LPR & (LPR - 1)) == 0) {            // the lanes of a fused op are adjacent and LPR-aligned
      for (int o = 1; o < LPR; o <<= 1) part += __shfl_xor(part, o, 64);
      sum += part;
    } else {
      for (int j = 0; j < LPR; ++j) sum += __shfl(part, (hb + j) & 63, 64);
    }
    if (active && k < K && ll == 0) {
      const float tk = (float)sum;
      op_time[fo_cnode[k]] = tk > 0.0f ? tk : 0.0f;
      if (fo_pred) fo_pred[k] = tk;
    }
  }
}

// The time of a fused op that repeats an earlier one of the batch: that one's.
__global__ __launch_bounds__(256) void fo_repeat_kernel(FusedOpsArgs a) {
  if (a.status[0] != 0) return;
  const int c = blockIdx.x;
  const int nslot = a.cand_off[c] + c, G = a.Gc[c], n0 = a.c_node_off[c];
  for (int g = threadIdx.x; g < G; g += blockDim.x) {
    const int first = a.dup_of[nslot + g];
    if (first >= 0) a.op_time[n0 + g] = a.op_time[first];
  }
}

}  // namespace

// Places of the table for up to `max_fused_ops` entries: a power of two, at most half full.
size_t fused_op_table_entries(long long max_fused_ops) {
  size_t n = 1024;
  while (n < 2 * (size_t)(max_fused_ops > 0 ? max_fused_ops : 1)) n <<= 1;
  return n;
}

hipError_t launch_fused_op_extract(const FusedOpsArgs& a, Profiler* prof, hipStream_t s) {
  if (a.n_cand <= 0) return hipSuccess;
  if (prof) prof->begin(kFamFusedOps, s);
  if (a.table)
    hipLaunchKernelGGL(fo_clear_table_kernel, dim3(a.n_cu * 8), dim3(256), 0, s, a.table, a.table_mask, a.totals);
  hipLaunchKernelGGL(fo_count_kernel, dim3(a.n_cand), dim3(256), 0, s, a);
  hipLaunchKernelGGL(fo_scan_kernel, dim3(1), dim3(1024), 0, s, a);
  if (a.bf16) hipLaunchKernelGGL(fo_fill_kernel<true>, dim3(a.n_cand), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(fo_fill_kernel<false>, dim3(a.n_cand), dim3(256), 0, s, a);
  if (prof) prof->end(s);
  return hipGetLastError();
}

hipError_t launch_fused_op_readout(const FusedOpsArgs& a, const void* h_last, void* R, hipStream_t s) {
  const dim3 grid(a.n_cu * 8), block(256);
  if (a.bf16)
    hipLaunchKernelGGL(fo_readout_kernel<true>, grid, block, 0, s, h_last, a.H, a.fb.node_off, a.totals, R, a.status);
  else
    hipLaunchKernelGGL(fo_readout_kernel<false>, grid, block, 0, s, h_last, a.H, a.fb.node_off, a.totals, R, a.status);
  return hipGetLastError();
}

hipError_t launch_fused_op_times(const FusedOpsArgs& a, const void* Z2, const float* w3b3, float* fo_pred,
                                 hipStream_t s) {
  const dim3 grid(a.n_cu * 8), block(256);
  if (a.bf16)
    hipLaunchKernelGGL(fo_time_kernel<true>, grid, block, 0, s, Z2, a.H, w3b3, a.fo_cnode, a.totals, a.op_time,
                       fo_pred, a.status);
  else
    hipLaunchKernelGGL(fo_time_kernel<false>, grid, block, 0, s, Z2, a.H, w3b3, a.fo_cnode, a.totals, a.op_time,
                       fo_pred, a.status);
  if (a.table && a.n_cand > 0) hipLaunchKernelGGL(fo_repeat_kernel, dim3(a.n_cand), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace dc

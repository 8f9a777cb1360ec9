// Graph contraction of fusion candidates (gfx950).
//
// A candidate is a base training DAG plus one label per node; nodes with equal
// labels form one fused op or one fused gradient tensor (strategy space of
// Sec. 3.2).  The fused op is the subgraph of its original ops (Sec. 3.3), so the
// candidate module is the quotient graph: dependencies inside a group vanish,
// those that cross groups stay, parallel ones collapse (0/1 adjacency,
// Sec. 3.3.1).  Node features are summed per group (Sec. 2.3: the size of a fused
// tensor is the sum of its members' sizes).
//
// One workgroup contracts one candidate entirely in LDS (or, for base graphs
// that do not fit, in a per-workgroup slab of global memory with the same
// layout).  Results go to per-candidate scratch slots; after a scan of the
// contracted sizes over the batch a second kernel places them block-diagonally
// and reduces the features.
//
// Output is canonical, hence unique: groups are numbered by ascending smallest
// member index and every neighbour list is ascending.
#include <limits.h>

#include "common.h"

namespace dc {
namespace {

constexpr int kCT = 1024;       // threads per contraction workgroup
constexpr int kCW = kCT / 64;   // waves per workgroup
constexpr int kSmallRow = 16;   // lists up to this length are sorted by one thread in registers, up to 64 by a wave
constexpr unsigned short kSelf = 0xFFFF;

typedef unsigned short u16;

// Byte offsets of the per-candidate working arrays (same on host and device).
struct Slab {
  int A, MS, UL, BM, NID, MEM, RAW, LST, total;
};
__host__ __device__ inline int align16(int x) { return (x + 15) & ~15; }
__host__ __device__ inline Slab slab_layout(int N, int E) {
  Slab s;
  int o = 0;
  s.A = o;   o = align16(o + 4 * (N + 1));          // int   [N+1] label->first / cursors / raw offsets
  s.MS = o;  o = align16(o + 4 * (N + 1));          // int   [N+1] group start in MEM
  s.UL = o;  o = align16(o + 4 * (N + 1));          // int   [N+1] flags / row lengths / local rowptr
  s.BM = o;  o = align16(o + 4 * kCW * ((N + 31) / 32 + 1));  // per-wave bitmaps
  s.NID = o; o = align16(o + 2 * (N + 1));          // u16   [N] contracted id per base node
  s.MEM = o; o = align16(o + 2 * (N + 1));          // u16   [N] base nodes grouped by contracted id
  s.RAW = o; o = align16(o + 2 * ((E > N ? E : N) + 1));   // u16 [max(E,N)] labels, later remapped neighbours by row
  s.LST = o; o = align16(o + 2 * (N + 1));          // u16   [N] lists set aside for the second sorting pass
  s.total = o;
  return s;
}

// Short lists (up to 16 entries) are sorted by one thread each, in registers, with a
// fixed compare-exchange network (Batcher's odd-even merge sort): no dependent chain
// through memory, and the same instruction stream for every lane.  Unused places hold
// kSelf (0xFFFF), which sorts to the end.
template <int NN>
__device__ __forceinline__ void sort_network(unsigned (&v)[NN]) {
#pragma unroll
  for (int p = 1; p < NN; p <<= 1)
#pragma unroll
    for (int k = p; k >= 1; k >>= 1)
#pragma unroll
      for (int j = k % p; j + k < NN; j += 2 * k)
#pragma unroll
        for (int i = 0; i < k; ++i)
          if (i + j + k < NN && (i + j) / (2 * p) == (i + j + k) / (2 * p)) {
            const unsigned lo = min(v[i + j], v[i + j + k]), hi = max(v[i + j], v[i + j + k]);
            v[i + j] = lo;
            v[i + j + k] = hi;
          }
}

// Sorts a[0..n) ascending, drops entries equal to kSelf and repeats; returns the count kept.
template <int NN>
__device__ __forceinline__ int sort_unique_small(u16* a, int n) {
  unsigned v[NN];
#pragma unroll
  for (int k = 0; k < NN; ++k) v[k] = k < n ? (unsigned)a[k] : (unsigned)kSelf;
  sort_network<NN>(v);
  int m = 0;
#pragma unroll
  for (int k = 0; k < NN; ++k) {
    const bool keep = v[k] != (unsigned)kSelf && (k == 0 || v[k] != v[k - 1]);
    if (keep) a[m++] = (u16)v[k];
  }
  return m;
}

// Picks the smallest network that covers every list of the wave (n is 0 for lanes without one).
__device__ __forceinline__ int sort_unique_by_class(u16* a, int n) {
  if (__any(n > 8)) return sort_unique_small<16>(a, n);
  if (__any(n > 4)) return sort_unique_small<8>(a, n);
  if (__any(n > 1)) return sort_unique_small<4>(a, n);
  return (n == 1 && a[0] != kSelf) ? 1 : 0;
}

// Same for one list of up to 64 entries held by a whole wave (lane i holds entry i).
__device__ __forceinline__ bool rank64(unsigned x, int lane, int n, int& pos, int& m) {
  bool first = lane < n && x != kSelf;
  for (int j = 0; j < n; ++j) {
    const unsigned y = (unsigned)__shfl((int)x, j, 64);
    if (j < lane && y == x) first = false;
  }
  const unsigned long long kb = __ballot(first);
  int p = 0;
  for (int j = 0; j < n; ++j) {
    const unsigned y = (unsigned)__shfl((int)x, j, 64);
    if (((kb >> j) & 1ull) && y < x) ++p;
  }
  pos = p;
  m = __popcll(kb);
  return first;
}

// The body works on plain pointers; instantiated once with LDS pointers and
// once with global-memory pointers.
template <bool kLds>
__device__ __forceinline__ void contract_one(const BaseGraphs& bg, int c, int b, int N, char* base, const Slab& L,
                                             const int* cand_off, const int* label, const ContractTmp& tmp,
                                             int* new_id_out, int* status, int* wsum) {
  const int t = threadIdx.x, T = blockDim.x, lane = t & 63, wave = t >> 6;
  int* A = reinterpret_cast<int*>(base + L.A);
  int* MS = reinterpret_cast<int*>(base + L.MS);
  int* UL = reinterpret_cast<int*>(base + L.UL);
  const int bm_words = (N + 31) / 32 + 1;
  unsigned* BM = reinterpret_cast<unsigned*>(base + L.BM) + wave * bm_words;
  u16* NID = reinterpret_cast<u16*>(base + L.NID);
  u16* MEM = reinterpret_cast<u16*>(base + L.MEM);
  u16* RAW = reinterpret_cast<u16*>(base + L.RAW);
  u16* LST = reinterpret_cast<u16*>(base + L.LST);
  int* lst_cnt = wsum + kCW;       // one more word behind the scan's wave sums

  const int coff = cand_off[c];
  const int* lab = label + coff;
  int* nid_out = new_id_out + coff;
  const int nslot = coff + c;
  const int eslot = tmp.tmp_eoff[c];

  // ---- relabel: groups numbered by ascending smallest member -----------------
  int bad = 0;
  u16* LAB = RAW;                 // labels stay in LDS until the ids are known; RAW is unused until then
#pragma unroll 4
  for (int v = t; v < N; v += T) {
    A[v] = INT_MAX;
    int l = lab[v];
    bad |= (l < 0) | (l >= N);
    LAB[v] = (u16)l;
  }
  {
    unsigned* bmall = reinterpret_cast<unsigned*>(base + L.BM);
    for (int i = t; i < kCW * bm_words; i += T) bmall[i] = 0u;
  }
  if (__syncthreads_or(bad)) {
    if (t == 0) {
      set_error(status, (int)DC_ERR_BAD_PARTITION);
      tmp.Gc[c] = 0;
      tmp.Ec[c] = 0;
    }
    return;
  }
  for (int v = t; v < N; v += T) atomicMin(&A[LAB[v]], v);
  __syncthreads();
  for (int v = t; v < N; v += T) UL[v] = (A[LAB[v]] == v) ? 1 : 0;
  __syncthreads();
  const int G = kLds ? block_exscan(UL, UL, N, wsum) : block_exscan_lines(UL, UL, N, wsum);
  if (t == 0) UL[N] = G;
  __syncthreads();
  for (int v = t; v < N; v += T)
    if (UL[v + 1] != UL[v]) A[LAB[v]] = UL[v];   // head of its group: rank among heads
  __syncthreads();
  for (int v = t; v < N; v += T) {
    int g = A[LAB[v]];
    NID[v] = (u16)g;
    nid_out[v] = g;
  }
  __syncthreads();

  // ---- member lists: counting sort by group, ascending inside a group ---------
  for (int g = t; g < G; g += T) A[g] = 0;
  __syncthreads();
  for (int v = t; v < N; v += T) atomicAdd(&A[NID[v]], 1);
  __syncthreads();
  if (kLds) block_exscan(A, MS, G, wsum); else block_exscan_lines(A, MS, G, wsum);
  if (t == 0) MS[G] = N;
  __syncthreads();
  for (int g = t; g < G; g += T) A[g] = MS[g];
  __syncthreads();
  for (int v = t; v < N; v += T) {
    int pos = atomicAdd(&A[NID[v]], 1);
    MEM[pos] = (u16)v;
  }
  __syncthreads();
  {
    // ascending order inside each group (the atomics above placed members in arrival order):
    // groups of up to 16 at once, one thread each; longer ones are set aside and taken
    // densely packed afterwards (up to 32: one thread; up to 64: one wave; else all nodes)
    if (t == 0) *lst_cnt = 0;
    __syncthreads();
    for (int g0 = 0; g0 < G; g0 += T) {         // uniform trip count: the wave votes on the network size
      const int g = g0 + t;
      int s = 0, n = 0;
      if (g < G) {
        s = MS[g];
        n = MS[g + 1] - s;
      }
      if (n > kSmallRow) {
        LST[atomicAdd(lst_cnt, 1)] = (u16)g;
        n = 0;
      }
      sort_unique_by_class(MEM + s, n);          // members are distinct: all are kept
    }
    __syncthreads();
    const int nl = *lst_cnt;
    int big = 0;
    for (int i0 = 0; i0 < nl; i0 += T) {
      const int i = i0 + t;
      int s = 0, n = 0;
      if (i < nl) {
        const int g = LST[i];
        s = MS[g];
        n = MS[g + 1] - s;
        if (n > 32) {
          big = 1;
          n = 0;
        }
      }
      if (__any(n > 0)) sort_unique_small<32>(MEM + s, n);
    }
    if (__syncthreads_or(big)) {
      for (int i = wave; i < nl; i += kCW) {
        const int g = LST[i];
        const int s = MS[g], n = MS[g + 1] - s;
        if (n <= 32) continue;
        if (n <= 64) {
          const unsigned x = lane < n ? MEM[s + lane] : kSelf;
          int pos, m;
          const bool keep = rank64(x, lane, n, pos, m);
          if (keep) MEM[s + pos] = (u16)x;
          continue;
        }
        // large groups: ordered compaction over all nodes
        int cnt = 0;
        for (int v0 = 0; v0 < N; v0 += 64) {
          int v = v0 + lane;
          bool f = v < N && NID[v] == g;
          unsigned long long m = __ballot(f);
          if (f) MEM[s + cnt + __popcll(m & ((1ull << lane) - 1ull))] = (u16)v;
          cnt += __popcll(m);
        }
      }
    }
    __syncthreads();
  }
  for (int i = t; i < N; i += T) tmp.members[coff + i] = MEM[i];
  for (int g = t; g <= G; g += T) tmp.mstart[nslot + g] = MS[g];

  // ---- neighbour lists: successors (dir 0), then predecessors (dir 1) ----------
  int Ec = 0;
  for (int dir = 0; dir < 2; ++dir) {
    const int* rp = (dir == 0 ? bg.rowptr : bg.crowptr) + bg.gno[b] + b;
    const int* ci = (dir == 0 ? bg.col : bg.ccol) + bg.geo[b];
    int* t_rp = (dir == 0 ? tmp.orp : tmp.irp) + nslot;
    int* t_ci = (dir == 0 ? tmp.oc : tmp.ic) + eslot;

#pragma unroll 4
    for (int i = t; i < N; i += T) {
      int u = MEM[i];
      A[i] = rp[u + 1] - rp[u];
    }
    __syncthreads();
    const int Eraw = kLds ? block_exscan(A, A, N, wsum) : block_exscan_lines(A, A, N, wsum);
    if (t == 0) A[N] = Eraw;
    __syncthreads();
    // four member slots per thread and round: their row starts and first neighbours are
    // requested together so that the global-memory latency is paid once per round
    for (int i0 = t; i0 < N; i0 += 4 * T) {
      int uu[4], o[4], dg[4], r0[4], c0[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * T;
        const bool ok = i < N;
        uu[j] = ok ? MEM[i] : 0;
        o[j] = ok ? A[i] : 0;
        dg[j] = ok ? A[i + 1] - A[i] : 0;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) r0[j] = dg[j] > 0 ? rp[uu[j]] : 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) c0[j] = dg[j] > 0 ? ci[r0[j]] : 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (dg[j] > 0) {
          const int g = NID[uu[j]];
          int w = NID[c0[j]];
          RAW[o[j]] = (w == g) ? kSelf : (u16)w;
          for (int k = 1; k < dg[j]; ++k) {
            w = NID[ci[r0[j] + k]];
            RAW[o[j] + k] = (w == g) ? kSelf : (u16)w;
          }
        }
      }
    }
    __syncthreads();
    // same three passes as for the member lists; here entries equal to kSelf and repeats go
    if (t == 0) *lst_cnt = 0;
    __syncthreads();
    for (int g0 = 0; g0 < G; g0 += T) {         // uniform trip count: the wave votes on the network size
      const int g = g0 + t;
      int s = 0, n = 0;
      if (g < G) {
        s = A[MS[g]];
        n = A[MS[g + 1]] - s;
      }
      const bool here = n <= kSmallRow;
      if (!here) {
        LST[atomicAdd(lst_cnt, 1)] = (u16)g;
        n = 0;
      }
      const int m = sort_unique_by_class(RAW + s, n);
      if (here && g < G) UL[g] = m;
    }
    __syncthreads();
    const int nl = *lst_cnt;
    int big = 0;
    for (int i0 = 0; i0 < nl; i0 += T) {
      const int i = i0 + t;
      int s = 0, n = 0, g = 0;
      if (i < nl) {
        g = LST[i];
        s = A[MS[g]];
        n = A[MS[g + 1]] - s;
        if (n > 32) {
          big = 1;
          n = 0;
        }
      }
      if (__any(n > 0)) {
        const int m = sort_unique_small<32>(RAW + s, n);
        if (n > 0) UL[g] = m;
      }
    }
    if (__syncthreads_or(big)) {
      const int W = (G + 31) / 32;
      for (int i = wave; i < nl; i += kCW) {
        const int g = LST[i];
        const int s = A[MS[g]], n = A[MS[g + 1]] - s;
        if (n <= 32) continue;
        if (n <= 64) {
          const unsigned x = lane < n ? RAW[s + lane] : kSelf;
          int pos, m;
          const bool keep = rank64(x, lane, n, pos, m);
          if (keep) RAW[s + pos] = (u16)x;
          if (lane == 0) UL[g] = m;
          continue;
        }
        // long rows: mark neighbours in a per-wave bitmap, then list the set bits
        for (int i2 = lane; i2 < n; i2 += 64) {
          u16 x = RAW[s + i2];
          if (x != kSelf) atomicOr(&BM[x >> 5], 1u << (x & 31));
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        int cnt = 0;
        for (int w0 = 0; w0 < W; w0 += 64) {
          const int w = w0 + lane;
          unsigned bits = (w < W) ? BM[w] : 0u;
          if (bits) BM[w] = 0u;
          const int pc = __popc(bits);
          const int inc = wave_incl_scan(pc);
          int o = s + cnt + inc - pc;
          while (bits) {
            int bpos = __ffs(bits) - 1;
            RAW[o++] = (u16)((w << 5) + bpos);
            bits &= bits - 1;
          }
          cnt += __shfl(inc, 63, 64);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        if (lane == 0) UL[g] = cnt;
      }
    }
    __syncthreads();
    Ec = kLds ? block_exscan(UL, UL, G, wsum) : block_exscan_lines(UL, UL, G, wsum);
    if (t == 0) UL[G] = Ec;
    __syncthreads();
    for (int g = t; g <= G; g += T) t_rp[g] = UL[g];
    for (int g = t; g < G; g += T) {
      const int s = A[MS[g]], o = UL[g], n = UL[g + 1] - o;
      for (int k = 0; k < n; ++k) t_ci[o + k] = RAW[s + k];
    }
    __syncthreads();
  }
  if (t == 0) {
    tmp.Gc[c] = G;
    tmp.Ec[c] = Ec;
  }
}

extern __shared__ __attribute__((aligned(16))) char dc_smem[];

template <bool kLds>
__global__ __launch_bounds__(kCT) void contract_kernel(BaseGraphs bg, int C, const int* cand_graph,
                                                        const int* cand_off, const int* label, ContractTmp tmp,
                                                        int* new_id_out, int* status, char* gslab,
                                                        size_t slab_stride, int lds_bytes) {
  __shared__ int wsum[kCW + 1];
  if (status[0] != 0) return;
  if (kLds) {
    for (int c = blockIdx.x; c < C; c += gridDim.x) {
      const int b = cand_graph[c];
      const int N = bg.gno[b + 1] - bg.gno[b];
      const int E = bg.geo[b + 1] - bg.geo[b];
      const Slab L = slab_layout(N, E);
      if (L.total > lds_bytes) continue;
      contract_one<true>(bg, c, b, N, dc_smem, L, cand_off, label, tmp, new_id_out, status, wsum);
      __syncthreads();
    }
  } else {
    // The candidates that work in global memory are few and long and differ several times in size: they
    // are handed out one at a time, largest first (the order prep_kernel leaves), through a counter.
    __shared__ int next_item;
    const int n_big = tmp.big_meta[0];
    for (;;) {
      if (threadIdx.x == 0) next_item = atomicAdd(&tmp.big_meta[1], 1);
      __syncthreads();
      const int i = next_item;
      __syncthreads();                          // everyone has read it before thread 0 writes the next one
      if (i >= n_big) break;
      const int c = tmp.big_order[i];
      const int b = cand_graph[c];
      const int N = bg.gno[b + 1] - bg.gno[b];
      const int E = bg.geo[b + 1] - bg.geo[b];
      const Slab L = slab_layout(N, E);
      contract_one<false>(bg, c, b, N, gslab + (size_t)blockIdx.x * slab_stride, L, cand_off, label, tmp,
                          new_id_out, status, wsum);
      __syncthreads();
    }
  }
}

// Validates the candidate list and scans the base edge counts (one workgroup).
__global__ __launch_bounds__(1024) void prep_kernel(BaseGraphs bg, int C, const int* cand_graph, const int* cand_off,
                                                     int* tmp_eoff, long long max_base_nodes,
                                                     long long max_base_edges, int* status, int* big_order,
                                                     int* big_meta, int lds_bytes, int need_max) {
  __shared__ int wsum[16];
  const int t = threadIdx.x, T = blockDim.x;
  int bad = 0;
  for (int c = t; c < C; c += T) {
    const int b = cand_graph[c];
    int e = 0;
    if (b < 0 || b >= bg.n_graphs) {
      bad = 1;
    } else {
      const int n = bg.gno[b + 1] - bg.gno[b];
      if (cand_off[c + 1] - cand_off[c] != n) bad = 1;
      e = bg.geo[b + 1] - bg.geo[b];
    }
    tmp_eoff[c] = e;
  }
  if (t == 0 && cand_off[0] != 0) bad = 1;
  bad = __syncthreads_or(bad);
  if (bad) {
    if (t == 0) set_error(status, (int)DC_ERR_BAD_PARTITION);
    return;
  }
  // 64-bit check of the edge total before the 32-bit scan
  long long es = 0;
  for (int c = t; c < C; c += T) es += tmp_eoff[c];
  __shared__ long long esum[16];
  for (int o = 32; o > 0; o >>= 1) es += __shfl_down(es, o, 64);
  if ((t & 63) == 0) esum[t >> 6] = es;
  __syncthreads();
  long long tot = 0;
  for (int i = 0; i < (T >> 6); ++i) tot += esum[i];
  if (tot > max_base_edges || (long long)cand_off[C] > max_base_nodes) {
    if (t == 0) set_error(status, (int)DC_ERR_CAPACITY);
    return;
  }
  const int total = block_exscan(tmp_eoff, tmp_eoff, C, wsum);
  if (t == 0) tmp_eoff[C] = total;
  // The candidates whose base graph does not fit LDS, in sixteen classes of working-set size, largest class
  // first (the order inside a class is whatever the atomics give: it decides which workgroup contracts a
  // candidate, not what is written).
  __shared__ int hist[16], base[16];
  if (t < 16) hist[t] = 0;
  __syncthreads();
  const int span = need_max > lds_bytes ? need_max - lds_bytes : 1;
  auto size_class = [&](int c) {
    const int b = cand_graph[c];
    const int need = slab_layout(bg.gno[b + 1] - bg.gno[b], bg.geo[b + 1] - bg.geo[b]).total;
    if (need <= lds_bytes) return -1;
    const long long k = (long long)(need - lds_bytes) * 16 / span;
    return (int)(k > 15 ? 15 : k);
  };
  for (int c = t; c < C; c += T) {
    const int k = size_class(c);
    if (k >= 0) atomicAdd(&hist[k], 1);
  }
  __syncthreads();
  if (t == 0) {
    int run = 0;
    for (int k = 15; k >= 0; --k) {
      base[k] = run;
      run += hist[k];
    }
    big_meta[0] = run;
    big_meta[1] = 0;
  }
  __syncthreads();
  for (int c = t; c < C; c += T) {
    const int k = size_class(c);
    if (k >= 0) big_order[atomicAdd(&base[k], 1)] = c;
  }
}

// Scans contracted sizes over the batch and checks the output capacities.
__global__ __launch_bounds__(1024) void scan_sizes_kernel(int C, const int* Gc, const int* Ec, int* node_off,
                                                           int* edge_off, long long cap_nodes, long long cap_edges,
                                                           int* status, int* totals) {
  __shared__ int wsum[16];
  if (status[0] != 0) return;
  const int nt = block_exscan(Gc, node_off, C, wsum);
  const int et = block_exscan(Ec, edge_off, C, wsum);
  if (threadIdx.x == 0) {
    node_off[C] = nt;
    edge_off[C] = et;
    totals[0] = nt;
    totals[1] = et;
    if (nt > cap_nodes || et > cap_edges) set_error(status, (int)DC_ERR_CAPACITY);
  }
}


// Places candidate c's lists at their block-diagonal position and sums features.
template <bool kBf16>
__global__ __launch_bounds__(256) void finalize_kernel(BaseGraphs bg, int C, const int* cand_graph,
                                                        const int* cand_off, ContractTmp tmp, BatchView out, int F,
                                                        const int* status) {
  if (status[0] != 0) return;
  const int c = blockIdx.x, t = threadIdx.x, T = blockDim.x;
  const int b = cand_graph[c];
  const int coff = cand_off[c];
  const int nslot = coff + c, eslot = tmp.tmp_eoff[c];
  const int n0 = out.node_off[c], e0 = out.edge_off[c];
  const int G = tmp.Gc[c], E = tmp.Ec[c];
  const int gend = (c == C - 1) ? G + 1 : G;   // the last candidate also writes the closing entry
  for (int g = t; g < gend; g += T) {
    out.out_rowptr[n0 + g] = e0 + tmp.orp[nslot + g];
    out.in_rowptr[n0 + g] = e0 + tmp.irp[nslot + g];
  }
  for (int k = t; k < E; k += T) {
    out.out_col[e0 + k] = n0 + tmp.oc[eslot + k];
    out.in_col[e0 + k] = n0 + tmp.ic[eslot + k];
  }
  // feature sums: members in ascending base index, fp32 accumulation, one rounding.  A thread works on
  // four (group, column quad) items at a time, so that the dependent loads of an item (list bounds,
  // member numbers, member rows) overlap with those of three others: the loop is bound by memory latency.
  const int q = F >> 2;
  const float4* X4 = reinterpret_cast<const float4*>(bg.X) + (size_t)bg.gno[b] * q;
  const int* ms = tmp.mstart + nslot;
  const int* mem = tmp.members + coff;
  const int items = G * q;
  for (int i0 = t; i0 < items; i0 += 4 * T) {
    int f[4], m[4], me[4], g[4];
    float4 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = i0 + j * T;
      const bool ok = i < items;
      g[j] = ok ? i / q : 0;
      f[j] = ok ? i - g[j] * q : 0;
      m[j] = ok ? ms[g[j]] : 0;
      me[j] = ok ? ms[g[j] + 1] : 0;
      acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    // rounds of up to two members per item, the four items' loads in flight together; the member numbers of the
    // next round are asked for together with the rows of this one, so that a round costs one memory round trip
    int i0m[4], i1m[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      i0m[j] = m[j] < me[j] ? mem[m[j]] : -1;
      i1m[j] = m[j] + 1 < me[j] ? mem[m[j] + 1] : -1;
    }
    bool more = true;
    while (more) {
      float4 x0[4], x1[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        x0[j] = i0m[j] >= 0 ? X4[(size_t)i0m[j] * q + f[j]] : make_float4(0.f, 0.f, 0.f, 0.f);
        x1[j] = i1m[j] >= 0 ? X4[(size_t)i1m[j] * q + f[j]] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      int n0m[4], n1m[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        n0m[j] = m[j] + 2 < me[j] ? mem[m[j] + 2] : -1;
        n1m[j] = m[j] + 3 < me[j] ? mem[m[j] + 3] : -1;
      }
      more = false;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // added in member order; a member that does not exist adds nothing (not even +0 to a -0 sum)
        if (i0m[j] >= 0) { acc[j].x += x0[j].x; acc[j].y += x0[j].y; acc[j].z += x0[j].z; acc[j].w += x0[j].w; }
        if (i1m[j] >= 0) { acc[j].x += x1[j].x; acc[j].y += x1[j].y; acc[j].z += x1[j].z; acc[j].w += x1[j].w; }
        m[j] += 2;
        more |= m[j] < me[j];
        i0m[j] = n0m[j];
        i1m[j] = n1m[j];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = i0 + j * T;
      if (i >= items) continue;
      const size_t row = (size_t)(n0 + g[j]);
      if (kBf16) {
        uint2 p;
        p.x = pack_bf16x2(acc[j].x, acc[j].y);
        p.y = pack_bf16x2(acc[j].z, acc[j].w);
        reinterpret_cast<uint2*>(out.Xc)[row * q + f[j]] = p;
      } else {
        reinterpret_cast<float4*>(out.Xc)[row * q + f[j]] = acc[j];
      }
    }
  }
}

}  // namespace

int contract_working_set_bytes(int n_nodes, int n_edges) { return slab_layout(n_nodes, n_edges).total; }

__global__ void reset_status_kernel(int* status) { status[0] = 0; }

hipError_t launch_contract(const ContractLaunch& a, Profiler* prof, hipStream_t s) {
  if (a.n_cand <= 0) return hipSuccess;
  const int C = a.n_cand;
  if (prof) prof->begin(kFamPrep, s);
  const int need = slab_layout(a.max_graph_nodes, a.max_graph_edges).total;
  const int lds_bytes = need <= a.lds_limit ? need : a.lds_limit;
  hipLaunchKernelGGL(prep_kernel, dim3(1), dim3(1024), 0, s, a.bg, C, a.cand_graph, a.cand_off, a.tmp.tmp_eoff,
                     a.max_base_nodes, a.max_base_edges, a.status, a.tmp.big_order, a.tmp.big_meta, lds_bytes, need);
  if (prof) prof->end(s);
  if (prof) prof->begin(kFamContract, s);
  if (a.min_graph_need <= a.lds_limit) {   // at least one base graph fits in LDS
    hipLaunchKernelGGL(contract_kernel<true>, dim3(C), dim3(kCT), lds_bytes, s, a.bg, C, a.cand_graph, a.cand_off,
                       a.group_id, a.tmp, a.out.new_id, a.status, (char*)nullptr, (size_t)0, lds_bytes);
  }
  if (need > a.lds_limit) {                // at least one base graph needs the global slab
    hipLaunchKernelGGL(contract_kernel<false>, dim3(a.slab_wgs), dim3(kCT), 0, s, a.bg, C, a.cand_graph,
                       a.cand_off, a.group_id, a.tmp, a.out.new_id, a.status, a.slab, a.slab_stride, lds_bytes);
  }
  if (prof) prof->end(s);
  if (prof) prof->begin(kFamFinalize, s);
  hipLaunchKernelGGL(scan_sizes_kernel, dim3(1), dim3(1024), 0, s, C, a.tmp.Gc, a.tmp.Ec, a.out.node_off,
                     a.out.edge_off, a.out.cap_nodes, a.out.cap_edges, a.status, a.totals);
  if (a.bf16)
    hipLaunchKernelGGL(finalize_kernel<true>, dim3(C), dim3(256), 0, s, a.bg, C, a.cand_graph, a.cand_off, a.tmp,
                       a.out, a.F, a.status);
  else
    hipLaunchKernelGGL(finalize_kernel<false>, dim3(C), dim3(256), 0, s, a.bg, C, a.cand_graph, a.cand_off, a.tmp,
                       a.out, a.F, a.status);
  if (prof) prof->end(s);
  return hipGetLastError();
}

hipError_t contract_set_lds_limit(int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&contract_kernel<true>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace dc

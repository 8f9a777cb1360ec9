// Backtracking search over fusion strategies (Alg. 1, Sec. 4) on top of the batched cost model.
//
// A strategy is a labelling of the base nodes; H_in is the all-singleton labelling.  Per step
// up to `parents` entries leave the priority queue (ascending cost, then age); every parent
// gets one child per optimisation method, drawn on the device by mutate_kernel (RandomApply:
// n = Random(0, beta) applications of the method); the children are costed in one
// dc_cost_candidates call and then handled in order on the host: a valid child (finite cost)
// replaces H_opt when cheaper, which restarts the counter of unchanged evaluations, and is
// enqueued when Cost(H') <= alpha * Cost(H_opt).  The search ends when the queue is empty, the
// counter reaches its limit (checked between steps) or max_steps is reached.  parents = 1 is
// the loop as printed.
//
// Methods (Sec. 4, (i) and (iii); (ii) duplicates an op, which no labelling of the node set
// expresses):  op fusion, one application, in one of two forms.  DC_DRAW_DEPENDENCY: a dependency
// u -> v between two computation ops of the base module is drawn uniformly; if its ends lie in
// different groups, the group of u joins the group of v.  DC_DRAW_OP (the paper's wording): a
// computation op of the current module is drawn uniformly (the groups of the labelling, in the
// order of their smallest member), then one of its predecessor ops in the current module
// uniformly (the groups with a dependency into it, same order), and the predecessor joins the
// op; an op without predecessors leaves the module as it is; the low half of the 64-bit draw
// picks the op, the high half the predecessor.  Tensor fusion, one application: an all-reduce node a and a side are
// drawn uniformly; the nearest bucket on that side in production order, if there is one,
// joins the bucket of a.  Validity is what the cost reports: a cyclic module costs +infinity.
//
// Draws: key = mix(seed ^ mix(step * 2^32 + child)), draw d = mix(key + d * 0xD1342543DE82EF95)
// with mix = splitmix64's output function; draw 0 gives n, draws 1.. the applications.
#include <math.h>
#include <string.h>

#include <set>
#include <tuple>
#include <vector>

#include "common.h"

namespace dc {
namespace {

constexpr int kMutateLdsLimit = 160 * 1024 - 2048;   // dynamic LDS of mutate_kernel next to its static arrays

__host__ __device__ inline unsigned long long mix64(unsigned long long x) {
  unsigned long long z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

extern __shared__ __attribute__((aligned(16))) unsigned short dc_search_lab[];

// The k-th (from 0) position q of the op list, in ascending order, for which pred(q) holds, or -1 if
// fewer than k + 1 do; `pick` is called with the count of such positions and returns k.  Every
// thread of the workgroup takes a contiguous run of the list.  Three barriers; the result is
// uniform.  cnt: 256 ints, sel: 4 ints of LDS.
template <typename Pred, typename Pick>
__device__ int select_kth(int n_op, int* cnt, int* sel, Pred pred, Pick pick) {
  const int t = threadIdx.x, T = blockDim.x;
  const int ch = (n_op + T - 1) / T, lo = min(n_op, t * ch), hi = min(n_op, lo + ch);
  int c = 0;
  for (int q = lo; q < hi; ++q) c += pred(q) ? 1 : 0;
  cnt[t] = c;
  __syncthreads();
  if (t == 0) {
    int total = 0;
    for (int i = 0; i < T; ++i) total += cnt[i];
    sel[0] = -1;
    if (total > 0) {
      int k = pick(total), w = 0;
      while (k >= cnt[w]) k -= cnt[w++];
      sel[0] = w;
      sel[1] = k;
    }
  }
  __syncthreads();
  if (sel[0] == t) {
    int k = sel[1], q = lo;
    for (;; ++q)
      if (pred(q) && k-- == 0) break;
    sel[2] = q;
  }
  __syncthreads();
  const int r = sel[0] < 0 ? -1 : sel[2];
  __syncthreads();                           // sel and cnt may be written again
  return r;
}

// One workgroup per child: child j descends from parent j / 2 by method j % 2.  op_draw != 0 takes
// the paper's draw for op fusion and needs, behind the labels, 4 N bytes (smallest member per
// label) and N bytes (marks) of LDS.
__global__ __launch_bounds__(256) void mutate_kernel(const int* __restrict__ pool, const int* __restrict__ parent_slot,
                                                      int N, int n_edges, const int* __restrict__ esrc,
                                                      const int* __restrict__ edst, int n_ar,
                                                      const int* __restrict__ ar_nodes, int n_op,
                                                      const int* __restrict__ op_nodes, int op_draw,
                                                      unsigned long long seed, unsigned long long step, int beta,
                                                      int* __restrict__ children) {
  __shared__ int pair[2];
  __shared__ int cnt[256];
  __shared__ int sel[4];
  unsigned short* lab = dc_search_lab;
  int* first = reinterpret_cast<int*>(lab + ((N + 1) & ~1));
  unsigned char* mark = reinterpret_cast<unsigned char*>(first + N);
  const int j = blockIdx.x, t = threadIdx.x, T = blockDim.x;
  const int method = j & 1;
  const int* src = pool + (size_t)parent_slot[j >> 1] * N;
  for (int v = t; v < N; v += T) lab[v] = (unsigned short)src[v];
  const unsigned long long key = mix64(seed ^ mix64((step << 32) + (unsigned long long)j));
  const int n = (int)(mix64(key) % (unsigned long long)(beta + 1));
  __syncthreads();
  for (int i = 0; i < n; ++i) {
    const unsigned long long r = mix64(key + (unsigned long long)(1 + i) * 0xD1342543DE82EF95ull);
    int from = -1, to = -1;
    if (method == 0 && op_draw != 0) {
      // smallest member of every group of ops; a group's place in the order is that member's
      for (int v = t; v < N; v += T) {
        first[v] = 0x7FFFFFFF;
        mark[v] = 0;
      }
      __syncthreads();
      for (int q = t; q < n_op; q += T) atomicMin(&first[lab[op_nodes[q]]], op_nodes[q]);
      __syncthreads();
      const int qo = select_kth(
          n_op, cnt, sel, [&](int q) { return first[lab[op_nodes[q]]] == op_nodes[q]; },
          [&](int total) { return (int)((r & 0xFFFFFFFFull) % (unsigned long long)total); });
      if (qo >= 0) {
        const int op = lab[op_nodes[qo]];
        for (int e = t; e < n_edges; e += T) {
          const int lu = lab[esrc[e]];
          if (lab[edst[e]] == op && lu != op) mark[first[lu]] = 1;
        }
        __syncthreads();
        const int qp = select_kth(
            n_op, cnt, sel, [&](int q) { return mark[op_nodes[q]] != 0; },
            [&](int total) { return (int)((r >> 32) % (unsigned long long)total); });
        if (qp >= 0) {
          from = lab[op_nodes[qp]];
          to = op;
        }
      }
    } else {
      if (t == 0) {
        if (method == 0) {
          if (n_edges > 0) {
            const int k = (int)(r % (unsigned long long)n_edges);
            from = lab[esrc[k]];
            to = lab[edst[k]];
          }
        } else if (n_ar > 0) {
          const int pa = (int)(r % (unsigned long long)n_ar);
          const int side = ((r >> 32) & 1ull) ? 1 : -1;
          const int la = lab[ar_nodes[pa]];
          int pb = pa + side;
          while (pb >= 0 && pb < n_ar && lab[ar_nodes[pb]] == la) pb += side;
          if (pb >= 0 && pb < n_ar) {
            from = lab[ar_nodes[pb]];
            to = la;
          }
        }
        pair[0] = from;
        pair[1] = to;
      }
      __syncthreads();
      from = pair[0];
      to = pair[1];
    }
    if (from >= 0 && from != to)
      for (int v = t; v < N; v += T)
        if (lab[v] == from) lab[v] = (unsigned short)to;
    __syncthreads();
  }
  int* dst = children + (size_t)j * N;
  for (int v = t; v < N; v += T) dst[v] = lab[v];
}

// Copies the children that were kept into their pool slots: pair i = (child, slot).
__global__ __launch_bounds__(256) void keep_kernel(const int* __restrict__ children, int* __restrict__ pool, int N,
                                                    const int* __restrict__ pairs) {
  const int* src = children + (size_t)pairs[2 * blockIdx.x] * N;
  int* dst = pool + (size_t)pairs[2 * blockIdx.x + 1] * N;
  for (int v = threadIdx.x; v < N; v += blockDim.x) dst[v] = src[v];
}

__global__ void iota_kernel(int* p, int n, int mul) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i * mul;
}
__global__ void fill_kernel(int* p, int n, int v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

struct DevMem {
  std::vector<void*> ptrs;
  void* pinned = nullptr;
  ~DevMem() {
    for (void* p : ptrs) (void)hipFree(p);
    if (pinned) (void)hipHostFree(pinned);
  }
  template <typename T>
  T* take(size_t n, hipError_t* e) {
    void* p = nullptr;
    if (*e == hipSuccess) *e = hipMalloc(&p, (n ? n : 1) * sizeof(T));
    if (p) ptrs.push_back(p);
    return static_cast<T*>(p);
  }
};

}  // namespace

dc_status run_search(dc_ctx* ctx, const SearchView& g, int32_t graph, const dc_search_params& p, int32_t* labels_opt,
                     dc_search_result* res, hipStream_t s) {
  const int N = g.n, P = p.parents, C = 2 * P;
  // op-op dependencies in CSR order and all-reduce nodes in production order, built on the host
  std::vector<int> rp(N + 1), ci(g.e > 0 ? g.e : 1);
  std::vector<float> ar(N > 0 ? N : 1);
  hipError_t e = hipMemcpyAsync(rp.data(), g.rowptr, (N + 1) * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess && g.e > 0) e = hipMemcpyAsync(ci.data(), g.col, (size_t)g.e * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess && N > 0) e = hipMemcpyAsync(ar.data(), g.ar_size, (size_t)N * sizeof(float), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return DC_ERR_HIP;
  std::vector<int> esrc, edst, arn, opn;
  for (int u = 0; u < N; ++u) {
    if (ar[u] >= 0.0f) {
      arn.push_back(u);
      continue;
    }
    opn.push_back(u);
    for (int k = rp[u]; k < rp[u + 1]; ++k)
      if (ar[ci[k]] < 0.0f) {
        esrc.push_back(u);
        edst.push_back(ci[k]);
      }
  }
  const int slots = p.max_queue + C + 4;
  DevMem mem;
  int* d_esrc = mem.take<int>(esrc.size(), &e);
  int* d_edst = mem.take<int>(edst.size(), &e);
  int* d_arn = mem.take<int>(arn.size(), &e);
  int* d_opn = mem.take<int>(opn.size(), &e);
  int* pool = mem.take<int>((size_t)slots * N, &e);
  int* children = mem.take<int>((size_t)C * N, &e);
  int* d_parent = mem.take<int>(P, &e);
  int* d_pairs = mem.take<int>(2 * (size_t)(C + 1), &e);
  int* cand_graph = mem.take<int>(C, &e);
  int* cand_off = mem.take<int>(C + 1, &e);
  float* d_cost = mem.take<float>(C, &e);
  if (e == hipSuccess)
    e = hipHostMalloc(&mem.pinned, (size_t)C * sizeof(float) + ((size_t)P + 2 * (size_t)(C + 1)) * sizeof(int),
                      hipHostMallocDefault);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? DC_ERR_OOM : DC_ERR_HIP;
  }
  float* h_cost = static_cast<float*>(mem.pinned);
  int* h_parent = reinterpret_cast<int*>(h_cost + C);
  int* h_pairs = h_parent + P;
  if (!esrc.empty()) {
    e = hipMemcpyAsync(d_esrc, esrc.data(), esrc.size() * sizeof(int), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(d_edst, edst.data(), edst.size() * sizeof(int), hipMemcpyHostToDevice, s);
  }
  if (e == hipSuccess && !arn.empty()) e = hipMemcpyAsync(d_arn, arn.data(), arn.size() * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && !opn.empty()) e = hipMemcpyAsync(d_opn, opn.data(), opn.size() * sizeof(int), hipMemcpyHostToDevice, s);
  if (e != hipSuccess) return DC_ERR_HIP;
  const int op_draw = p.op_draw == DC_DRAW_OP ? 1 : 0;
  // labels as 16-bit values; the paper's op draw also keeps a 32-bit smallest member per label and a byte per node
  const size_t lds = (size_t)((N + 1) & ~1) * sizeof(unsigned short) + (op_draw ? (size_t)N * 5 + 4 : 0);
  if (lds > (size_t)kMutateLdsLimit) return DC_ERR_UNSUPPORTED;
  if (lds > 48 * 1024) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mutate_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds);
    if (e != hipSuccess) return DC_ERR_HIP;
  }
  hipLaunchKernelGGL(fill_kernel, dim3((C + 255) / 256), dim3(256), 0, s, cand_graph, C, graph);
  hipLaunchKernelGGL(iota_kernel, dim3((C + 1 + 255) / 256), dim3(256), 0, s, cand_off, C + 1, N);
  // slot 0: H_opt; slot 1: H_in (identity labels)
  std::vector<int> free_slots;
  for (int i = slots - 1; i >= 2; --i) free_slots.push_back(i);
  hipLaunchKernelGGL(iota_kernel, dim3((N + 255) / 256), dim3(256), 0, s, pool, N, 1);
  hipLaunchKernelGGL(iota_kernel, dim3((N + 255) / 256), dim3(256), 0, s, pool + (size_t)N, N, 1);
  auto cost_of = [&](const int* labels, int n) -> dc_status {
    dc_status st = dc_cost_candidates(ctx, n, cand_graph, cand_off, labels, p.ar_c, p.ar_d, d_cost, s);
    if (st != DC_OK) return st;
    if (hipMemcpyAsync(h_cost, d_cost, (size_t)n * sizeof(float), hipMemcpyDeviceToHost, s) != hipSuccess) return DC_ERR_HIP;
    return dc_check(ctx, s);                 // synchronises the stream
  };
  dc_status st = cost_of(pool + (size_t)N, 1);
  if (st != DC_OK) return st;
  const float cost_in = h_cost[0];
  float cost_opt = cost_in;
  typedef std::tuple<float, long long, int> Entry;   // cost, age, slot
  std::set<Entry> queue;
  queue.insert(Entry(cost_in, 0, 1));
  long long next_id = 1, step = 0, evaluated = 0, valid = 0, enqueued = 0, improved = 0;
  int unchanged = 0;
  std::vector<int> used;
  while (!queue.empty() && unchanged < p.max_unchanged && step < p.max_steps) {
    used.clear();
    while ((int)used.size() < P && !queue.empty()) {
      used.push_back(std::get<2>(*queue.begin()));
      queue.erase(queue.begin());
    }
    const int np = (int)used.size(), nc = 2 * np;
    for (int i = 0; i < np; ++i) h_parent[i] = used[i];
    if (hipMemcpyAsync(d_parent, h_parent, np * sizeof(int), hipMemcpyHostToDevice, s) != hipSuccess) return DC_ERR_HIP;
    hipLaunchKernelGGL(mutate_kernel, dim3(nc), dim3(256), lds, s, pool, d_parent, N, (int)esrc.size(), d_esrc, d_edst,
                       (int)arn.size(), d_arn, (int)opn.size(), d_opn, op_draw, (unsigned long long)p.seed,
                       (unsigned long long)step, p.beta, children);
    if (hipGetLastError() != hipSuccess) return DC_ERR_HIP;
    st = cost_of(children, nc);
    if (st != DC_OK) return st;
    // decisions first, on the host; the label vectors that are kept move afterwards in one launch.
    // A slot that is given up within the step (queue full) may be handed out again: its earlier
    // pair is then dropped, so that no two pairs write one slot.
    int n_pairs = 0, best_child = -1;
    for (int j = 0; j < nc; ++j) {
      const float c = h_cost[j];
      ++evaluated;
      if (!isfinite(c)) continue;
      ++valid;
      if (c < cost_opt) {
        cost_opt = c;
        ++improved;
        unchanged = 0;
        best_child = j;
      } else {
        ++unchanged;
      }
      if ((double)c <= (double)p.alpha * (double)cost_opt) {
        if (free_slots.empty()) {            // the queue is full: its most expensive entry makes room
          if (queue.empty()) return DC_ERR_CAPACITY;
          auto last = std::prev(queue.end());
          const int gone = std::get<2>(*last);
          for (int i = 0; i < n_pairs; ++i)
            if (h_pairs[2 * i + 1] == gone) {
              h_pairs[2 * i] = h_pairs[2 * (n_pairs - 1)];
              h_pairs[2 * i + 1] = h_pairs[2 * (n_pairs - 1) + 1];
              --n_pairs;
              break;
            }
          free_slots.push_back(gone);
          queue.erase(last);
        }
        const int slot = free_slots.back();
        free_slots.pop_back();
        h_pairs[2 * n_pairs] = j;
        h_pairs[2 * n_pairs + 1] = slot;
        ++n_pairs;
        queue.insert(Entry(c, next_id++, slot));
        ++enqueued;
      }
    }
    if (best_child >= 0) {                   // slot 0 holds H_opt
      h_pairs[2 * n_pairs] = best_child;
      h_pairs[2 * n_pairs + 1] = 0;
      ++n_pairs;
    }
    if (n_pairs > 0) {
      if (hipMemcpyAsync(d_pairs, h_pairs, 2 * (size_t)n_pairs * sizeof(int), hipMemcpyHostToDevice, s) != hipSuccess)
        return DC_ERR_HIP;
      hipLaunchKernelGGL(keep_kernel, dim3(n_pairs), dim3(256), 0, s, children, pool, N, d_pairs);
      if (hipGetLastError() != hipSuccess) return DC_ERR_HIP;
      // h_pairs is reused next step: the copy above must have been taken before then; the next
      // step synchronises on its costs before it writes h_pairs again
    }
    for (int i = 0; i < np; ++i) free_slots.push_back(used[i]);
    while ((long long)queue.size() > (long long)p.max_queue) {
      auto last = std::prev(queue.end());
      free_slots.push_back(std::get<2>(*last));
      queue.erase(last);
    }
    ++step;
  }
  if (labels_opt) {
    if (hipMemcpyAsync(labels_opt, pool, (size_t)N * sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess) return DC_ERR_HIP;
  }
  if (hipStreamSynchronize(s) != hipSuccess) return DC_ERR_HIP;
  if (res) {
    res->cost_in = cost_in;
    res->cost_opt = cost_opt;
    res->steps = step;
    res->evaluated = evaluated;
    res->valid = valid;
    res->enqueued = enqueued;
    res->improved = improved;
    res->queued = (int64_t)queue.size();
    res->unchanged = unchanged;
  }
  return DC_OK;
}

}  // namespace dc

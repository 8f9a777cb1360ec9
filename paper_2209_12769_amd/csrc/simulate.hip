// End-to-end time of a candidate module by list scheduling (Sec. 3.4; gfx950).
//
// Computation ops run one at a time on one device in the order of a FIFO ready queue (an
// op enters the tail when its last dependency clears; it starts when the device is free
// and its predecessors are done).  All-reduce instructions run one at a time on a
// communication channel, in the order in which their tensors are produced, each starting
// when its tensor is produced and the channel is clear, for T = C x + D (Sec. 3.1,
// Profiler); they overlap with computation.  The result is the later of the two ends.
// Where the text is silent: the queue starts with the source ops in ascending index; an
// all-reduce goes on the channel the moment its last predecessor is processed, before the
// next op is taken, ties in ascending index; successors are released in ascending index;
// a module whose graph has a cycle (an invalid fusion) costs +infinity.
//
// The walk over one module is a serial chain, so the batch supplies the parallelism: one
// wave per candidate, with the whole module (successor lists, durations, dependency
// counters, ready times, both queues) in LDS; the lanes release the successors of the
// current node together (lists are duplicate free, so no two lanes touch one node) and
// append the newly ready ones in lane order = ascending index.  Modules too large for LDS
// keep the same arrays in a slice of global memory.  Times are fp64, added in the order
// the rules fix, so the result does not depend on the implementation.
#include <math.h>

#include <mutex>

#include "common.h"

namespace dc {
namespace {

// The arrays of a module in global memory ...
__host__ __device__ inline size_t sim_bytes(long long G, long long E) {
  // ready[G] f64 | val[G] f32 | dep[G] i32 | queue[G] i32 | rp[G+1] i32 | ci[E] u16 (padded to 8 bytes)
  return (size_t)G * (8 + 4 + 4 + 4) + (size_t)(G + 1) * 4 + (((size_t)E * 2 + 7) & ~(size_t)7) + 8;
}
// ... and in LDS, where a byte saved is a module more per CU: dependency counters and queue entries of 16 bits
// (a module has fewer than 65536 nodes; the counter keeps bit 15 for the all-reduce flag, so it takes modules
// of up to 32768 nodes, more than LDS holds anyway).
__host__ __device__ inline size_t sim_lds_bytes(long long G, long long E) {
  // ready[G] f64 | val[G] f32 | rp[G+1] i32 | dep[G] u16 | queue[G] u16 | ci[E] u16 (padded to 8 bytes)
  if (G > 32768) return ~(size_t)0;
  return (size_t)G * (8 + 4) + (size_t)(G + 1) * 4 + (((size_t)G * 4 + (size_t)E * 2 + 7) & ~(size_t)7) + 8;
}
template <bool kLds>
struct SimTypes {                 // global memory
  typedef int dep_t;
  typedef int q_t;
  static constexpr int kAr = 1 << 30;      // flag in the dependency counter: the node is an all-reduce
};
template <>
struct SimTypes<true> {           // LDS
  typedef unsigned short dep_t;
  typedef unsigned short q_t;
  static constexpr int kAr = 1 << 15;
};

extern __shared__ __attribute__((aligned(16))) char dc_sim_smem[];

// The workgroup is one wave.  LDS operations of a wave are carried out in issue order, so
// between a lane's write and another lane's later read only the compiler has to be kept from
// reordering; global memory needs the writes to have completed.
template <bool kLds>
__device__ __forceinline__ void sync_wave() {
  if (kLds) __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  else __syncthreads();
}

template <bool kLds>
__global__ __launch_bounds__(64) void simulate_kernel(const int* __restrict__ node_off,
                                                       const int* __restrict__ out_rp, const int* __restrict__ out_ci,
                                                       const int* __restrict__ in_rp,
                                                       const float* __restrict__ op_time,
                                                       const float* __restrict__ ar_size, int C, float ar_c,
                                                       float ar_d, float* __restrict__ cost, char* gscratch,
                                                       size_t gstride, int lds_lo, int lds_hi, int* status) {
  // kLds: this launch walks the modules whose arrays need more than lds_lo and at most lds_hi
  // bytes (its LDS allocation); !kLds: those that need more than lds_hi, in global memory
  typedef typename SimTypes<kLds>::dep_t dep_t;
  typedef typename SimTypes<kLds>::q_t q_t;
  constexpr int kAr = SimTypes<kLds>::kAr;
  if (status[0] != 0) return;
  const int lane = threadIdx.x;
  for (int c = blockIdx.x; c < C; c += gridDim.x) {
    const int n0 = node_off[c], G = node_off[c + 1] - n0;
    const int e0 = out_rp[n0], E = out_rp[n0 + G] - e0;
    const size_t need = sim_lds_bytes(G, E);
    if (kLds ? (need <= (size_t)lds_lo || need > (size_t)lds_hi) : need <= (size_t)lds_hi) continue;
    if (!kLds && sim_bytes(G, E) > gstride) {       // larger than any base graph of this context
      if (lane == 0) {
        set_error(status, (int)DC_ERR_CAPACITY);
        cost[c] = INFINITY;
      }
      continue;
    }
    char* base = kLds ? dc_sim_smem : gscratch + (size_t)blockIdx.x * gstride;
    double* ready = reinterpret_cast<double*>(base);
    float* val = reinterpret_cast<float*>(ready + G);      // execution time, or tensor size of an all-reduce
    dep_t* dep;
    q_t* qu;                 // every node is queued once: ops fill it from the front, all-reduces from the back
    int* rp;
    unsigned short* ci;
    if (kLds) {
      rp = reinterpret_cast<int*>(val + G);
      dep = reinterpret_cast<dep_t*>(rp + G + 1);
      qu = reinterpret_cast<q_t*>(dep + G);
      ci = reinterpret_cast<unsigned short*>(qu + G);
    } else {
      dep = reinterpret_cast<dep_t*>(val + G);
      qu = reinterpret_cast<q_t*>(dep + G);
      rp = reinterpret_cast<int*>(qu + G);
      ci = reinterpret_cast<unsigned short*>(rp + G + 1);
    }
    const double dc = (double)ar_c, dd = (double)ar_d;

    // ---- load the module
    for (int v = lane; v < G; v += 64) {
      const float x = ar_size[n0 + v];
      const bool ar = x >= 0.0f;
      ready[v] = 0.0;
      val[v] = ar ? x : op_time[n0 + v];
      dep[v] = (dep_t)((in_rp[n0 + v + 1] - in_rp[n0 + v]) | (ar ? kAr : 0));
      rp[v] = out_rp[n0 + v] - e0;
    }
    if (lane == 0) rp[G] = E;
    for (int k = lane; k < E; k += 64) ci[k] = (unsigned short)(out_ci[e0 + k] - n0);
    sync_wave<kLds>();

    // ---- sources, in ascending index, onto the two queues
    int qt = 0, at = 0;                   // entries queued so far (wave-uniform)
    for (int v0 = 0; v0 < G; v0 += 64) {
      const int v = v0 + lane;
      const int d = v < G ? dep[v] : 1;
      const bool src_op = d == 0, src_ar = d == kAr;
      const unsigned long long mo = __ballot(src_op), ma = __ballot(src_ar);
      const unsigned long long below = (1ull << lane) - 1ull;
      if (src_op) qu[qt + __popcll(mo & below)] = (q_t)v;
      if (src_ar) qu[G - 1 - (at + __popcll(ma & below))] = (q_t)v;
      qt += __popcll(mo);
      at += __popcll(ma);
    }
    sync_wave<kLds>();

    // ---- the walk
    int qh = 0, ah = 0, processed = 0;
    double dev = 0.0, chan = 0.0;
    while (ah < at || qh < qt) {
      int u;
      double done;
      if (ah < at) {                      // tensors already produced go on the channel first
        u = qu[G - 1 - ah++];
        const double r = ready[u];
        done = (r > chan ? r : chan) + (dc * (double)val[u] + dd);
        chan = done;
      } else {
        u = qu[qh++];
        const double r = ready[u];
        done = (r > dev ? r : dev) + (double)val[u];
        dev = done;
      }
      ++processed;
      const int s = rp[u], e = rp[u + 1];
      for (int k0 = s; k0 < e; k0 += 64) {
        const int k = k0 + lane;
        bool new_op = false, new_ar = false;
        int w = 0;
        if (k < e) {
          w = ci[k];
          if (done > ready[w]) ready[w] = done;
          const int d = (int)dep[w] - 1;
          dep[w] = (dep_t)d;
          new_op = d == 0;
          new_ar = d == kAr;
        }
        const unsigned long long mo = __ballot(new_op), ma = __ballot(new_ar);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (new_op) qu[qt + __popcll(mo & below)] = (q_t)w;
        if (new_ar) qu[G - 1 - (at + __popcll(ma & below))] = (q_t)w;
        qt += __popcll(mo);
        at += __popcll(ma);
      }
      sync_wave<kLds>();                  // the releases are visible before the next node is taken
    }
    if (lane == 0) cost[c] = processed == G ? (float)(dev > chan ? dev : chan) : INFINITY;
    sync_wave<kLds>();
  }
}

}  // namespace

size_t simulate_scratch_bytes(long long max_graph_nodes, long long max_graph_edges, int n_slices) {
  return sim_bytes(max_graph_nodes, max_graph_edges) * (size_t)n_slices;
}

hipError_t launch_simulate(const SimArgs& a, hipStream_t s) {
  if (a.n_cand <= 0) return hipSuccess;
  // Modules are walked on chip in five launches by size class, each with just the LDS its class
  // needs (10, 6, 4, 3 or 2 waves per CU of 160 KB); a workgroup whose candidate belongs to another
  // class returns at once.  The rest walk in slices of global memory (a persistent grid).
  constexpr int kClasses = 5;
  int classes[kClasses + 1] = {0, 16 * 1024, 26 * 1024 + 512, 40 * 1024, 53 * 1024, a.lds_bytes};
  for (int k = 1; k < kClasses; ++k) classes[k] = classes[k] < a.lds_bytes ? classes[k] : a.lds_bytes;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&simulate_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, a.lds_bytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  for (int k = 0; k < kClasses; ++k)
    if (classes[k + 1] > classes[k])
    hipLaunchKernelGGL(simulate_kernel<true>, dim3(a.n_cand), dim3(64), classes[k + 1], s, a.node_off, a.out_rowptr,
                       a.out_col, a.in_rowptr, a.op_time, a.ar_size, a.n_cand, a.ar_c, a.ar_d, a.cost, nullptr,
                       (size_t)0, classes[k], classes[k + 1], a.status);
  if (a.n_slices > 0)
    hipLaunchKernelGGL(simulate_kernel<false>, dim3(a.n_slices), dim3(64), 0, s, a.node_off, a.out_rowptr, a.out_col,
                       a.in_rowptr, a.op_time, a.ar_size, a.n_cand, a.ar_c, a.ar_d, a.cost, a.scratch, a.scratch_stride,
                       0, a.lds_bytes, a.status);
  return hipGetLastError();
}

// ---- the simulator for callers that cannot allocate ------------------------------------------------
namespace {

constexpr int kStaticLdsBytes = 80 * 1024;              // modules up to this size are walked in LDS
constexpr int kStaticSlices = 64;                       // workgroups of the global-memory walk
constexpr size_t kStaticSliceBytes = 256 * 1024;        // working set of the largest module accepted
constexpr size_t kStaticHeaderBytes = 256;              // status words
// Device memory of the library itself: the status words and the slices of the global-memory walk.
// In host code this name only stands for the symbol; the address on each device comes from
// hipGetSymbolAddress (static_scratch below) and is what every kernel and launch receives.
static __device__ __align__(256) char dc_sim_static_scratch[kStaticHeaderBytes + kStaticSlices * kStaticSliceBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
char* g_static_ptr[kMaxDevices] = {};
int g_static_cus[kMaxDevices] = {};

// The scratch array's address on the current device (every device holds its own copy), looked up once.
hipError_t static_scratch(char** ptr, int* n_cu) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(dc_sim_static_scratch));
    if (e != hipSuccess) return e;
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    g_static_cus[dev] = cus > 0 ? cus : 1;
    g_static_ptr[dev] = static_cast<char*>(p);
  }
  *ptr = g_static_ptr[dev];
  *n_cu = g_static_cus[dev];
  return hipSuccess;
}

__global__ void export_status_kernel(const int* __restrict__ status, int* __restrict__ out) { out[0] = status[0]; }

thread_local const char* t_static_error = "";

}  // namespace
}  // namespace dc

extern "C" dc_status dc_simulate_static(const dc_batch* in, int32_t max_module_nodes, int32_t max_module_edges,
                                        const float* op_time, const float* ar_size, float ar_c, float ar_d, float* cost,
                                        int32_t* dev_status, void* stream) {
  using namespace dc;
  t_static_error = "";
  if (!in || in->n_cand < 0 || max_module_nodes < 0 || max_module_edges < 0) {
    t_static_error = "null batch or negative size";
    return DC_ERR_INVALID_ARG;
  }
  if (in->n_cand == 0) return DC_OK;
  if (!cost || !op_time || !ar_size || !in->node_off || !in->out_rowptr || !in->out_col || !in->in_rowptr || !in->in_col) {
    t_static_error = "null array";
    return DC_ERR_INVALID_ARG;
  }
  if (max_module_nodes >= 65536) {
    t_static_error = "a module has fewer than 65536 nodes";
    return DC_ERR_CAPACITY;
  }
  if (sim_bytes(max_module_nodes, max_module_edges) > kStaticSliceBytes) {
    t_static_error = "the largest module needs more than the 256 KiB working set this entry point holds: "
                     "24 bytes per node + 2 bytes per edge; use dc_simulate";
    return DC_ERR_CAPACITY;
  }
  char* scratch = nullptr;
  int n_cu = 0;
  hipError_t e = static_scratch(&scratch, &n_cu);
  if (e != hipSuccess) {
    t_static_error = hipGetErrorString(e);
    return DC_ERR_HIP;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  int* status = reinterpret_cast<int*>(scratch);
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, status);          // a fill kernel, not a memset
  launch_check_batch(in->node_off, in->n_cand, (long long)in->cap_nodes, (long long)in->cap_edges, in->out_rowptr,
                     in->out_col, in->in_rowptr, in->in_col, status, n_cu, s);
  SimArgs a;
  a.n_cand = in->n_cand;
  a.node_off = in->node_off;
  a.out_rowptr = in->out_rowptr;
  a.out_col = in->out_col;
  a.in_rowptr = in->in_rowptr;
  a.op_time = op_time;
  a.ar_size = ar_size;
  a.ar_c = ar_c;
  a.ar_d = ar_d;
  a.cost = cost;
  a.lds_bytes = kStaticLdsBytes;
  a.scratch = scratch + kStaticHeaderBytes;
  a.scratch_stride = kStaticSliceBytes;
  a.n_slices = kStaticSlices;
  a.status = status;
  e = launch_simulate(a, s);
  if (e == hipSuccess && dev_status) {
    hipLaunchKernelGGL(export_status_kernel, dim3(1), dim3(1), 0, s, status, dev_status);
    e = hipGetLastError();
  }
  if (e != hipSuccess) {
    t_static_error = hipGetErrorString(e);
    return DC_ERR_HIP;
  }
  return DC_OK;
}

extern "C" const char* dc_simulate_static_error(void) { return dc::t_static_error; }

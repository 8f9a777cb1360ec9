// Internal declarations shared by the HIP sources of libdisco (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "disco.h"

namespace dc {

// Device status words: [0] first error of the running call (later kernels of the
// call read it and return without writing), [1] first error since dc_check.
__device__ __forceinline__ void set_error(int* status, int code) {
  atomicCAS(&status[0], 0, code);
  atomicCAS(&status[1], 0, code);
}

// Base graphs as the kernels see them (device pointers).
struct BaseGraphs {
  int n_graphs;
  const int* gno;      // [n_graphs+1] node offsets
  const int* geo;      // [n_graphs+1] edge offsets
  const int* rowptr;   // successors: graph b at gno[b] + b, N_b+1 local entries
  const int* col;      // graph b at geo[b], local node numbers
  const int* crowptr;  // predecessors, same layout
  const int* ccol;
  const float* X;      // [sum N_b, F]
};

// Scratch written by the per-candidate contraction kernel and consumed by the
// finalise kernel.  Node-indexed arrays use slot cand_off[c] + c (one extra
// entry per candidate), edge-indexed arrays use slot tmp_eoff[c].
struct ContractTmp {
  int* tmp_eoff;   // [C+1] exclusive scan of base edge counts
  int* members;    // [sum N] base nodes grouped by contracted node, ascending inside a group
  int* mstart;     // [sum N + C] start of each group in members (G+1 entries per candidate)
  int* orp;        // [sum N + C] local out rowptr (G+1 entries)
  int* irp;        // [sum N + C] local in rowptr
  int* oc;         // [sum E] local out columns
  int* ic;         // [sum E] local in columns
  int* Gc;         // [C] contracted node count
  int* Ec;         // [C] contracted edge count
  int* big_order;  // [C] the candidates whose base graph does not fit LDS, largest working sets first
  int* big_meta;   // [0] how many of them, [1] the counter that hands them out
};

struct BatchView {
  int* node_off;
  int* edge_off;
  int* new_id;
  int* out_rowptr;
  int* out_col;
  int* in_rowptr;
  int* in_col;
  void* Xc;
  long long cap_nodes;
  long long cap_edges;
};

// Optional per-kernel timing with HIP events on the launch stream.
enum Family { kFamPrep = 0, kFamContract, kFamFinalize, kFamAggregate, kFamUpdate, kFamFused, kFamLayer256, kFamLayer64, kFamHeavy, kFamDesc, kFamAttProject, kFamAttScores, kFamAttAggregate, kFamReadout, kFamSimulate, kFamFusedOps, kFamFusedHead, kFamTrainAggregate, kFamTrainUpdate, kFamTrainHead, kFamTrainWgrad, kFamTrainDgrad, kFamTrainGatherBack, kFamTrainAdam, kFamCount };
struct Profiler {
  bool on = false;
  static constexpr int kCap = 4096;
  hipEvent_t ev[2 * kCap];
  int fam[kCap];
  int n = 0;
  int created = 0;
  void begin(int family, hipStream_t s);
  void end(hipStream_t s);
};

struct ContractLaunch {
  BaseGraphs bg;
  int max_graph_nodes, max_graph_edges;   // largest base graph
  int min_graph_need;                      // smallest per-graph working-set bytes
  int n_cand;
  const int* cand_graph;
  const int* cand_off;
  const int* group_id;
  ContractTmp tmp;
  BatchView out;
  int F, bf16;
  long long max_base_nodes, max_base_edges;
  int* status;
  int* totals;       // [2] contracted nodes, edges of this call
  char* slab;        // global working sets for graphs that do not fit in LDS
  size_t slab_stride;
  int slab_wgs;
  int lds_limit;
};
hipError_t launch_contract(const ContractLaunch& a, Profiler* prof, hipStream_t s);
int contract_working_set_bytes(int n_nodes, int n_edges);
hipError_t contract_set_lds_limit(int bytes);

// ints of the pre-pass's work counters: one counter per XCD, each on a cache line of its own
constexpr int kHeavyCtrInts = 8 * 32;

struct GnnArgs {
  int n_cand;
  const int* node_off;
  const int* out_rowptr;
  const int* out_col;
  const int* in_rowptr;
  const int* in_col;
  const void* Xc;
  int F, H, L, bf16;
  const void* W;        // layer matrices in device layout
  const float* b;       // biases fp32
  const float* head;    // fp32 head (bf16-representable matrices on the bf16 path)
  void* act[2];         // ping/pong activations [max_nodes, H]
  void* agg[2];         // predecessor mean / successor mean [max_nodes, max(F,H)]
  void* desc[2];        // gather descriptors [max_nodes] x 16 bytes per direction
  int* heavy[2] = {nullptr, nullptr};   // per direction and tile of 128 rows: the rows with long lists (128 places per tile)
  int* heavy_cnt = nullptr;             // [2 * tiles] how many of them: entry 2 * tile + direction
  int* heavy_off = nullptr;             // [2 * tiles + 1] exclusive scan of heavy_cnt
  unsigned* heavy_list = nullptr;       // the long rows of all tiles as one list: row number, bit 31 = successors' side
  int* heavy_ctr = nullptr;             // [kHeavyCtrInts] the pre-pass's work counters, one per XCD (cleared by every launch)
  // the last layer forming the readout's sums itself (bulk bf16 shapes): per chunk of 64 rows and graph one row of
  // H partial sums at row chunk + graph, and per chunk the graph its first row belongs to; 0 / nullptr: not used
  int fuse_readout = 0;
  float* ro_part = nullptr;             // [max_nodes / 64 + max_cand + 2][H]
  int* ro_first = nullptr;              // [max_nodes / 64 + 2]
  float* pred;
  const int* status;
  int n_cu;
  int allow_fused;      // 0 forces the separate aggregate + update kernels
  // attention aggregation (heads > 0): W holds one [d, H] block per layer
  int heads = 0;
  const float* att = nullptr;   // per layer a_src[H] | a_dst[H]
  float* score[2] = {nullptr, nullptr};   // per node and head: a_src . z, a_dst . z  [max_nodes, heads]
};
hipError_t launch_gnn_forward(const GnnArgs& a, Profiler* prof, hipStream_t s);
// The message-passing layers alone; *h_last receives the final embeddings [node_off[n_cand], H].
hipError_t launch_gnn_layers(const GnnArgs& a, Profiler* prof, hipStream_t s, const void** h_last);
// out = ReLU(A Wp + bias) for the node_off[n_cand] rows of A [rows, d]; Wp in the device layout of one layer block.
void launch_dense_bias_relu(const GnnArgs& a, const void* A, int d, const void* Wp, const float* bias, void* out,
                            hipStream_t s);
// The two neighbour means of every row of h [rows, d] (separate kernel; any d that is a multiple of 16 bytes).
void launch_mean_aggregate(const GnnArgs& a, const void* h, int d, void* h_in, void* h_out, hipStream_t s);
// out [rows, a.H] = [A0 | A1 | A2] Wl (nseg = 3) or A0 Wl (nseg = 1), rows = a.node_off[a.n_cand]; with a bias
// the result is ReLU(. + bias), without one it is stored as it is.  a.H must be a multiple of 32.
void launch_dense_update(const GnnArgs& a, const void* A0, const void* A1, const void* A2, int d, int nseg,
                         const void* Wl, const float* bias, void* out, hipStream_t s);
// Elements (of the storage dtype) of all layer matrices in device layout; nseg row blocks of
// d rows per layer (3: self / predecessor mean / successor mean; 1: attention).
size_t packed_weight_elems(int F, int H, int L, int nseg);
// Host side: converts row-major fp32 W^l into the device layout of the dtype
// (fp32: unchanged; bf16: [k/8][H][8] so that a lane's 8 consecutive k sit together).
void pack_weights_host(const float* W_layers, int F, int H, int L, int nseg, int bf16, void* dst);
// gnn_attention.hip: per-node score terms from z, then softmax-weighted sums over N_i
bool attention_shape_supported(int H, int heads);
hipError_t launch_attention_scores(const GnnArgs& a, const void* z, const float* att_l, hipStream_t s);
hipError_t launch_attention_aggregate(const GnnArgs& a, const void* z, const float* bias, void* out, hipStream_t s);
bool gnn_shape_supported(int F, int H, int L);
// gnn_fused.hip: one layer with both neighbour means folded into the A-tile load (bf16).
bool fused_layer_supported(int d, int H, int bf16);
hipError_t launch_fused_layer(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                              hipStream_t s);

// gnn_layer256.hip: wave-specialised fused layer for H = 256, d = 256 or 64 (bf16); uses a.agg[] for rows with long lists.
bool layer256_supported(int d, int H, int bf16);
hipError_t launch_build_desc(const GnnArgs& a, hipStream_t s);
// readout: the layer leaves the readout's chunk sums in a.ro_part instead of its rows in out (needs
// launch_chunk_first on the same batch before)
hipError_t launch_layer256(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                           bool readout, Profiler* prof, hipStream_t s);
hipError_t launch_chunk_first(const GnnArgs& a, hipStream_t s);
// gnn_layer256w.hip: the same layer (five gather slots) with sixteen waves per workgroup; descriptors and
// pre-pass means as for launch_layer256
hipError_t launch_build_desc_sorted(const GnnArgs& a, hipStream_t s);
// Means of the rows with more than five neighbours (listed by launch_build_desc_sorted), written at the rows'
// own places in a.agg[0] (predecessors) and a.agg[1] (successors); h [rows, d], d = 256 or 64, bf16.
hipError_t launch_heavy_means(const void* h, int d, const GnnArgs& a, hipStream_t s);
hipError_t launch_layer256w(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                            bool readout, hipStream_t s);
hipError_t launch_dense256(const void* h, int d, const GnnArgs& a, const void* Wl, const float* bias, void* out,
                           hipStream_t s);

// simulate.hip: list-scheduling estimate of the end-to-end time of each candidate module
struct SimArgs {
  int n_cand;
  const int* node_off;
  const int* out_rowptr;
  const int* out_col;
  const int* in_rowptr;
  const float* op_time;     // [Ntot] execution time of computation nodes
  const float* ar_size;     // [Ntot] tensor size of all-reduce nodes, negative for computation nodes
  float ar_c, ar_d;         // T = ar_c * size + ar_d
  float* cost;              // [n_cand]
  int lds_bytes;            // LDS per wave for modules walked on chip
  char* scratch;            // slices of global memory for the others
  size_t scratch_stride;
  int n_slices;
  int* status;
};
size_t simulate_scratch_bytes(long long max_graph_nodes, long long max_graph_edges, int n_slices);
hipError_t launch_simulate(const SimArgs& a, hipStream_t s);

// fused_ops.hip: the batch of fused-op subgraphs of the candidates just contracted, and the
// per-node times the simulator takes
struct FusedOpsArgs {
  BaseGraphs bg;
  const float* op_time_base;   // [sum N_b] profiled time of each op
  const float* ar_size_base;   // [sum N_b] tensor size of each all-reduce node, negative for ops
  int n_cand;
  const int* cand_graph;
  const int* cand_off;
  const int* members;          // left by the contraction: base nodes grouped by contracted node
  const int* mstart;           // start of each group in members (slot cand_off[c] + c)
  const int* Gc;               // contracted node count per candidate
  const int* new_id;           // contracted node (local) of each base node
  const int* c_node_off;       // [C+1] contracted node offsets
  // scratch, slot cand_off[c] + c with one extra entry per candidate
  int* gfm;                    // per group: rows of fused ops before it (local)
  int* gfk;                    // per group: fused ops before it (local)
  int* dgo;                    // per member position: edges inside groups before it, successors
  int* dgi;                    // the same, predecessors
  int* cnt;                    // [3][C+1] fused ops / rows / edges per candidate, scanned in place
  int* totals;                 // {0, rows} {0, fused ops} edges, [5] fused ops that repeat an earlier one
  BatchView fb;                // one graph per fused op; new_id holds the base node of each row
  int* fo_cnode;               // contracted node (global) of each fused op
  // Fused ops with the same members in the same base graph have the same subgraph and hence the same
  // estimate: with a table (not null) the estimator runs on the first of each kind only
  int* table;                  // [table_mask + 1] open addressing, entry = contracted node (global) of that first one, -1 = free
  unsigned table_mask;
  int* dup_of;                 // slot cand_off[c] + c, per group: the contracted node (global) it repeats, or -1
  long long cap_ops, cap_rows, cap_edges;
  float* op_time;              // [contracted nodes] out
  float* ar_size;              // [contracted nodes] out
  int F, H, bf16;
  int* status;
  int n_cu;
};
hipError_t launch_fused_op_extract(const FusedOpsArgs& a, Profiler* prof, hipStream_t s);
hipError_t launch_fused_op_readout(const FusedOpsArgs& a, const void* h_last, void* R, hipStream_t s);
hipError_t launch_fused_op_times(const FusedOpsArgs& a, const void* Z2, const float* w3b3, float* fo_pred,
                                 hipStream_t s);
size_t fused_op_table_entries(long long max_fused_ops);

// search.hip: the backtracking search driver; it sees one base graph and calls the public cost entry point
struct SearchView {
  const int* rowptr;     // device, N + 1 local entries
  const int* col;        // device, local node numbers
  const float* ar_size;  // device [N], negative for computation ops
  int n, e;
};
dc_status run_search(dc_ctx* ctx, const SearchView& g, int32_t graph, const dc_search_params& p, int32_t* labels_opt,
                     dc_search_result* res, hipStream_t s);

// train.hip: one pass of supervised training of the estimator (fp32): forward with kept activations,
// loss, reverse pass into one gradient vector laid out W_layers | b_layers | head; Adam.
struct TrainPass {
  // the batch of sample graphs
  int n_samples;               // host-known number of graphs
  const int* node_off;         // [n_samples + 1]
  const int* out_rowptr;
  const int* out_col;
  const int* in_rowptr;
  const int* in_col;
  const float* X;              // [rows, F]
  const float* target;         // [n_samples]
  // parameters (row-major fp32)
  const float* W;
  const float* b;
  const float* head;
  int F, H, L;
  float floor;
  // buffers
  float* hs;                   // [L][max_rows, H] activations after each layer
  float* means;                // [L][2][max_rows, max(F,H)] predecessor mean, successor mean of every layer's input
  float* dZ[2];                // [max_rows, H] gradient at the pre-activations, ping-pong
  float* dA;                   // [max_rows, 3H]
  float* R;                    // [max_samples, H] each: R, Z1, Z2, dZ2, dZ1, dR
  float* Z1;
  float* Z2;
  float* dZ2;
  float* dZ1;
  float* dR;
  float* y;                    // [max_samples]
  float* dy;
  double* lterm;               // [max_samples] per-sample loss terms
  int* gid;                    // [max_rows] sample of each row
  int* cnt;                    // {0, n_samples}
  float* WT;                   // [H, 3H] transposed matrix of the layer at hand
  float* part;                 // [slabs][3 max(F,H) H + H] partial sums of the weight gradients
  int slabs;
  long long max_rows;
  float* grad;                 // [n_params]
  float* loss;                 // [1]
  float* pred;                 // [n_samples] or null
  int* status;
  int n_cu;
};
hipError_t launch_train_pass(const TrainPass& t, Profiler* prof, hipStream_t s);
int train_slabs(int n_cu, int F, int H);
hipError_t launch_adam(float* theta, const float* grad, float* m, float* v, long long n, float lr, float beta1,
                       float beta2, float eps, double c1, double c2, const int* status, hipStream_t s);

__global__ void reset_status_kernel(int* status);
// Device-side validation of a caller's batch (sizes within the capacities, graphs below 65536 nodes, row
// pointers ascending, neighbours inside their own graph); sets the status word on a violation.
void launch_check_batch(const int* node_off, int n_cand, long long max_nodes, long long cap_edges, const int* out_rp,
                        const int* out_ci, const int* in_rp, const int* in_ci, int* status, int n_cu, hipStream_t s);

// fp32 -> bf16, round to nearest even, in hardware (v_cvt_pk_bf16_f32): a in the low half
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ unsigned short to_bf16(float a) { return (unsigned short)(pack_bf16x2(a, 0.f) & 0xFFFFu); }

// Adds the two bf16 values packed in x to the fp32 accumulators (lo half -> lo, hi half
// -> hi), each scaled by the bf16 factor `one` (1.0 = 0x3F80 to add, 0 to skip), with one
// V_DOT2C_F32_BF16 per half: acc + x.lo*one + x.hi*0.  The products are exact; the
// hardware's final add may differ from an IEEE round-to-nearest add by one fp32 ulp,
// so every kernel that forms a neighbour sum uses this one helper.  The factor must live
// in a register: the assembler folds the constant 0x3F80 into the inline operand "1.0",
// which this instruction does not read as a packed bf16 pair (checked on the device).
__device__ __forceinline__ unsigned bf16_one_reg() {
  unsigned k;
  asm volatile("v_mov_b32 %0, 0x3f80" : "=v"(k));
  return k;
}
__device__ __forceinline__ void bf16_pair_add(float& lo, float& hi, unsigned x, unsigned one) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t v = __builtin_bit_cast(bf16x2_t, x);
  lo = __builtin_amdgcn_fdot2_f32_bf16(v, __builtin_bit_cast(bf16x2_t, one), lo, false);
  hi = __builtin_amdgcn_fdot2_f32_bf16(v, __builtin_bit_cast(bf16x2_t, one << 16), hi, false);
}

__device__ __forceinline__ int wave_incl_scan(int x) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  return x;
}

// Exclusive scan of in[0..n) into out[0..n) (may alias) by the whole workgroup;
// returns the total.  Each thread owns a contiguous chunk.  Ends with a barrier.
__device__ __forceinline__ int block_exscan(const int* in, int* out, int n, int* wsum) {
  const int t = threadIdx.x, T = blockDim.x;
  const int K = (n + T - 1) / T;
  const int lo = min(t * K, n), hi = min(lo + K, n);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += in[i];
  const int inc = wave_incl_scan(s);
  if ((t & 63) == 63) wsum[t >> 6] = inc;
  __syncthreads();
  int woff = 0, total = 0;
  const int nw = T >> 6;
  for (int i = 0; i < nw; ++i) {
    int x = wsum[i];
    if (i < (t >> 6)) woff += x;
    total += x;
  }
  int run = woff + inc - s;
  for (int i = lo; i < hi; ++i) {
    int x = in[i];
    out[i] = run;
    run += x;
  }
  __syncthreads();
  return total;
}

// The same scan for arrays in global memory: rounds of four neighbouring entries per thread, so that a wave reads
// and writes whole cache lines (a contiguous run per thread touches a line per entry).  blockDim.x <= 1024.
__device__ __forceinline__ int block_exscan_lines(const int* in, int* out, int n, int* wsum) {
  const int t = threadIdx.x, T = blockDim.x, lane = t & 63, wave = t >> 6, nw = T >> 6;
  int carry = 0;
  for (int i0 = 0; i0 < n; i0 += 4 * T) {
    const int i = i0 + 4 * t;
    int x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) x[k] = i + k < n ? in[i + k] : 0;
    const int s = x[0] + x[1] + x[2] + x[3];
    const int inc = wave_incl_scan(s);
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    int before = carry;
    for (int w = 0; w < nw; ++w) {
      const int ws = wsum[w];
      if (w < wave) before += ws;
      carry += ws;
    }
    int run = before + inc - s;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (i + k < n) out[i + k] = run;
      run += x[k];
    }
    __syncthreads();
  }
  return carry;
}

static inline __host__ __device__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace dc

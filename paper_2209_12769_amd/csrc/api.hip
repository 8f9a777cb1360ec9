// C ABI of libdisco: context, argument checks, memory, launches (gfx950 only).
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <string>
#include <vector>

#include "common.h"

using namespace dc;

namespace dc {
void Profiler::begin(int family, hipStream_t s) {
  if (!on || n >= kCap) return;
  while (created < 2 * (n + 1)) {
    if (hipEventCreate(&ev[created]) != hipSuccess) return;
    ++created;
  }
  fam[n] = family;
  (void)hipEventRecord(ev[2 * n], s);
}
void Profiler::end(hipStream_t s) {
  if (!on || n >= kCap || created < 2 * (n + 1)) return;
  (void)hipEventRecord(ev[2 * n + 1], s);
  ++n;
}
}  // namespace dc

struct dc_ctx {
  dc_config cfg;
  int device = 0;
  int n_cu = 256;
  int lds_limit = 64 * 1024;
  // one device arena for all scratch
  char* arena = nullptr;
  size_t arena_bytes = 0;
  ContractTmp tmp{};
  BatchView ib{};           // context-owned batch used by dc_eval_candidates
  void* act[2] = {nullptr, nullptr};
  void* agg[2] = {nullptr, nullptr};
  void* desc[2] = {nullptr, nullptr};
  int* heavy[2] = {nullptr, nullptr};
  int* heavy_cnt = nullptr;
  int* heavy_ctr = nullptr;
  int* heavy_off = nullptr;
  unsigned* heavy_list = nullptr;
  float* ro_part = nullptr; // chunk sums of the readout when the last layer forms them
  int* ro_first = nullptr;
  int* status = nullptr;    // [2]
  int* totals = nullptr;    // [2]
  int* h_pinned = nullptr;  // [4] pinned host mirror for status / totals
  // weights
  void* W = nullptr;
  float* b = nullptr;
  float* head = nullptr;
  float* att = nullptr;     // attention vectors (DC_AGG_ATTENTION only)
  float* score[2] = {nullptr, nullptr};
  bool have_weights = false;
  // base graphs
  BaseGraphs bg{};
  char* bg_mem = nullptr;
  int max_gn = 0, max_ge = 0, min_need = 0;
  bool have_graphs = false;
  char* slab = nullptr;
  size_t slab_stride = 0;
  int slab_wgs = 0;
  char* sim_scratch = nullptr;   // slices for modules the simulator cannot hold in LDS
  size_t sim_stride = 0;
  int sim_slices = 0;
  // Cost(H) path: profiled data, the batch of fused-op subgraphs and per-node times (dc_set_profile)
  bool bg_canonical = false;     // every base row strictly ascending, no self loop
  long long bg_nodes = 0;
  char* cost_mem = nullptr;
  FusedOpsArgs fo{};             // the pointers that do not change from call to call
  float* m_op_time = nullptr;    // [max_nodes] per contracted node, for dc_cost_candidates
  float* m_ar_size = nullptr;
  float* fo_pred = nullptr;      // raw estimate of each fused op of the last call
  void* headW = nullptr;         // W1 | W2 of the regression network in the layer kernels' layout
  bool have_profile = false;
  std::vector<int> h_gno, h_geo;   // host copies of the base graphs' offsets
  int allow_fused = 1;
  int every_fused_op = 0;        // 1: the estimator also runs on fused ops that repeat an earlier one of the batch
  // training (dc_train_begin)
  bool training = false;
  dc_train_params tp{};
  long long train_t = 0;         // Adam steps taken
  char* train_mem = nullptr;
  TrainPass tb{};                // the buffers of a pass
  float* adam_m = nullptr;
  float* adam_v = nullptr;
  Profiler prof;
  std::string err;
};

namespace {

const char* const kFamilyNames[kFamCount] = {"prep_scan", "contract", "finalize", "aggregate", "update",
                                             "fused_layer", "layer256", "layer256_d64", "aggregate_heavy", "build_desc",
                                             "attention_project", "attention_scores", "attention_aggregate",
                                             "readout_head", "simulate", "fused_op_extract", "fused_op_head",
                                             "train_aggregate", "train_update", "train_head", "train_wgrad",
                                             "train_dgrad", "train_gather_back", "train_adam"};

size_t al(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr int kSimLdsBytes = 80 * 1024;   // two simulator waves per CU

struct Arena {
  size_t off = 0;
  char* base = nullptr;
  template <typename T>
  T* take(size_t count) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += al(count * sizeof(T));
    return p;
  }
};

struct Caps {
  long long C, NB, EB, NN, NE;
};
Caps caps_of(const dc_config& c) {
  Caps k;
  k.C = c.max_cand;
  k.NB = c.max_base_nodes;
  k.EB = c.max_base_edges;
  k.NN = c.max_nodes > 0 ? c.max_nodes : c.max_base_nodes;
  k.NE = c.max_edges > 0 ? c.max_edges : c.max_base_edges;
  return k;
}

// Lays out every scratch array; with base == nullptr only the size is computed.
size_t carve(const dc_config& cfg, char* base, dc_ctx* ctx) {
  const Caps k = caps_of(cfg);
  const size_t es = cfg.dtype == DC_BF16 ? 2 : 4;
  const size_t D = cfg.F > cfg.H ? cfg.F : cfg.H;
  Arena a;
  a.base = base;
  int* status = a.take<int>(64);
  int* totals = a.take<int>(64);
  ContractTmp t;
  t.tmp_eoff = a.take<int>(k.C + 1);
  t.members = a.take<int>(k.NB + 1);
  t.mstart = a.take<int>(k.NB + k.C + 1);
  t.orp = a.take<int>(k.NB + k.C + 1);
  t.irp = a.take<int>(k.NB + k.C + 1);
  t.oc = a.take<int>(k.EB + 1);
  t.ic = a.take<int>(k.EB + 1);
  t.Gc = a.take<int>(k.C + 1);
  t.Ec = a.take<int>(k.C + 1);
  t.big_order = a.take<int>(k.C + 1);
  t.big_meta = a.take<int>(64);
  BatchView b;
  b.node_off = a.take<int>(k.C + 1);
  b.edge_off = a.take<int>(k.C + 1);
  b.new_id = a.take<int>(k.NB + 1);
  b.out_rowptr = a.take<int>(k.NN + 1);
  b.in_rowptr = a.take<int>(k.NN + 1);
  b.out_col = a.take<int>(k.NE + 1);
  b.in_col = a.take<int>(k.NE + 1);
  b.Xc = a.take<char>((size_t)(k.NN + 1) * cfg.F * es);
  b.cap_nodes = k.NN;
  b.cap_edges = k.NE;
  void* act0 = a.take<char>((size_t)(k.NN + 1) * cfg.H * es);
  void* act1 = a.take<char>((size_t)(k.NN + 1) * cfg.H * es);
  void* agg0 = a.take<char>((size_t)(k.NN + 1) * D * es);
  void* agg1 = a.take<char>((size_t)(k.NN + 1) * D * es);
  // one 16-byte descriptor per node and direction, room for whole tiles of 128
  void* desc0 = a.take<char>((size_t)(k.NN + 128) * 16);
  void* desc1 = a.take<char>((size_t)(k.NN + 128) * 16);
  int* heavy0 = a.take<int>((size_t)k.NN + 128);
  int* heavy1 = a.take<int>((size_t)k.NN + 128);
  int* heavy_cnt = a.take<int>(2 * ((size_t)k.NN / 128 + 2));
  int* heavy_ctr = a.take<int>(kHeavyCtrInts);
  int* heavy_off = a.take<int>(2 * ((size_t)k.NN / 128 + 2) + 1);
  unsigned* heavy_list = a.take<unsigned>(2 * ((size_t)k.NN + 128));
  // chunk sums of the readout formed by the last layer (bulk bf16 shapes with uniform coefficients only)
  const bool ro = cfg.dtype == DC_BF16 && cfg.H == 256 && cfg.aggregator != DC_AGG_ATTENTION;
  float* ro_part = a.take<float>(ro ? ((size_t)k.NN / 64 + (size_t)k.C + 2) * 256 : 0);
  int* ro_first = a.take<int>(ro ? (size_t)k.NN / 64 + 2 : 0);
  const size_t nscore = cfg.aggregator == DC_AGG_ATTENTION ? (size_t)(k.NN + 1) * cfg.heads : 0;
  float* score0 = a.take<float>(nscore);
  float* score1 = a.take<float>(nscore);
  if (ctx) {
    ctx->score[0] = score0;
    ctx->score[1] = score1;
    ctx->status = status;
    ctx->totals = totals;
    ctx->tmp = t;
    ctx->ib = b;
    ctx->act[0] = act0;
    ctx->act[1] = act1;
    ctx->agg[0] = agg0;
    ctx->agg[1] = agg1;
    ctx->desc[0] = desc0;
    ctx->desc[1] = desc1;
    ctx->heavy[0] = heavy0;
    ctx->heavy[1] = heavy1;
    ctx->heavy_cnt = heavy_cnt;
    ctx->heavy_ctr = heavy_ctr;
    ctx->heavy_off = heavy_off;
    ctx->heavy_list = heavy_list;
    ctx->ro_part = ro ? ro_part : nullptr;
    ctx->ro_first = ro ? ro_first : nullptr;
  }
  return a.off;
}

dc_status cfg_check(const dc_config* c, std::string* why) {
  if (!c) return DC_ERR_INVALID_ARG;
  if (c->dtype != DC_F32 && c->dtype != DC_BF16) return DC_ERR_INVALID_ARG;
  if (c->max_cand < 0 || c->max_base_nodes < 0 || c->max_base_edges < 0 || c->max_nodes < 0 || c->max_edges < 0)
    return DC_ERR_INVALID_ARG;
  if (!gnn_shape_supported(c->F, c->H, c->L)) {
    if (why) *why = "need F % 16 == 0, H % 32 == 0, F,H <= 512, L >= 1";
    return (c->F <= 0 || c->H <= 0 || c->L <= 0) ? DC_ERR_INVALID_ARG : DC_ERR_UNSUPPORTED;
  }
  if (c->aggregator != DC_AGG_MEAN && c->aggregator != DC_AGG_ATTENTION) return DC_ERR_INVALID_ARG;
  if (c->aggregator == DC_AGG_ATTENTION && !attention_shape_supported(c->H, c->heads)) {
    if (why) *why = "attention needs H a power of two in [32, 512] and heads a power of two with H / heads >= 8";
    return c->heads <= 0 ? DC_ERR_INVALID_ARG : DC_ERR_UNSUPPORTED;
  }
  const long long lim = 2000000000LL;
  if (c->max_cand > lim || c->max_base_nodes + c->max_cand > lim || c->max_base_edges > lim) {
    if (why) *why = "totals must fit in int32";
    return DC_ERR_UNSUPPORTED;
  }
  return DC_OK;
}

dc_status fail(dc_ctx* ctx, dc_status st, const std::string& msg) {
  if (ctx) ctx->err = msg;
  return st;
}

dc_status hip_fail(dc_ctx* ctx, hipError_t e, const char* what) {
  char buf[256];
  snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
  if (ctx) ctx->err = buf;
  return e == hipErrorOutOfMemory ? DC_ERR_OOM : DC_ERR_HIP;
}

// features = false: the contracted graphs without the feature sums (Cost(H) takes its per-node inputs from the
// profile and the estimator's batch, not from the features of the module's nodes)
dc_status do_contract(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                      const int32_t* group_id, const BatchView& out, hipStream_t s, bool features = true) {
  ContractLaunch a;
  a.bg = ctx->bg;
  a.max_graph_nodes = ctx->max_gn;
  a.max_graph_edges = ctx->max_ge;
  a.min_graph_need = ctx->min_need;
  a.n_cand = n_cand;
  a.cand_graph = cand_graph;
  a.cand_off = cand_off;
  a.group_id = group_id;
  a.tmp = ctx->tmp;
  a.out = out;
  a.F = features ? ctx->cfg.F : 0;
  a.bf16 = ctx->cfg.dtype == DC_BF16;
  a.max_base_nodes = ctx->cfg.max_base_nodes;
  a.max_base_edges = ctx->cfg.max_base_edges;
  a.status = ctx->status;
  a.totals = ctx->totals;
  a.slab = ctx->slab;
  a.slab_stride = ctx->slab_stride;
  a.slab_wgs = ctx->slab_wgs;
  a.lds_limit = ctx->lds_limit;
  hipError_t e = launch_contract(a, ctx->prof.on ? &ctx->prof : nullptr, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "contraction launch");
  return DC_OK;
}

GnnArgs gnn_args(dc_ctx* ctx, int32_t n_cand, const BatchView& in, float* pred);

dc_status do_forward(dc_ctx* ctx, int32_t n_cand, const BatchView& in, float* pred, hipStream_t s) {
  GnnArgs g = gnn_args(ctx, n_cand, in, pred);
  g.fuse_readout = 1;                        // nothing but the readout looks at the last layer's rows here
  hipError_t e = launch_gnn_forward(g, ctx->prof.on ? &ctx->prof : nullptr, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "forward launch");
  return DC_OK;
}

GnnArgs gnn_args(dc_ctx* ctx, int32_t n_cand, const BatchView& in, float* pred) {
  GnnArgs g;
  g.n_cand = n_cand;
  g.node_off = in.node_off;
  g.out_rowptr = in.out_rowptr;
  g.out_col = in.out_col;
  g.in_rowptr = in.in_rowptr;
  g.in_col = in.in_col;
  g.Xc = in.Xc;
  g.F = ctx->cfg.F;
  g.H = ctx->cfg.H;
  g.L = ctx->cfg.L;
  g.bf16 = ctx->cfg.dtype == DC_BF16;
  g.W = ctx->W;
  g.b = ctx->b;
  g.head = ctx->head;
  g.act[0] = ctx->act[0];
  g.act[1] = ctx->act[1];
  g.agg[0] = ctx->agg[0];
  g.agg[1] = ctx->agg[1];
  g.desc[0] = ctx->desc[0];
  g.desc[1] = ctx->desc[1];
  g.heavy[0] = ctx->heavy[0];
  g.heavy[1] = ctx->heavy[1];
  g.heavy_cnt = ctx->heavy_cnt;
  g.heavy_ctr = ctx->heavy_ctr;
  g.heavy_off = ctx->heavy_off;
  g.heavy_list = ctx->heavy_list;
  g.ro_part = ctx->ro_part;
  g.ro_first = ctx->ro_first;
  g.pred = pred;
  g.status = ctx->status;
  g.n_cu = ctx->n_cu;
  g.allow_fused = ctx->allow_fused;
  if (ctx->cfg.aggregator == DC_AGG_ATTENTION) {
    g.heads = ctx->cfg.heads;
    g.att = ctx->att;
    g.score[0] = ctx->score[0];
    g.score[1] = ctx->score[1];
  }
  return g;
}

dc_status do_simulate(dc_ctx* ctx, int32_t n_cand, const BatchView& in, const float* op_time, const float* ar_size,
                      float ar_c, float ar_d, float* cost, hipStream_t s) {
  SimArgs a;
  a.n_cand = n_cand;
  a.node_off = in.node_off;
  a.out_rowptr = in.out_rowptr;
  a.out_col = in.out_col;
  a.in_rowptr = in.in_rowptr;
  a.op_time = op_time;
  a.ar_size = ar_size;
  a.ar_c = ar_c;
  a.ar_d = ar_d;
  a.cost = cost;
  a.lds_bytes = kSimLdsBytes;
  a.scratch = ctx->sim_scratch;
  a.scratch_stride = ctx->sim_stride;
  a.n_slices = ctx->sim_slices;
  a.status = ctx->status;
  if (ctx->prof.on) ctx->prof.begin(kFamSimulate, s);
  hipError_t e = launch_simulate(a, s);
  if (ctx->prof.on) ctx->prof.end(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "simulator launch");
  return DC_OK;
}

// After a contraction into `cb`: the batch of fused-op subgraphs, the estimator on it, and the
// time / tensor size of every node of the contracted batch.
dc_status do_module_times(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                          const BatchView& cb, float* op_time, float* ar_size, hipStream_t s) {
  Profiler* prof = ctx->prof.on ? &ctx->prof : nullptr;
  FusedOpsArgs a = ctx->fo;
  a.bg = ctx->bg;
  a.n_cand = n_cand;
  a.cand_graph = cand_graph;
  a.cand_off = cand_off;
  a.members = ctx->tmp.members;
  a.mstart = ctx->tmp.mstart;
  a.Gc = ctx->tmp.Gc;
  a.new_id = cb.new_id;
  a.c_node_off = cb.node_off;
  a.op_time = op_time;
  a.ar_size = ar_size;
  if (ctx->every_fused_op) a.table = nullptr;
  hipError_t e = launch_fused_op_extract(a, prof, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "fused-op extraction launch");
  // the layer kernels only need the total row count: the batch is handed over as one graph
  GnnArgs g = gnn_args(ctx, 1, a.fb, nullptr);
  g.node_off = a.totals;
  const void* h_last = nullptr;
  e = launch_gnn_layers(g, prof, s, &h_last);
  if (e != hipSuccess) return hip_fail(ctx, e, "fused-op forward launch");
  const size_t es = ctx->cfg.dtype == DC_BF16 ? 2 : 4;
  const size_t HH = (size_t)ctx->cfg.H * ctx->cfg.H;
  const int H = ctx->cfg.H;
  if (prof) prof->begin(kFamFusedHead, s);
  void* R = ctx->agg[0];
  void* Z1 = ctx->agg[1];
  void* Z2 = ctx->agg[0];
  e = launch_fused_op_readout(a, h_last, R, s);
  GnnArgs gh = g;
  gh.node_off = a.totals + 2;               // rows = fused ops
  launch_dense_bias_relu(gh, R, H, ctx->headW, ctx->head + HH, Z1, s);
  launch_dense_bias_relu(gh, Z1, H, static_cast<char*>(ctx->headW) + HH * es, ctx->head + 2 * HH + H, Z2, s);
  if (e == hipSuccess) e = launch_fused_op_times(a, Z2, ctx->head + 2 * HH + 2 * H, ctx->fo_pred, s);
  if (prof) prof->end(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "fused-op head launch");
  return DC_OK;
}

// Device-side guard for dc_gnn_forward on caller-provided batches: sizes within the
// capacity, every graph below 65536 nodes, row pointers ascending and within the edge
// capacity, every neighbour inside its own graph.  One thread per node; on any
// violation the status word is set and every later kernel of the call returns at once.
__global__ __launch_bounds__(256) void check_batch_kernel(const int* __restrict__ node_off, int C, long long max_nodes,
                                                           long long cap_edges, const int* __restrict__ out_rp,
                                                           const int* __restrict__ out_ci,
                                                           const int* __restrict__ in_rp,
                                                           const int* __restrict__ in_ci, int* status) {
  const long long ntot = node_off[C];
  if (ntot > max_nodes || ntot < 0 || node_off[0] != 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) set_error(status, (int)DC_ERR_CAPACITY);
    return;
  }
  bool bad = false;
  for (long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x; c < C; c += (long long)gridDim.x * blockDim.x) {
    const int n = node_off[c + 1] - node_off[c];
    bad |= n < 0 || n >= 65536;
  }
  for (long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x; v < ntot;
       v += (long long)gridDim.x * blockDim.x) {
    int lo = 0, hi = C;                       // graph of v: last c with node_off[c] <= v
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (node_off[mid] <= v) lo = mid; else hi = mid;
    }
    const int g0 = node_off[lo], g1 = node_off[lo + 1];
    bad |= v >= g1;                           // offsets not ascending
    for (int dir = 0; dir < 2 && !bad; ++dir) {
      const int* rp = dir ? out_rp : in_rp;
      const int* ci = dir ? out_ci : in_ci;
      const int s = rp[v], e = rp[v + 1];
      if (s < 0 || e < s || e > cap_edges || e - s >= 65536) {
        bad = true;
        break;
      }
      for (int k = s; k < e; ++k) {
        const int u = ci[k];
        bad |= u < g0 || u >= g1;
      }
    }
  }
  if (bad) set_error(status, (int)DC_ERR_BAD_GRAPH);
}

__global__ void empty_batch_kernel(int* node_off, int* edge_off, int* orp, int* irp, int* totals) {
  node_off[0] = 0;
  edge_off[0] = 0;
  orp[0] = 0;
  irp[0] = 0;
  totals[0] = 0;
  totals[1] = 0;
}

}  // namespace

namespace dc {
void launch_check_batch(const int* node_off, int n_cand, long long max_nodes, long long cap_edges, const int* out_rp,
                        const int* out_ci, const int* in_rp, const int* in_ci, int* status, int n_cu, hipStream_t s) {
  hipLaunchKernelGGL(check_batch_kernel, dim3(n_cu * 4), dim3(256), 0, s, node_off, n_cand, max_nodes, cap_edges, out_rp,
                     out_ci, in_rp, in_ci, status);
}
}  // namespace dc

extern "C" {

size_t dc_workspace_bytes(const dc_config* cfg) {
  if (cfg_check(cfg, nullptr) != DC_OK) return 0;
  return carve(*cfg, nullptr, nullptr);
}

dc_status dc_create(dc_ctx** out, const dc_config* cfg) {
  if (!out) return DC_ERR_INVALID_ARG;
  *out = nullptr;
  std::string why;
  dc_status st = cfg_check(cfg, &why);
  if (st != DC_OK) return st;
  dc_ctx* ctx = new (std::nothrow) dc_ctx();
  if (!ctx) return DC_ERR_OOM;
  ctx->cfg = *cfg;
  hipError_t e = hipGetDevice(&ctx->device);
  if (e != hipSuccess) {
    delete ctx;
    return DC_ERR_HIP;
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, ctx->device) == hipSuccess) {
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    size_t lds = prop.sharedMemPerBlock;
    if (prop.sharedMemPerBlockOptin > lds) lds = prop.sharedMemPerBlockOptin;
    if (lds > 160 * 1024) lds = 160 * 1024;
    // keep room for the kernel's static LDS
    ctx->lds_limit = (int)lds - 1024;
    if (ctx->lds_limit > 48 * 1024 && contract_set_lds_limit(ctx->lds_limit) != hipSuccess) {
      (void)hipGetLastError();
      ctx->lds_limit = 48 * 1024;
    }
  }
  ctx->arena_bytes = carve(*cfg, nullptr, nullptr);
  e = hipMalloc(reinterpret_cast<void**>(&ctx->arena), ctx->arena_bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return DC_ERR_OOM;
  }
  carve(*cfg, ctx->arena, ctx);
  e = hipMemset(ctx->status, 0, 64 * sizeof(int));
  if (e == hipSuccess) e = hipMemset(ctx->totals, 0, 64 * sizeof(int));
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ctx->h_pinned), 64 * sizeof(int), hipHostMallocDefault);
  const size_t es = cfg->dtype == DC_BF16 ? 2 : 4;
  const size_t HH = (size_t)cfg->H * cfg->H;
  if (e == hipSuccess) e = hipMalloc(&ctx->W, packed_weight_elems(cfg->F, cfg->H, cfg->L, 3) * es);
  if (e == hipSuccess && cfg->aggregator == DC_AGG_ATTENTION)
    e = hipMalloc(reinterpret_cast<void**>(&ctx->att), (size_t)cfg->L * 2 * cfg->H * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->b), (size_t)cfg->L * cfg->H * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->head), (2 * HH + 3 * cfg->H + 1) * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&ctx->headW, 2 * HH * es);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    dc_destroy(ctx);
    return e == hipErrorOutOfMemory ? DC_ERR_OOM : DC_ERR_HIP;
  }
  *out = ctx;
  return DC_OK;
}

dc_status dc_destroy(dc_ctx* ctx) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  (void)hipDeviceSynchronize();
  for (int i = 0; i < ctx->prof.created; ++i) (void)hipEventDestroy(ctx->prof.ev[i]);
  if (ctx->arena) (void)hipFree(ctx->arena);
  if (ctx->h_pinned) (void)hipHostFree(ctx->h_pinned);
  if (ctx->W) (void)hipFree(ctx->W);
  if (ctx->b) (void)hipFree(ctx->b);
  if (ctx->head) (void)hipFree(ctx->head);
  if (ctx->att) (void)hipFree(ctx->att);
  if (ctx->headW) (void)hipFree(ctx->headW);
  if (ctx->cost_mem) (void)hipFree(ctx->cost_mem);
  if (ctx->bg_mem) (void)hipFree(ctx->bg_mem);
  if (ctx->slab) (void)hipFree(ctx->slab);
  if (ctx->sim_scratch) (void)hipFree(ctx->sim_scratch);
  if (ctx->train_mem) (void)hipFree(ctx->train_mem);
  delete ctx;
  return DC_OK;
}

static dc_status set_weights_common(dc_ctx* ctx, const float* W_layers, const float* att, const float* b_layers,
                                    const float* head, hipStream_t s) {
  const dc_config& c = ctx->cfg;
  const int bf16 = c.dtype == DC_BF16;
  const int nseg = c.aggregator == DC_AGG_ATTENTION ? 1 : 3;
  const size_t es = bf16 ? 2 : 4;
  const size_t nW = packed_weight_elems(c.F, c.H, c.L, nseg);
  std::vector<char> packed(nW * es);
  pack_weights_host(W_layers, c.F, c.H, c.L, nseg, bf16, packed.data());
  const size_t HH = (size_t)c.H * c.H;
  std::vector<float> hd(head, head + 2 * HH + 3 * c.H + 1);
  if (bf16) {
    // the head matrices are stored as bf16-representable fp32 values
    auto rnd = [](float x) {
      unsigned u;
      memcpy(&u, &x, 4);
      if ((u & 0x7F800000u) == 0x7F800000u) return x;
      u += 0x7FFFu + ((u >> 16) & 1u);
      u &= 0xFFFF0000u;
      memcpy(&x, &u, 4);
      return x;
    };
    for (size_t i = 0; i < HH; ++i) hd[i] = rnd(hd[i]);
    for (size_t i = 0; i < HH; ++i) hd[HH + c.H + i] = rnd(hd[HH + c.H + i]);
    for (int i = 0; i < c.H; ++i) hd[2 * HH + 2 * c.H + i] = rnd(hd[2 * HH + 2 * c.H + i]);
  }
  // W1 and W2 once more in the layout of a layer block: the fused-op path runs them as GEMMs
  std::vector<char> hw(2 * HH * es);
  pack_weights_host(head, c.H, c.H, 1, 1, bf16, hw.data());
  pack_weights_host(head + HH + c.H, c.H, c.H, 1, 1, bf16, hw.data() + HH * es);
  hipError_t e = hipMemcpyAsync(ctx->W, packed.data(), nW * es, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(ctx->headW, hw.data(), hw.size(), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(ctx->b, b_layers, (size_t)c.L * c.H * sizeof(float), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(ctx->head, hd.data(), hd.size() * sizeof(float), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && att)
    e = hipMemcpyAsync(ctx->att, att, (size_t)c.L * 2 * c.H * sizeof(float), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);   // host staging buffers die at return
  if (e != hipSuccess) return hip_fail(ctx, e, "weight copy");
  ctx->have_weights = true;
  return DC_OK;
}

dc_status dc_set_weights(dc_ctx* ctx, const float* W_layers, const float* b_layers, const float* head,
                         void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!W_layers || !b_layers || !head) return fail(ctx, DC_ERR_INVALID_ARG, "null weight pointer");
  if (ctx->cfg.aggregator != DC_AGG_MEAN)
    return fail(ctx, DC_ERR_INVALID_ARG, "this context aggregates with attention: use dc_set_attention_weights");
  return set_weights_common(ctx, W_layers, nullptr, b_layers, head, static_cast<hipStream_t>(stream));
}

dc_status dc_set_attention_weights(dc_ctx* ctx, const float* W_layers, const float* att, const float* b_layers,
                                   const float* head, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!W_layers || !att || !b_layers || !head) return fail(ctx, DC_ERR_INVALID_ARG, "null weight pointer");
  if (ctx->cfg.aggregator != DC_AGG_ATTENTION)
    return fail(ctx, DC_ERR_INVALID_ARG, "this context aggregates with the mean: use dc_set_weights");
  return set_weights_common(ctx, W_layers, att, b_layers, head, static_cast<hipStream_t>(stream));
}

dc_status dc_set_base_graphs(dc_ctx* ctx, int32_t n_graphs, const int32_t* g_node_off, const int32_t* g_edge_off,
                             const int32_t* rowptr, const int32_t* col, const float* X, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (n_graphs <= 0 || !g_node_off || !g_edge_off || !rowptr || !X)
    return fail(ctx, DC_ERR_INVALID_ARG, "null pointer or no graphs");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (g_node_off[0] != 0 || g_edge_off[0] != 0) return fail(ctx, DC_ERR_BAD_GRAPH, "offsets must start at 0");
  int max_gn = 0, max_ge = 0, min_need = INT32_MAX;
  bool canonical = true;
  for (int b = 0; b < n_graphs; ++b) {
    const long long n = (long long)g_node_off[b + 1] - g_node_off[b];
    const long long e = (long long)g_edge_off[b + 1] - g_edge_off[b];
    if (n < 0 || e < 0) return fail(ctx, DC_ERR_BAD_GRAPH, "offsets not monotone");
    if (n >= 65536) return fail(ctx, DC_ERR_UNSUPPORTED, "a base graph must have fewer than 65536 nodes");
    if (e > 0 && !col) return fail(ctx, DC_ERR_INVALID_ARG, "null col");
    const int32_t* rp = rowptr + g_node_off[b] + b;
    if (rp[0] != 0 || rp[n] != e) return fail(ctx, DC_ERR_BAD_GRAPH, "rowptr must run from 0 to the edge count");
    for (long long v = 0; v < n; ++v)
      if (rp[v + 1] < rp[v]) return fail(ctx, DC_ERR_BAD_GRAPH, "rowptr not monotone");
    const int32_t* ci = col + g_edge_off[b];
    for (long long k = 0; k < e; ++k)
      if (ci[k] < 0 || ci[k] >= n) return fail(ctx, DC_ERR_BAD_GRAPH, "col out of range");
    for (long long v = 0; v < n && canonical; ++v)
      for (long long k = rp[v]; k < rp[v + 1]; ++k)
        if (ci[k] == v || (k > rp[v] && ci[k] <= ci[k - 1])) canonical = false;
    if (n > max_gn) max_gn = (int)n;
    if (e > max_ge) max_ge = (int)e;
    const int need = contract_working_set_bytes((int)n, (int)e);
    if (need < min_need) min_need = need;
  }
  const long long NT = g_node_off[n_graphs], ET = g_edge_off[n_graphs];
  // predecessor lists (transpose), sources ascending
  std::vector<int32_t> crp((size_t)NT + n_graphs), cci((size_t)(ET > 0 ? ET : 1));
  for (int b = 0; b < n_graphs; ++b) {
    const int n = g_node_off[b + 1] - g_node_off[b];
    const int32_t* rp = rowptr + g_node_off[b] + b;
    const int32_t* ci = col + g_edge_off[b];
    int32_t* trp = crp.data() + g_node_off[b] + b;
    int32_t* tci = cci.data() + g_edge_off[b];
    for (int v = 0; v <= n; ++v) trp[v] = 0;
    for (int k = 0; k < rp[n]; ++k) trp[ci[k] + 1] += 1;
    for (int v = 0; v < n; ++v) trp[v + 1] += trp[v];
    std::vector<int32_t> cur(trp, trp + n);
    for (int u = 0; u < n; ++u)
      for (int k = rp[u]; k < rp[u + 1]; ++k) tci[cur[ci[k]]++] = u;
  }
  // one device block: gno | geo | rowptr | col | crowptr | ccol | X
  Arena a;
  a.take<int>(n_graphs + 1);
  a.take<int>(n_graphs + 1);
  a.take<int>(NT + n_graphs);
  a.take<int>(ET + 1);
  a.take<int>(NT + n_graphs);
  a.take<int>(ET + 1);
  a.take<float>((size_t)NT * ctx->cfg.F + 4);
  char* mem = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&mem), a.off);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, DC_ERR_OOM, "base graph allocation failed");
  }
  Arena d;
  d.base = mem;
  int* d_gno = d.take<int>(n_graphs + 1);
  int* d_geo = d.take<int>(n_graphs + 1);
  int* d_rp = d.take<int>(NT + n_graphs);
  int* d_ci = d.take<int>(ET + 1);
  int* d_crp = d.take<int>(NT + n_graphs);
  int* d_cci = d.take<int>(ET + 1);
  float* d_X = d.take<float>((size_t)NT * ctx->cfg.F + 4);
  e = hipMemcpyAsync(d_gno, g_node_off, (n_graphs + 1) * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(d_geo, g_edge_off, (n_graphs + 1) * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(d_rp, rowptr, (size_t)(NT + n_graphs) * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && ET > 0) e = hipMemcpyAsync(d_ci, col, (size_t)ET * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(d_crp, crp.data(), (size_t)(NT + n_graphs) * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && ET > 0) e = hipMemcpyAsync(d_cci, cci.data(), (size_t)ET * sizeof(int), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && NT > 0) e = hipMemcpyAsync(d_X, X, (size_t)NT * ctx->cfg.F * sizeof(float), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  char* slab = nullptr;
  size_t slab_stride = 0;
  int slab_wgs = 0;
  if (e == hipSuccess && contract_working_set_bytes(max_gn, max_ge) > ctx->lds_limit) {
    slab_stride = al((size_t)contract_working_set_bytes(max_gn, max_ge));
    slab_wgs = ctx->n_cu * 2;
    e = hipMalloc(reinterpret_cast<void**>(&slab), slab_stride * slab_wgs);
  }
  // the simulator keeps a module in LDS if it fits kSimLdsBytes; a contracted graph is never
  // larger than its base graph, so slices of the largest base graph serve all the others
  char* sim = nullptr;
  size_t sim_stride = 0;
  int sim_slices = 0;
  if (e == hipSuccess && simulate_scratch_bytes(max_gn, max_ge, 1) > (size_t)kSimLdsBytes) {
    sim_stride = al(simulate_scratch_bytes(max_gn, max_ge, 1));
    // one wave per slice; many waves per CU hide the latency of the walk (up to 2 GB of slices)
    sim_slices = ctx->n_cu * 16;
    const size_t fit = ((size_t)2 << 30) / sim_stride;
    if ((size_t)sim_slices > fit) sim_slices = (int)(fit > (size_t)ctx->n_cu ? fit : (size_t)ctx->n_cu);
    e = hipMalloc(reinterpret_cast<void**>(&sim), sim_stride * sim_slices);
  }
  if (e != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(mem);
    if (slab) (void)hipFree(slab);
    return hip_fail(ctx, e, "dc_set_base_graphs copy");
  }
  (void)hipDeviceSynchronize();   // earlier calls may still read the old graphs
  if (ctx->bg_mem) (void)hipFree(ctx->bg_mem);
  if (ctx->slab) (void)hipFree(ctx->slab);
  if (ctx->sim_scratch) (void)hipFree(ctx->sim_scratch);
  ctx->sim_scratch = sim;
  ctx->sim_stride = sim_stride;
  ctx->sim_slices = sim_slices;
  ctx->bg_mem = mem;
  ctx->slab = slab;
  ctx->slab_stride = slab_stride;
  ctx->slab_wgs = slab_wgs;
  ctx->bg.n_graphs = n_graphs;
  ctx->bg.gno = d_gno;
  ctx->bg.geo = d_geo;
  ctx->bg.rowptr = d_rp;
  ctx->bg.col = d_ci;
  ctx->bg.crowptr = d_crp;
  ctx->bg.ccol = d_cci;
  ctx->bg.X = d_X;
  ctx->max_gn = max_gn;
  ctx->max_ge = max_ge;
  ctx->min_need = min_need;
  ctx->have_graphs = true;
  ctx->bg_canonical = canonical;
  ctx->bg_nodes = NT;
  ctx->h_gno.assign(g_node_off, g_node_off + n_graphs + 1);
  ctx->h_geo.assign(g_edge_off, g_edge_off + n_graphs + 1);
  if (ctx->cost_mem) (void)hipFree(ctx->cost_mem);   // the profile belongs to the graphs it was recorded on
  ctx->cost_mem = nullptr;
  ctx->have_profile = false;
  return DC_OK;
}

dc_status dc_contract_graphs(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                             const int32_t* group_id, dc_batch* out, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!out || n_cand < 0) return fail(ctx, DC_ERR_INVALID_ARG, "null batch or negative count");
  if (!ctx->have_graphs) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_base_graphs has not been called");
  if (n_cand > ctx->cfg.max_cand) return fail(ctx, DC_ERR_CAPACITY, "n_cand exceeds max_cand");
  if (!out->node_off || !out->edge_off || !out->new_id || !out->out_rowptr || !out->out_col || !out->in_rowptr ||
      !out->in_col || !out->Xc || out->cap_nodes < 0 || out->cap_edges < 0)
    return fail(ctx, DC_ERR_INVALID_ARG, "dc_batch has a null array or negative capacity");
  if (n_cand > 0 && (!cand_graph || !cand_off || !group_id)) return fail(ctx, DC_ERR_INVALID_ARG, "null candidate array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  out->n_cand = n_cand;
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  BatchView v;
  v.node_off = out->node_off;
  v.edge_off = out->edge_off;
  v.new_id = out->new_id;
  v.out_rowptr = out->out_rowptr;
  v.out_col = out->out_col;
  v.in_rowptr = out->in_rowptr;
  v.in_col = out->in_col;
  v.Xc = out->Xc;
  v.cap_nodes = out->cap_nodes;
  v.cap_edges = out->cap_edges;
  if (n_cand == 0) {
    hipLaunchKernelGGL(empty_batch_kernel, dim3(1), dim3(1), 0, s, out->node_off, out->edge_off, out->out_rowptr,
                       out->in_rowptr, ctx->totals);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? DC_OK : hip_fail(ctx, e, "empty batch");
  }
  return do_contract(ctx, n_cand, cand_graph, cand_off, group_id, v, s);
}

dc_status dc_gnn_forward(dc_ctx* ctx, const dc_batch* in, float* pred, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!in || in->n_cand < 0) return fail(ctx, DC_ERR_INVALID_ARG, "null batch or negative count");
  if (!ctx->have_weights) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_weights has not been called");
  if (in->n_cand > ctx->cfg.max_cand) return fail(ctx, DC_ERR_CAPACITY, "n_cand exceeds max_cand");
  if (in->n_cand == 0) return DC_OK;
  if (!pred || !in->node_off || !in->out_rowptr || !in->out_col || !in->in_rowptr || !in->in_col || !in->Xc)
    return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  const Caps k = caps_of(ctx->cfg);
  hipLaunchKernelGGL(check_batch_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, s, in->node_off, in->n_cand,
                     (long long)(in->cap_nodes < k.NN ? in->cap_nodes : k.NN), (long long)in->cap_edges, in->out_rowptr, in->out_col, in->in_rowptr,
                     in->in_col, ctx->status);
  BatchView v;
  v.node_off = in->node_off;
  v.edge_off = in->edge_off;
  v.new_id = in->new_id;
  v.out_rowptr = in->out_rowptr;
  v.out_col = in->out_col;
  v.in_rowptr = in->in_rowptr;
  v.in_col = in->in_col;
  v.Xc = in->Xc;
  v.cap_nodes = in->cap_nodes;
  v.cap_edges = in->cap_edges;
  return do_forward(ctx, in->n_cand, v, pred, s);
}

dc_status dc_simulate(dc_ctx* ctx, const dc_batch* in, const float* op_time, const float* ar_size, float ar_c,
                      float ar_d, float* cost, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!in || in->n_cand < 0) return fail(ctx, DC_ERR_INVALID_ARG, "null batch or negative count");
  if (!ctx->have_graphs) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_base_graphs has not been called");
  if (in->n_cand > ctx->cfg.max_cand) return fail(ctx, DC_ERR_CAPACITY, "n_cand exceeds max_cand");
  if (in->n_cand == 0) return DC_OK;
  if (!cost || !op_time || !ar_size || !in->node_off || !in->out_rowptr || !in->out_col || !in->in_rowptr ||
      !in->in_col)
    return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  const Caps k = caps_of(ctx->cfg);
  hipLaunchKernelGGL(check_batch_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, s, in->node_off, in->n_cand,
                     (long long)(in->cap_nodes < k.NN ? in->cap_nodes : k.NN), (long long)in->cap_edges,
                     in->out_rowptr, in->out_col, in->in_rowptr, in->in_col, ctx->status);
  BatchView v{};
  v.node_off = in->node_off;
  v.out_rowptr = in->out_rowptr;
  v.out_col = in->out_col;
  v.in_rowptr = in->in_rowptr;
  v.in_col = in->in_col;
  return do_simulate(ctx, in->n_cand, v, op_time, ar_size, ar_c, ar_d, cost, s);
}

dc_status dc_eval_candidates(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                             const int32_t* group_id, float* pred, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (n_cand < 0) return fail(ctx, DC_ERR_INVALID_ARG, "negative count");
  if (!ctx->have_graphs) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_base_graphs has not been called");
  if (!ctx->have_weights) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_weights has not been called");
  if (n_cand > ctx->cfg.max_cand) return fail(ctx, DC_ERR_CAPACITY, "n_cand exceeds max_cand");
  if (n_cand == 0) return DC_OK;
  if (!cand_graph || !cand_off || !group_id || !pred) return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  dc_status st = do_contract(ctx, n_cand, cand_graph, cand_off, group_id, ctx->ib, s);
  if (st != DC_OK) return st;
  return do_forward(ctx, n_cand, ctx->ib, pred, s);
}

dc_status dc_set_profile(dc_ctx* ctx, const float* op_time, const float* ar_size, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!op_time || !ar_size) return fail(ctx, DC_ERR_INVALID_ARG, "null profile array");
  if (!ctx->have_graphs) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_base_graphs has not been called");
  if (!ctx->bg_canonical)
    return fail(ctx, DC_ERR_BAD_GRAPH, "the cost path needs base rows strictly ascending (no duplicates, no self loops)");
  const Caps k = caps_of(ctx->cfg);
  if (k.NN < k.NB || k.NE < k.EB)
    return fail(ctx, DC_ERR_CAPACITY, "the cost path runs the estimator on up to max_base_nodes rows: create the "
                                      "context with max_nodes = 0 and max_edges = 0");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t es = ctx->cfg.dtype == DC_BF16 ? 2 : 4;
  const long long NT = ctx->bg_nodes;
  const long long cap_ops = k.NB / 2 + 1;
  FusedOpsArgs f{};
  float *tb = nullptr, *xb = nullptr, *mt = nullptr, *mx = nullptr, *fp = nullptr;
  size_t bytes = 0;
  for (int pass = 0; pass < 2; ++pass) {
    Arena a;
    a.base = pass ? ctx->cost_mem : nullptr;
    tb = a.take<float>(NT + 1);
    xb = a.take<float>(NT + 1);
    f.gfm = a.take<int>(k.NB + k.C + 1);
    f.gfk = a.take<int>(k.NB + k.C + 1);
    f.dgo = a.take<int>(k.NB + k.C + 1);
    f.dgi = a.take<int>(k.NB + k.C + 1);
    f.cnt = a.take<int>(3 * (k.C + 1));
    f.totals = a.take<int>(64);
    f.fb.node_off = a.take<int>(cap_ops + 1);
    f.fb.edge_off = a.take<int>(cap_ops + 1);
    f.fo_cnode = a.take<int>(cap_ops + 1);
    f.table = a.take<int>(fused_op_table_entries(cap_ops));
    f.dup_of = a.take<int>(k.NB + k.C + 1);
    f.fb.new_id = a.take<int>(k.NB + 1);
    f.fb.out_rowptr = a.take<int>(k.NB + 1);
    f.fb.in_rowptr = a.take<int>(k.NB + 1);
    f.fb.out_col = a.take<int>(k.EB + 1);
    f.fb.in_col = a.take<int>(k.EB + 1);
    f.fb.Xc = a.take<char>((size_t)(k.NB + 1) * ctx->cfg.F * es);
    mt = a.take<float>(k.NN + 1);
    mx = a.take<float>(k.NN + 1);
    fp = a.take<float>(cap_ops + 1);
    bytes = a.off;
    if (pass == 0) {
      (void)hipDeviceSynchronize();   // earlier calls may still use the old block
      if (ctx->cost_mem) (void)hipFree(ctx->cost_mem);
      ctx->cost_mem = nullptr;
      ctx->have_profile = false;
      if (hipMalloc(reinterpret_cast<void**>(&ctx->cost_mem), bytes) != hipSuccess) {
        (void)hipGetLastError();
        ctx->cost_mem = nullptr;
        return fail(ctx, DC_ERR_OOM, "cost path allocation failed");
      }
    }
  }
  f.fb.cap_nodes = k.NB;
  f.fb.cap_edges = k.EB;
  f.cap_ops = cap_ops;
  f.table_mask = (unsigned)(fused_op_table_entries(cap_ops) - 1);
  f.cap_rows = k.NB;
  f.cap_edges = k.EB;
  f.op_time_base = tb;
  f.ar_size_base = xb;
  f.F = ctx->cfg.F;
  f.H = ctx->cfg.H;
  f.bf16 = ctx->cfg.dtype == DC_BF16;
  f.status = ctx->status;
  f.n_cu = ctx->n_cu;
  hipError_t e = hipMemsetAsync(f.totals, 0, 64 * sizeof(int), s);
  if (e == hipSuccess && NT > 0) e = hipMemcpyAsync(tb, op_time, (size_t)NT * sizeof(float), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && NT > 0) e = hipMemcpyAsync(xb, ar_size, (size_t)NT * sizeof(float), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "dc_set_profile copy");
  ctx->fo = f;
  ctx->m_op_time = mt;
  ctx->m_ar_size = mx;
  ctx->fo_pred = fp;
  ctx->have_profile = true;
  return DC_OK;
}

static dc_status cost_call_check(dc_ctx* ctx, int32_t n_cand) {
  if (n_cand < 0) return fail(ctx, DC_ERR_INVALID_ARG, "negative count");
  if (!ctx->have_graphs) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_base_graphs has not been called");
  if (!ctx->have_weights) return fail(ctx, DC_ERR_INVALID_ARG, "the estimator weights have not been set");
  if (!ctx->have_profile) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_profile has not been called");
  if (n_cand > ctx->cfg.max_cand) return fail(ctx, DC_ERR_CAPACITY, "n_cand exceeds max_cand");
  return DC_OK;
}

dc_status dc_module_times(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                          const int32_t* group_id, dc_batch* out, float* op_time, float* ar_size, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  dc_status st = cost_call_check(ctx, n_cand);
  if (st != DC_OK) return st;
  if (n_cand > 0 && (!op_time || !ar_size)) return fail(ctx, DC_ERR_INVALID_ARG, "null output array");
  st = dc_contract_graphs(ctx, n_cand, cand_graph, cand_off, group_id, out, stream);
  if (st != DC_OK || n_cand == 0) return st;
  BatchView v{};
  v.node_off = out->node_off;
  v.new_id = out->new_id;
  return do_module_times(ctx, n_cand, cand_graph, cand_off, v, op_time, ar_size, static_cast<hipStream_t>(stream));
}

dc_status dc_cost_candidates(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                             const int32_t* group_id, float ar_c, float ar_d, float* cost, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  dc_status st = cost_call_check(ctx, n_cand);
  if (st != DC_OK) return st;
  if (n_cand == 0) return DC_OK;
  if (!cand_graph || !cand_off || !group_id || !cost) return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  st = do_contract(ctx, n_cand, cand_graph, cand_off, group_id, ctx->ib, s, false);
  if (st != DC_OK) return st;
  st = do_module_times(ctx, n_cand, cand_graph, cand_off, ctx->ib, ctx->m_op_time, ctx->m_ar_size, s);
  if (st != DC_OK) return st;
  return do_simulate(ctx, n_cand, ctx->ib, ctx->m_op_time, ctx->m_ar_size, ar_c, ar_d, cost, s);
}

dc_status dc_search(dc_ctx* ctx, int32_t graph, const dc_search_params* params, int32_t* labels_opt,
                    dc_search_result* res, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!params) return fail(ctx, DC_ERR_INVALID_ARG, "null parameters");
  dc_status st = cost_call_check(ctx, 0);
  if (st != DC_OK) return st;
  const dc_search_params& p = *params;
  if (graph < 0 || graph >= ctx->bg.n_graphs) return fail(ctx, DC_ERR_INVALID_ARG, "graph index out of range");
  if (!(p.alpha >= 1.0f) || p.beta < 0 || p.max_unchanged < 0 || p.parents < 1 || p.max_queue < 1 || p.max_steps < 0)
    return fail(ctx, DC_ERR_INVALID_ARG, "need alpha >= 1, beta >= 0, parents >= 1, max_queue >= 1");
  if (p.op_draw != DC_DRAW_DEPENDENCY && p.op_draw != DC_DRAW_OP)
    return fail(ctx, DC_ERR_INVALID_ARG, "op_draw must be DC_DRAW_DEPENDENCY or DC_DRAW_OP");
  SearchView g;
  g.n = ctx->h_gno[graph + 1] - ctx->h_gno[graph];
  g.e = ctx->h_geo[graph + 1] - ctx->h_geo[graph];
  g.rowptr = ctx->bg.rowptr + ctx->h_gno[graph] + graph;
  g.col = ctx->bg.col + ctx->h_geo[graph];
  g.ar_size = ctx->fo.ar_size_base + ctx->h_gno[graph];
  const long long kids = 2LL * p.parents;
  if (kids > ctx->cfg.max_cand || kids * g.n > ctx->cfg.max_base_nodes || kids * g.e > ctx->cfg.max_base_edges)
    return fail(ctx, DC_ERR_CAPACITY, "the context must hold 2 * parents candidates of this graph per call");
  if (g.n == 0) return fail(ctx, DC_ERR_INVALID_ARG, "empty graph");
  st = run_search(ctx, g, graph, p, labels_opt, res, static_cast<hipStream_t>(stream));
  if (st == DC_ERR_UNSUPPORTED && ctx->err.empty()) ctx->err = "the graph is too large for the mutation kernel's LDS with this op_draw";
  if (st != DC_OK && ctx->err.empty()) ctx->err = "search failed";
  return st;
}

dc_status dc_last_fused_ops(dc_ctx* ctx, int64_t* n_fused_ops, int64_t* n_rows, int64_t* n_edges, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!ctx->have_profile) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_profile has not been called");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(ctx->h_pinned + 8, ctx->fo.totals, 8 * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "dc_last_fused_ops");
  if (n_rows) *n_rows = ctx->h_pinned[8 + 1];
  if (n_fused_ops) *n_fused_ops = ctx->h_pinned[8 + 3];
  if (n_edges) *n_edges = ctx->h_pinned[8 + 4];
  return DC_OK;
}

dc_status dc_last_fused_op_repeats(dc_ctx* ctx, int64_t* n_repeats, void* stream) {
  if (!ctx || !n_repeats) return DC_ERR_INVALID_ARG;
  if (!ctx->have_profile) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_profile has not been called");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(ctx->h_pinned + 8, ctx->fo.totals, 8 * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "dc_last_fused_op_repeats");
  *n_repeats = ctx->every_fused_op ? 0 : ctx->h_pinned[8 + 5];
  return DC_OK;
}

// ---------------------------------------------------------------------------
// training of the estimator
// ---------------------------------------------------------------------------
namespace {
__global__ void zero_kernel(float* p, long long n) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

size_t n_layer_weights(const dc_config& c) { return packed_weight_elems(c.F, c.H, c.L, 3); }
size_t n_head_params(const dc_config& c) { return 2 * (size_t)c.H * c.H + 3 * (size_t)c.H + 1; }

dc_status train_ready(dc_ctx* ctx, const dc_batch* in) {
  if (!ctx->training) return fail(ctx, DC_ERR_INVALID_ARG, "dc_train_begin has not been called");
  if (!in || in->n_cand < 0) return fail(ctx, DC_ERR_INVALID_ARG, "null batch or negative count");
  if (in->n_cand > ctx->tp.max_samples) return fail(ctx, DC_ERR_CAPACITY, "the batch has more graphs than max_samples");
  return DC_OK;
}

// forward, loss and (with a gradient vector) the reverse pass over one batch
dc_status train_pass(dc_ctx* ctx, const dc_batch* in, const float* target, float* loss, float* pred, float* grad,
                     hipStream_t s) {
  if (!target || !loss || !in->node_off || !in->out_rowptr || !in->out_col || !in->in_rowptr || !in->in_col || !in->Xc)
    return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  const long long cap = in->cap_nodes < ctx->tp.max_rows ? in->cap_nodes : ctx->tp.max_rows;
  hipLaunchKernelGGL(check_batch_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, s, in->node_off, in->n_cand, cap,
                     (long long)in->cap_edges, in->out_rowptr, in->out_col, in->in_rowptr, in->in_col, ctx->status);
  TrainPass t = ctx->tb;
  t.n_samples = in->n_cand;
  t.node_off = in->node_off;
  t.out_rowptr = in->out_rowptr;
  t.out_col = in->out_col;
  t.in_rowptr = in->in_rowptr;
  t.in_col = in->in_col;
  t.X = static_cast<const float*>(in->Xc);
  t.target = target;
  t.W = static_cast<const float*>(ctx->W);
  t.b = ctx->b;
  t.head = ctx->head;
  t.grad = grad;
  t.loss = loss;
  t.pred = pred;
  hipError_t e = launch_train_pass(t, ctx->prof.on ? &ctx->prof : nullptr, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "training pass launch");
  return DC_OK;
}
}  // namespace

int64_t dc_num_params(const dc_ctx* ctx) {
  if (!ctx || ctx->cfg.aggregator != DC_AGG_MEAN) return 0;
  return (int64_t)(n_layer_weights(ctx->cfg) + (size_t)ctx->cfg.L * ctx->cfg.H + n_head_params(ctx->cfg));
}

dc_status dc_train_begin(dc_ctx* ctx, const dc_train_params* params, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!params) return fail(ctx, DC_ERR_INVALID_ARG, "null parameters");
  const dc_config& c = ctx->cfg;
  if (c.dtype != DC_F32 || c.aggregator != DC_AGG_MEAN)
    return fail(ctx, DC_ERR_UNSUPPORTED, "training needs a DC_F32 context with DC_AGG_MEAN");
  if (!ctx->have_weights) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_weights has not been called");
  const dc_train_params& p = *params;
  if (!(p.lr >= 0.f) || !(p.beta1 >= 0.f && p.beta1 < 1.f) || !(p.beta2 >= 0.f && p.beta2 < 1.f) || !(p.eps > 0.f) ||
      !(p.floor > 0.f))
    return fail(ctx, DC_ERR_INVALID_ARG, "need lr >= 0, 0 <= beta < 1, eps > 0, floor > 0");
  const Caps k = caps_of(c);
  if (p.max_samples < 1 || p.max_rows < 1) return fail(ctx, DC_ERR_INVALID_ARG, "max_samples and max_rows must be positive");
  if (p.max_rows > k.NN) return fail(ctx, DC_ERR_CAPACITY, "max_rows exceeds the context's max_nodes");
  if (p.max_samples > INT32_MAX / 2 || p.max_rows * 3 * (long long)c.H > (1LL << 40))
    return fail(ctx, DC_ERR_CAPACITY, "training batch too large");
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipStreamSynchronize(s);
  if (ctx->train_mem) (void)hipFree(ctx->train_mem);
  ctx->train_mem = nullptr;
  ctx->training = false;
  const size_t R = (size_t)p.max_rows, B = (size_t)p.max_samples, H = (size_t)c.H;
  const size_t dmax = (size_t)(c.F > c.H ? c.F : c.H);
  const size_t P = (size_t)dc_num_params(ctx);
  const int S = train_slabs(ctx->n_cu, c.F, c.H);
  TrainPass t{};
  float *m = nullptr, *v = nullptr;
  for (int pass = 0; pass < 2; ++pass) {
    Arena a;
    a.base = pass ? ctx->train_mem : nullptr;
    t.hs = a.take<float>((size_t)c.L * R * H);
    t.means = a.take<float>((size_t)c.L * 2 * R * dmax);
    t.dA = a.take<float>(R * 3 * H);
    t.R = a.take<float>(B * H);
    t.Z1 = a.take<float>(B * H);
    t.Z2 = a.take<float>(B * H);
    t.dZ2 = a.take<float>(B * H);
    t.dZ1 = a.take<float>(B * H);
    t.dR = a.take<float>(B * H);
    t.y = a.take<float>(B);
    t.dy = a.take<float>(B);
    t.lterm = a.take<double>(B);
    t.gid = a.take<int>(R);
    t.cnt = a.take<int>(2);
    t.WT = a.take<float>(3 * H * H);
    t.part = a.take<float>((size_t)S * (3 * dmax * H + H));
    t.grad = a.take<float>(P);
    m = a.take<float>(P);
    v = a.take<float>(P);
    if (!pass) {
      hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->train_mem), a.off);
      if (e != hipSuccess) {
        ctx->train_mem = nullptr;
        return hip_fail(ctx, e, "training buffers");
      }
    }
  }
  t.F = c.F;
  t.H = c.H;
  t.L = c.L;
  t.floor = p.floor;
  t.dZ[0] = static_cast<float*>(ctx->act[0]);
  t.dZ[1] = static_cast<float*>(ctx->act[1]);
  t.slabs = S;
  t.max_rows = p.max_rows;
  t.status = ctx->status;
  t.n_cu = ctx->n_cu;
  ctx->tb = t;
  ctx->adam_m = m;
  ctx->adam_v = v;
  ctx->tp = p;
  ctx->train_t = 0;
  hipLaunchKernelGGL(zero_kernel, dim3(256), dim3(256), 0, s, m, (long long)P);
  hipLaunchKernelGGL(zero_kernel, dim3(256), dim3(256), 0, s, v, (long long)P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "training state");
  ctx->training = true;
  return DC_OK;
}

dc_status dc_fused_op_batch(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                            const int32_t* group_id, dc_batch* out, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  dc_status st = cost_call_check(ctx, n_cand);
  if (st != DC_OK) return st;
  if (!out) return fail(ctx, DC_ERR_INVALID_ARG, "null batch");
  if (!out->node_off || !out->edge_off || !out->new_id || !out->out_rowptr || !out->out_col || !out->in_rowptr ||
      !out->in_col || !out->Xc || out->cap_nodes < 0 || out->cap_edges < 0)
    return fail(ctx, DC_ERR_INVALID_ARG, "dc_batch has a null array or negative capacity");
  out->n_cand = 0;
  if (n_cand == 0) return DC_OK;
  if (!cand_graph || !cand_off || !group_id) return fail(ctx, DC_ERR_INVALID_ARG, "null candidate array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(1), 0, s, ctx->status);
  st = do_contract(ctx, n_cand, cand_graph, cand_off, group_id, ctx->ib, s, false);
  if (st != DC_OK) return st;
  Profiler* prof = ctx->prof.on ? &ctx->prof : nullptr;
  FusedOpsArgs a = ctx->fo;
  a.bg = ctx->bg;
  a.n_cand = n_cand;
  a.cand_graph = cand_graph;
  a.cand_off = cand_off;
  a.members = ctx->tmp.members;
  a.mstart = ctx->tmp.mstart;
  a.Gc = ctx->tmp.Gc;
  a.new_id = ctx->ib.new_id;
  a.c_node_off = ctx->ib.node_off;
  a.op_time = ctx->m_op_time;
  a.ar_size = ctx->m_ar_size;
  a.table = nullptr;                        // every fused op is a sample of its own
  // the batch goes to the caller's arrays, within the caller's capacities
  a.fb.node_off = out->node_off;
  a.fb.edge_off = out->edge_off;
  a.fb.new_id = out->new_id;
  a.fb.out_rowptr = out->out_rowptr;
  a.fb.out_col = out->out_col;
  a.fb.in_rowptr = out->in_rowptr;
  a.fb.in_col = out->in_col;
  a.fb.Xc = out->Xc;
  a.fb.cap_nodes = out->cap_nodes;
  a.fb.cap_edges = out->cap_edges;
  if (out->cap_nodes < a.cap_rows) a.cap_rows = out->cap_nodes;
  if (out->cap_edges < a.cap_edges) a.cap_edges = out->cap_edges;
  if (out->cap_nodes / 2 + 1 < a.cap_ops) a.cap_ops = out->cap_nodes / 2 + 1;
  hipError_t e = launch_fused_op_extract(a, prof, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "fused-op extraction launch");
  int64_t K = 0;
  st = dc_last_fused_ops(ctx, &K, nullptr, nullptr, stream);
  if (st != DC_OK) return st;
  st = dc_check(ctx, stream);
  if (st != DC_OK) return st;
  out->n_cand = (int32_t)K;
  return DC_OK;
}

dc_status dc_loss_gradients(dc_ctx* ctx, const dc_batch* in, const float* target, float* loss, float* pred,
                            float* grad, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  dc_status st = train_ready(ctx, in);
  if (st != DC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!loss) return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  if (in->n_cand == 0) {
    hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(64), 0, s, loss, 1LL);
    if (grad) hipLaunchKernelGGL(zero_kernel, dim3(256), dim3(256), 0, s, grad, (long long)dc_num_params(ctx));
    return DC_OK;
  }
  // the reverse pass writes the context's gradient vector; a caller's array receives a copy
  st = train_pass(ctx, in, target, loss, pred, grad ? ctx->tb.grad : nullptr, s);
  if (st != DC_OK || !grad) return st;
  hipError_t e = hipMemcpyAsync(grad, ctx->tb.grad, (size_t)dc_num_params(ctx) * sizeof(float),
                                hipMemcpyDeviceToDevice, s);
  return e == hipSuccess ? DC_OK : hip_fail(ctx, e, "gradient copy");
}

dc_status dc_train_step(dc_ctx* ctx, const dc_batch* in, const float* target, float* loss, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  dc_status st = train_ready(ctx, in);
  if (st != DC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!loss) return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  if (in->n_cand == 0) {
    hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(64), 0, s, loss, 1LL);
    return DC_OK;
  }
  st = train_pass(ctx, in, target, loss, nullptr, ctx->tb.grad, s);
  if (st != DC_OK) return st;
  const dc_config& c = ctx->cfg;
  const dc_train_params& p = ctx->tp;
  const long long tstep = ++ctx->train_t;
  const double c1 = 1.0 / (1.0 - pow((double)p.beta1, (double)tstep));
  const double c2 = 1.0 / (1.0 - pow((double)p.beta2, (double)tstep));
  const long long nW = (long long)n_layer_weights(c), nb = (long long)c.L * c.H, nh = (long long)n_head_params(c);
  const float* g = ctx->tb.grad;
  if (ctx->prof.on) ctx->prof.begin(kFamTrainAdam, s);
  hipError_t e = launch_adam(static_cast<float*>(ctx->W), g, ctx->adam_m, ctx->adam_v, nW, p.lr, p.beta1, p.beta2,
                             p.eps, c1, c2, ctx->status, s);
  if (e == hipSuccess)
    e = launch_adam(ctx->b, g + nW, ctx->adam_m + nW, ctx->adam_v + nW, nb, p.lr, p.beta1, p.beta2, p.eps, c1, c2,
                    ctx->status, s);
  if (e == hipSuccess)
    e = launch_adam(ctx->head, g + nW + nb, ctx->adam_m + nW + nb, ctx->adam_v + nW + nb, nh, p.lr, p.beta1, p.beta2,
                    p.eps, c1, c2, ctx->status, s);
  if (ctx->prof.on) ctx->prof.end(s);
  // the copy of W1 | W2 that the fused-op path multiplies with (same layout in fp32)
  const size_t HH = (size_t)c.H * c.H;
  if (e == hipSuccess) e = hipMemcpyAsync(ctx->headW, ctx->head, HH * sizeof(float), hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess)
    e = hipMemcpyAsync(static_cast<float*>(ctx->headW) + HH, ctx->head + HH + c.H, HH * sizeof(float),
                       hipMemcpyDeviceToDevice, s);
  return e == hipSuccess ? DC_OK : hip_fail(ctx, e, "optimiser step");
}

dc_status dc_get_weights(dc_ctx* ctx, float* W_layers, float* b_layers, float* head, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  if (!W_layers || !b_layers || !head) return fail(ctx, DC_ERR_INVALID_ARG, "null array");
  const dc_config& c = ctx->cfg;
  if (c.dtype != DC_F32 || c.aggregator != DC_AGG_MEAN)
    return fail(ctx, DC_ERR_UNSUPPORTED, "dc_get_weights needs a DC_F32 context with DC_AGG_MEAN");
  if (!ctx->have_weights) return fail(ctx, DC_ERR_INVALID_ARG, "dc_set_weights has not been called");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(W_layers, ctx->W, n_layer_weights(c) * sizeof(float), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess)
    e = hipMemcpyAsync(b_layers, ctx->b, (size_t)c.L * c.H * sizeof(float), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipMemcpyAsync(head, ctx->head, n_head_params(c) * sizeof(float), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  return e == hipSuccess ? DC_OK : hip_fail(ctx, e, "dc_get_weights");
}

dc_status dc_check(dc_ctx* ctx, void* stream) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(ctx->h_pinned, ctx->status, 2 * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipMemsetAsync(ctx->status + 1, 0, sizeof(int), s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "dc_check");
  const int code = ctx->h_pinned[1];
  if (code != 0) {
    ctx->err = code == DC_ERR_BAD_PARTITION ? "device: label out of range or candidate/base-graph mismatch"
             : code == DC_ERR_CAPACITY      ? "device: sizes exceed the configured or provided capacity"
             : code == DC_ERR_BAD_GRAPH     ? "device: batch malformed (offsets, row pointers or a neighbour out of its graph)"
                                            : "device: error";
  }
  return static_cast<dc_status>(code);
}

dc_status dc_last_totals(dc_ctx* ctx, int64_t* n_nodes, int64_t* n_edges, void* stream) {
  if (!ctx || !n_nodes || !n_edges) return DC_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(ctx->h_pinned + 8, ctx->totals, 2 * sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e, "dc_last_totals");
  *n_nodes = ctx->h_pinned[8];
  *n_edges = ctx->h_pinned[9];
  return DC_OK;
}

dc_status dc_select_kernels(dc_ctx* ctx, int32_t which) {
  if (!ctx || which < 0 || which > 3) return DC_ERR_INVALID_ARG;
  ctx->allow_fused = !(which & DC_KERNELS_SEPARATE_LAYERS);
  ctx->every_fused_op = (which & DC_KERNELS_EVERY_FUSED_OP) != 0;
  return DC_OK;
}

const char* dc_last_error(const dc_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

dc_status dc_profile_begin(dc_ctx* ctx) {
  if (!ctx) return DC_ERR_INVALID_ARG;
  ctx->prof.on = true;
  ctx->prof.n = 0;
  return DC_OK;
}

int32_t dc_profile_end(dc_ctx* ctx, const char** names, float* total_ms, int32_t* launches, int32_t cap) {
  if (!ctx) return 0;
  ctx->prof.on = false;
  float ms[kFamCount] = {0};
  int cnt[kFamCount] = {0};
  for (int i = 0; i < ctx->prof.n; ++i) {
    if (hipEventSynchronize(ctx->prof.ev[2 * i + 1]) != hipSuccess) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, ctx->prof.ev[2 * i], ctx->prof.ev[2 * i + 1]) == hipSuccess) {
      ms[ctx->prof.fam[i]] += t;
      cnt[ctx->prof.fam[i]] += 1;
    }
  }
  ctx->prof.n = 0;
  for (int f = 0; f < kFamCount && f < cap; ++f) {
    if (names) names[f] = kFamilyNames[f];
    if (total_ms) total_ms[f] = ms[f];
    if (launches) launches[f] = cnt[f];
  }
  return kFamCount;
}

}  // extern "C"

/* disco.h -- C ABI of the MI355X fusion-candidate evaluator.
 *
 * The strategy search of the paper (Alg. 1) repeatedly asks a cost model
 * Cost(H') for the per-iteration training time of a candidate module H': the
 * base module H_in with an op-fusion strategy and a tensor-fusion strategy
 * applied (Sec. 3.2).  This library evaluates batches of such candidates on
 * one GPU.  A candidate is a base training DAG (compute ops plus gradient
 * all-reduce tensors) and one integer label per base node; nodes with equal
 * labels form one fused op / one fused gradient tensor.
 *
 *   dc_contract_graphs  builds the candidate modules: per candidate the
 *                       quotient graph by label (Sec. 3.3: a fused op is the
 *                       subgraph of its original ops; dependencies that cross
 *                       groups remain) with summed node features (Sec. 2.3:
 *                       the size of a fused tensor is the sum of its members'
 *                       sizes; every feature column is summed).
 *   dc_gnn_forward      runs the estimator on a batch of contracted graphs:
 *                       per layer the mean over predecessors and the mean
 *                       over successors next to the node's own vector, a
 *                       linear map, bias and ReLU (Sec. 3.3.1, neighbourhood
 *                       encoding); a sum over all nodes of each graph
 *                       (Sec. 3.3.1, second equation); fully connected layers
 *                       with ReLU and a scalar output (Sec. 3.3.2).
 *   dc_eval_candidates  = contract + forward: one estimate per candidate module.
 *   dc_simulate         list scheduling of the candidate modules (Sec. 3.4).
 *   dc_cost_candidates  Cost(H') as the paper composes it (Sec. 3.1, Simulator): the
 *                       estimator on every fused op, profiled times for single ops,
 *                       the linear model for (fused) all-reduce tensors, then
 *                       dc_simulate.
 *   dc_train_step       one step of the estimator's supervised training on a batch of
 *                       fused ops with profiled times (Sec. 3.3.3: loss of Eq. (1), Adam).
 *
 * Conventions
 *  - Every call returns a dc_status; nothing throws or aborts.
 *  - "host" pointers are read synchronously during the call.  "dev" pointers
 *    are device memory owned by the caller (e.g. torch tensors) and are
 *    read/written asynchronously on `stream` (a hipStream_t passed as void*,
 *    NULL = default stream).  Outputs are valid once the stream has reached
 *    the end of the call's work.
 *  - Errors the host can see (null pointer, negative size, shapes the kernels
 *    do not support, capacity exceeded by host-known sizes) return at once
 *    with nothing enqueued.  Errors only the device can see (label outside
 *    [0,N), candidate/base-graph mismatch, contracted totals above capacity)
 *    set a device status word; the affected call writes no further output and
 *    dc_check() reports it.
 *  - The library never validates that a fusion is legal (fusible op kinds, no
 *    dependency cycle): the search checks validity before it calls Cost()
 *    (Alg. 1, "if H' is valid").  Contraction and forward pass are defined
 *    for every labelling.
 *  - All integer arrays are int32.  Limits: a base graph has fewer than 65536
 *    nodes; all totals fit in int32; F is a multiple of 16, H a multiple of 32, both <= 512.
 *  - Calls on one dc_ctx must not overlap (the context owns scratch memory).
 */
#ifndef DISCO_H_
#define DISCO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dc_ctx dc_ctx; /* opaque; owns device copies of base graphs, weights and scratch */

typedef enum {
  DC_OK = 0,
  DC_ERR_INVALID_ARG = 1,   /* null pointer, negative size, call order                        */
  DC_ERR_BAD_GRAPH = 2,     /* base graph malformed (rowptr not monotone, col out of range)   */
  DC_ERR_BAD_PARTITION = 3, /* label outside [0,N) or candidate length != base graph size     */
  DC_ERR_CAPACITY = 4,      /* sizes exceed what dc_config / the dc_batch buffers allow        */
  DC_ERR_OOM = 5,           /* device allocation failed                                       */
  DC_ERR_HIP = 6,           /* a HIP runtime call failed (see dc_last_error)                  */
  DC_ERR_UNSUPPORTED = 7    /* shape outside the limits listed above                          */
} dc_status;

typedef enum { DC_F32 = 0, DC_BF16 = 1 } dc_dtype;

/* How a layer combines a node's neighbourhood (Sec. 3.3.1, first equation).
 *   DC_AGG_MEAN       uniform coefficients: mean over predecessors and mean over successors,
 *                     each with its own weight block next to the node's own (the default).
 *   DC_AGG_ATTENTION  K heads with attention coefficients over N_i = (i, predecessors,
 *                     successors).  The paper prints no formula for the coefficients; they
 *                     are taken as in graph attention networks:
 *                       z_j = W e'_j,  u_ij = LeakyReLU_0.2(a_src . z_i + a_dst . z_j) per head,
 *                       gamma_ij = softmax over j in N_i,  e_i = ReLU(sum_j gamma_ij z_j + b),
 *                     heads being contiguous blocks of H / heads columns.  A node that is both a
 *                     predecessor and a successor of i is in N_i twice.                          */
typedef enum { DC_AGG_MEAN = 0, DC_AGG_ATTENTION = 1 } dc_aggregator;

/* Model shape and per-call capacities.
 *   F, H, L          input features, hidden width, number of message-passing layers
 *   dtype            DC_F32: fp32 storage and fp32 matrix arithmetic.
 *                    DC_BF16: contracted features, activations, both means and the
 *                    layer/head matrices are bfloat16 (round to nearest even);
 *                    sums, means, matrix accumulation, bias, ReLU and the head are fp32.
 *                    The sum over a graph's nodes (Sec. 3.3.1, second equation) and the head's
 *                    dot products are accumulated in fp64; with DC_BF16, H = 256 and
 *                    DC_AGG_MEAN the node sum first adds each run of 64 consecutive rows in
 *                    fp32 in one fixed order (the last layer's kernel forms these partial
 *                    sums itself and writes no node embeddings), then the runs in fp64.
 *   max_cand         candidates per call
 *   max_base_nodes   bound on sum over candidates of base-graph node counts (= labels per call)
 *   max_base_edges   bound on sum over candidates of base-graph edge counts
 *   max_nodes        bound on contracted nodes per call; 0 means max_base_nodes
 *   max_edges        bound on contracted edges per call; 0 means max_base_edges
 *   aggregator       dc_aggregator; DC_AGG_ATTENTION needs H a power of two in [32, 512]
 *   heads            K (attention only): a power of two with H / K >= 8; ignored for the mean */
typedef struct {
  int32_t F, H, L;
  int32_t dtype;
  int64_t max_cand;
  int64_t max_base_nodes;
  int64_t max_base_edges;
  int64_t max_nodes;
  int64_t max_edges;
  int32_t aggregator;
  int32_t heads;
} dc_config;

/* A batch of contracted graphs, block diagonal: candidate c owns nodes
 * [node_off[c], node_off[c+1]) and edges [edge_off[c], edge_off[c+1]).  Groups are
 * numbered by ascending smallest member index.  out_rowptr/out_col list each node's
 * successors, in_rowptr/in_col its predecessors, both ascending; rowptr entries are
 * global edge positions, col entries global node numbers.  All arrays are device
 * memory owned by the caller; cap_* are the caller's allocation sizes.            */
typedef struct {
  int32_t n_cand;      /* written by dc_contract_graphs                                     */
  int64_t cap_nodes;   /* rows available in Xc; out_rowptr/in_rowptr hold cap_nodes+1       */
  int64_t cap_edges;   /* entries available in out_col / in_col                             */
  int32_t* node_off;   /* dev [n_cand+1]                                                    */
  int32_t* edge_off;   /* dev [n_cand+1]                                                    */
  int32_t* new_id;     /* dev [sum of base node counts] contracted node (local) per label   */
  int32_t* out_rowptr; /* dev [cap_nodes+1]                                                 */
  int32_t* out_col;    /* dev [cap_edges]                                                   */
  int32_t* in_rowptr;  /* dev [cap_nodes+1]                                                 */
  int32_t* in_col;     /* dev [cap_edges]                                                   */
  void* Xc;            /* dev [cap_nodes, F] row-major, fp32 or bf16 per dc_config.dtype    */
} dc_batch;

/* Creates a context and allocates all scratch for the given capacities (device memory;
 * see dc_workspace_bytes).  The current HIP device at the time of the call is used.   */
dc_status dc_create(dc_ctx** out, const dc_config* cfg);
dc_status dc_destroy(dc_ctx* ctx);

/* Device bytes dc_create will allocate for cfg (excluding base graphs and weights). */
size_t dc_workspace_bytes(const dc_config* cfg);

/* Estimator weights, host fp32; the context keeps a converted device copy.
 *   W_layers  concat over l of W^l, row-major [3d, H], d = F for l = 0 else H; rows
 *             [0,d) act on the node's own vector, [d,2d) on the predecessor mean,
 *             [2d,3d) on the successor mean.
 *   b_layers  concat of b^l [H].
 *   head      W1[H,H] | b1[H] | W2[H,H] | b2[H] | w3[H] | b3[1], W row-major [in,out]:
 *             z1 = ReLU(r W1 + b1), z2 = ReLU(z1 W2 + b2), t = z2.w3 + b3.              */
dc_status dc_set_weights(dc_ctx* ctx, const float* W_layers, const float* b_layers, const float* head,
                         void* stream);

/* Weights of a context created with DC_AGG_ATTENTION (dc_set_weights is for DC_AGG_MEAN; each
 * returns DC_ERR_INVALID_ARG on a context of the other kind).  Host fp32.
 *   W_layers  concat over l of W^l, row-major [d, H], d = F for l = 0 else H.
 *   att       concat over l of a_src^l [H] | a_dst^l [H]; head k owns columns [k H/K, (k+1) H/K).
 *   b_layers  concat of b^l [H];  head as for dc_set_weights.
 * On the bf16 path W and the head matrices are rounded to bfloat16, z = W e' is stored as
 * bfloat16; scores, softmax and the weighted sums are fp32.                                  */
dc_status dc_set_attention_weights(dc_ctx* ctx, const float* W_layers, const float* att, const float* b_layers,
                                   const float* head, void* stream);

/* Base graphs (set once, candidates refer to them by index).  All host pointers.
 *   g_node_off [n+1], g_edge_off [n+1]  node / edge offsets of the graphs
 *   rowptr     concatenated per-graph CSR row pointers: graph b has N_b+1 entries
 *              starting at position g_node_off[b] + b, values relative to the graph (start 0)
 *   col        concatenated successor lists, local node numbers; graph b at g_edge_off[b]
 *   X          [sum N_b, F] fp32 node features
 * Rows need not be sorted or duplicate free.  Returns DC_ERR_BAD_GRAPH on malformed input. */
dc_status dc_set_base_graphs(dc_ctx* ctx, int32_t n_graphs, const int32_t* g_node_off,
                             const int32_t* g_edge_off, const int32_t* rowptr, const int32_t* col,
                             const float* X, void* stream);

/* Contracts n_cand candidates.  cand_graph dev [n_cand] base-graph index; cand_off dev
 * [n_cand+1] offsets into group_id (cand_off[c+1]-cand_off[c] must equal the node count
 * of graph cand_graph[c]); group_id dev labels in [0, N).  Fills every array of *out
 * (host struct, device arrays) and sets out->n_cand.                                   */
dc_status dc_contract_graphs(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph,
                             const int32_t* cand_off, const int32_t* group_id, dc_batch* out, void* stream);

/* Forward pass over a batch laid out as above (typically the output of
 * dc_contract_graphs; node_off[n_cand] must not exceed the context's max_nodes).
 * The batch is validated on the device first (offsets ascending from 0, every graph
 * below 65536 nodes, row pointers ascending within cap_edges, every neighbour inside its
 * own graph); a violation makes the call a no-op that dc_check reports as
 * DC_ERR_BAD_GRAPH or DC_ERR_CAPACITY.
 * pred dev [n_cand] fp32: predicted per-iteration time per candidate.            */
dc_status dc_gnn_forward(dc_ctx* ctx, const dc_batch* in, float* pred, void* stream);

/* End-to-end time of each candidate module by list scheduling (Sec. 3.4): computation nodes
 * run one at a time on one device in FIFO order of a ready queue (a node enters the tail when
 * its last dependency clears and starts when the device is free and its predecessors are
 * done); all-reduce nodes run one at a time on a communication channel in the order in
 * which their tensors are produced, each for T = ar_c * size + ar_d (Sec. 3.1, Profiler),
 * overlapping with computation; the result is the later of the two ends.  Where the text is
 * silent: the queue starts with the source nodes in ascending index; an all-reduce goes on
 * the channel the moment its last predecessor is processed, before the next node is taken,
 * ties in ascending index; successors are released in ascending index.
 *   in        a batch as produced by dc_contract_graphs (validated on the device as for
 *             dc_gnn_forward; Xc and new_id are not read)
 *   op_time   dev [node_off[n_cand]] fp32: execution time of each computation node (profiled,
 *             or predicted by an estimator for fused ops); ignored for all-reduce nodes
 *   ar_size   dev [node_off[n_cand]] fp32: tensor size of each all-reduce node; negative marks
 *             a computation node
 *   cost      dev [n_cand] fp32; +infinity for a module whose graph has a cycle (an invalid
 *             fusion).  Times are accumulated in fp64 in the order the rules fix.
 * Needs dc_set_base_graphs (their sizes bound the scratch); no weights.  A graph larger than
 * every base graph of the context is reported by dc_check as DC_ERR_CAPACITY.            */
dc_status dc_simulate(dc_ctx* ctx, const dc_batch* in, const float* op_time, const float* ar_size, float ar_c,
                      float ar_d, float* cost, void* stream);

/* dc_simulate for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It takes no context and calls neither hipMalloc nor
 * hipFree nor any allocating routine: the status words and the working sets of modules too large for
 * LDS live in a device array that is part of the library itself (16 MiB + 256 bytes, held by every GPU
 * the library runs on until the process ends).  Arguments as for dc_simulate, with
 *   in                a caller's batch (node_off, out_rowptr, out_col, in_rowptr, in_col, n_cand,
 *                     cap_nodes and cap_edges = the lengths of the node and edge arrays); validated
 *                     on the device as dc_simulate does
 *   max_module_nodes, max_module_edges   the caller's bound on the largest module of the batch.
 *                     Limit: 24 bytes per node + 2 bytes per edge must not exceed 256 KiB (e.g.
 *                     9000 nodes with 20000 edges); beyond it the call returns DC_ERR_CAPACITY with
 *                     nothing enqueued (dc_simulate_static_error says why).  A module that exceeds
 *                     what the caller stated, but not the limit, is still simulated; one that
 *                     exceeds the limit gets cost +infinity and the status DC_ERR_CAPACITY
 *   dev_status        dev [1] or null: receives the first device-detected error of this call
 *                     (DC_OK, DC_ERR_BAD_GRAPH, DC_ERR_CAPACITY)
 * Results are those of dc_simulate, bit for bit.  Asynchronous on `stream`; the current HIP device is
 * used.  All calls on one GPU share the one array, which keeps the contents of the last call (what
 * must start at zero is cleared by a kernel at the start of each call): calls that overlap on one GPU,
 * on different streams or from different threads, race -- serialise them.                          */
dc_status dc_simulate_static(const dc_batch* in, int32_t max_module_nodes, int32_t max_module_edges,
                             const float* op_time, const float* ar_size, float ar_c, float ar_d, float* cost,
                             int32_t* dev_status, void* stream);
/* Detail of the last error dc_simulate_static returned on this thread; owned by the library. */
const char* dc_simulate_static_error(void);

/* Profiled data of the base graphs (Sec. 3.1, Profiler), host fp32 arrays over all base nodes in
 * the order of X in dc_set_base_graphs:
 *   op_time  execution time of each individual op (ignored for all-reduce nodes)
 *   ar_size  tensor size of each gradient all-reduce node; negative marks a computation op
 * Allocates the scratch of the cost path (about 40 bytes per base node and candidate slot plus
 * a feature copy) and must follow dc_set_base_graphs; a later dc_set_base_graphs discards it.
 * The cost path needs every base row strictly ascending (DC_ERR_BAD_GRAPH otherwise) and a
 * context created with max_nodes = max_edges = 0 (DC_ERR_CAPACITY otherwise).            */
dc_status dc_set_profile(dc_ctx* ctx, const float* op_time, const float* ar_size, void* stream);

/* Contracts the candidates into *out (as dc_contract_graphs) and gives every node of the
 * contracted batch what the simulator needs (Sec. 3.1, Simulator; Sec. 3.3):
 *   a group of two or more ops     the estimator's prediction for the fused op, i.e. for the
 *                                  subgraph of its members (ascending base index, their own
 *                                  features, the base edges with both ends in the group):
 *                                  layers, sum over the members, regression network; the
 *                                  result is clamped at zero (Sec. 3.3.2: the network ends in a ReLU)
 *   a single op                    its profiled time
 *   a group of all-reduce tensors  ar_size = sum of the members' sizes (Sec. 2.3; fp64 in
 *                                  ascending member order, rounded once), op_time = 0
 *   ops and tensors mixed          op_time = +infinity (no strategy of Sec. 3.2 produces it)
 * op_time, ar_size: dev [out->cap_nodes] fp32; ar_size is negative for computation nodes.
 * On the bf16 path the sums over members and the two hidden layers of the regression network
 * are stored as bfloat16 (they are inputs of MFMA GEMMs).
 * The candidates of a batch mostly share their fused ops (Alg. 1 mutates a few groups of a
 * parent per child): fused ops of one call with the same base graph and the same members are
 * the same subgraph, so the estimator runs on the first of each kind and the others take its
 * estimate (the same bits as if each had been estimated: a row's arithmetic does not depend on
 * where it stands in the batch).  Nothing is kept from one call to the next.                */
dc_status dc_module_times(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                          const int32_t* group_id, dc_batch* out, float* op_time, float* ar_size, void* stream);

/* Cost(H') of every candidate: dc_module_times into context-owned buffers followed by
 * dc_simulate with T = ar_c * size + ar_d.  cost dev [n_cand] fp32.                      */
dc_status dc_cost_candidates(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                             const int32_t* group_id, float ar_c, float ar_d, float* cost, void* stream);

/* After a synchronised dc_module_times / dc_cost_candidates: how many fused ops the estimator
 * ran on, their member rows and the edges inside them.  Synchronises `stream`.            */
dc_status dc_last_fused_ops(dc_ctx* ctx, int64_t* n_fused_ops, int64_t* n_rows, int64_t* n_edges, void* stream);

/* After the same calls: how many further fused ops of the batch repeated one of those and took
 * its estimate (Sec. 3.3: the estimate depends on the fused op's subgraph only).  Synchronises
 * `stream`.                                                                                 */
dc_status dc_last_fused_op_repeats(dc_ctx* ctx, int64_t* n_repeats, void* stream);

/* Backtracking search over fusion strategies (Alg. 1, Sec. 4) with dc_cost_candidates as Cost().
 * A strategy is a labelling of the nodes of base graph `graph`; the search starts from the
 * all-singleton labelling H_in with H_opt = H_in.  Per step up to `parents` entries leave the
 * priority queue (ascending cost, oldest first); each gets one child per optimisation method:
 *   op fusion      n = Random(0, beta) times, in the form op_draw selects     (Sec. 4, method (i))
 *                  DC_DRAW_DEPENDENCY: a dependency u -> v between two computation ops of the
 *                  base module is drawn uniformly; if its ends are in different groups, the
 *                  group of u joins the group of v.  Needs no view of the current module.
 *                  DC_DRAW_OP (the paper's wording): a computation op of the current module is
 *                  drawn uniformly (the groups of the labelling, in the order of their smallest
 *                  member; low 32 bits of the draw), then one of its predecessor ops in the
 *                  current module uniformly (the groups with a dependency into it, same order;
 *                  high 32 bits), and the predecessor joins the op; an op without predecessors
 *                  leaves the module as it is.  Needs 7 bytes of LDS per base node: graphs of
 *                  more than about 23,000 nodes return DC_ERR_UNSUPPORTED.
 *   tensor fusion  n times: an all-reduce node a and a side are drawn uniformly; the nearest
 *                  bucket on that side in production order joins a's      (Sec. 4, method (iii))
 * (method (ii) duplicates an op; a labelling cannot express that).  The children of a step are
 * costed together and then handled in order: a child with a finite cost (a cyclic module costs
 * +infinity) replaces H_opt when cheaper, which restarts the counter of unchanged evaluations,
 * otherwise the counter grows; it is enqueued when Cost(H') <= alpha * Cost(H_opt).  The search
 * ends when the queue is empty, when the counter has reached max_unchanged (checked between
 * steps) or after max_steps steps.  parents = 1 is the loop as the paper prints it.  A queue
 * above max_queue entries drops its most expensive ones.
 * Draws: key = mix(seed ^ mix(step * 2^32 + child)), draw d = mix(key + d * 0xD1342543DE82EF95),
 * mix = the output function of splitmix64; draw 0 mod (beta + 1) is n, draws 1.. mod the number
 * of choices pick the applications (tensor fusion takes the side from bit 32 of its draw).
 * Needs dc_set_profile and capacities for 2 * parents candidates of this graph per call.
 * labels_opt: host [N] out (may be NULL); res: host out.  Allocates its own device buffers
 * ((max_queue + 4 * parents) * N labels) for the duration of the call and synchronises `stream`
 * once per step.                                                                            */
enum { DC_DRAW_DEPENDENCY = 0, DC_DRAW_OP = 1 };
typedef struct {
  float alpha;           /* >= 1 */
  int32_t beta;          /* >= 0 */
  int32_t max_unchanged; /* the paper uses 1000 */
  int32_t parents;       /* >= 1 */
  int32_t max_queue;     /* >= 1 */
  int64_t max_steps;
  uint64_t seed;
  float ar_c, ar_d;      /* T = ar_c * size + ar_d */
  int32_t op_draw;       /* DC_DRAW_DEPENDENCY or DC_DRAW_OP */
} dc_search_params;
typedef struct {
  float cost_in, cost_opt;
  int64_t steps, evaluated, valid, enqueued, improved, queued, unchanged;
} dc_search_result;
dc_status dc_search(dc_ctx* ctx, int32_t graph, const dc_search_params* params, int32_t* labels_opt,
                    dc_search_result* res, void* stream);

/* ---- Training of the estimator (Sec. 3.3.3; samples as in Sec. 5.1, Fused Op Estimator) ----
 *
 * The graph layers and the regression network are trained together on a set G of fused ops
 * with profiled times y', by Adam on the loss of Eq. (1).  Eq. (1) as printed has no minimum
 * at a perfect fit; it is taken as the mean squared difference of the logarithms,
 *     L = 1/|G| sum_g (log max(y_g, floor) - log y'_g)^2 ,
 * where y_g is the raw output z2.w3 + b3 of the regression network and a sample with
 * y_g <= floor contributes its loss but no gradient.  Training needs a DC_F32, DC_AGG_MEAN
 * context whose weights have been set; it updates those weights in place, so every later
 * dc_gnn_forward / dc_eval_candidates / dc_cost_candidates runs the trained estimator.
 * Arithmetic: fp32 storage and fp32 MFMA accumulation; the sums over the ops of a fused op, the
 * per-sample loss terms and their total are formed in fp64.                                    */
typedef struct {
  float lr, beta1, beta2, eps; /* Adam: m = b1 m + (1-b1) g, v = b2 v + (1-b2) g^2,
                                  theta -= lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps), t from 1 */
  float floor;                 /* > 0                                                                */
  int64_t max_samples;         /* graphs per batch                                                   */
  int64_t max_rows;            /* rows per batch, at most the context's max_nodes                    */
} dc_train_params;

/* Number of fp32 parameters, in the order W_layers | b_layers | head of dc_set_weights. */
int64_t dc_num_params(const dc_ctx* ctx);

/* Allocates the training buffers (device; about (3 L + 6) * max_rows * max(F, H) * 4 bytes), clears both
 * moment vectors and the step count.  May be called again to restart or to change the sizes. */
dc_status dc_train_begin(dc_ctx* ctx, const dc_train_params* params, void* stream);

/* The training set of a list of labelings: contraction as in dc_contract_graphs, then every
 * group of two or more computation ops becomes one graph of `out` (rows = its members in
 * ascending base index with their own features, edges = the base edges with both ends in the
 * group), ordered by candidate and then by contracted node.  out->new_id receives the base
 * node (concatenated numbering) of each row; out->node_off / edge_off need cap_nodes / 2 + 2
 * entries.  Needs dc_set_profile (it tells ops from all-reduce nodes).  Synchronises `stream`
 * and sets out->n_cand to the number of graphs written.                                        */
dc_status dc_fused_op_batch(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                            const int32_t* group_id, dc_batch* out, void* stream);

/* Forward pass, loss and its gradient over one batch of sample graphs (any dc_batch: the
 * output of dc_fused_op_batch or of dc_contract_graphs).  All pointers device memory.
 *   target  [in->n_cand] profiled times, positive and finite; any other value makes the call a
 *           no-op (no loss, no gradient, no update) that dc_check reports as DC_ERR_INVALID_ARG
 *   loss    [1]
 *   pred    [in->n_cand] raw estimates y_g, or null
 *   grad    [dc_num_params] in the order of dc_num_params, or null
 * Nothing is updated.  Needs dc_train_begin.  No host synchronisation.                        */
dc_status dc_loss_gradients(dc_ctx* ctx, const dc_batch* in, const float* target, float* loss, float* pred,
                            float* grad, void* stream);

/* One training step: dc_loss_gradients followed by one Adam update of all parameters in place.
 * An empty batch (n_cand = 0) leaves everything as it is and reports a loss of 0.
 * No host synchronisation: steps may be queued back to back on one stream.  The step count t
 * of Adam's bias correction is host state of the context and enters the update kernel as an
 * argument, so a step must not be replayed from a captured graph.                              */
dc_status dc_train_step(dc_ctx* ctx, const dc_batch* in, const float* target, float* loss, void* stream);

/* Copies the current weights to host arrays laid out as for dc_set_weights (DC_F32 contexts).
 * Synchronises `stream`.                                                                       */
dc_status dc_get_weights(dc_ctx* ctx, float* W_layers, float* b_layers, float* head, void* stream);

/* dc_contract_graphs into context-owned buffers followed by dc_gnn_forward. */
dc_status dc_eval_candidates(dc_ctx* ctx, int32_t n_cand, const int32_t* cand_graph, const int32_t* cand_off,
                             const int32_t* group_id, float* pred, void* stream);

/* Waits for `stream`, then returns the first device-detected error since the last
 * dc_check (DC_OK if none) and clears it.                                          */
dc_status dc_check(dc_ctx* ctx, void* stream);

/* After a synchronised dc_contract_graphs / dc_eval_candidates: totals of the last
 * contraction (contracted nodes, contracted edges).  Synchronises `stream`.        */
dc_status dc_last_totals(dc_ctx* ctx, int64_t* n_nodes, int64_t* n_edges, void* stream);

/* Chooses between kernels that compute the same layer: a diagnostic switch for tests and
 * measurements, never needed to obtain a result.  `which` is 0 (the defaults) or
 *   DC_KERNELS_SEPARATE_LAYERS   neighbour means and node update as two kernels per layer with the
 *                                means written to memory, instead of the fused layer kernels
 *   DC_KERNELS_EVERY_FUSED_OP    dc_module_times / dc_cost_candidates run the estimator on every
 *                                fused op, also on those that repeat an earlier one of the batch
 * or both (bitwise or).  Takes effect from the next call on this context; host state only.     */
enum { DC_KERNELS_SEPARATE_LAYERS = 1, DC_KERNELS_EVERY_FUSED_OP = 2 };
dc_status dc_select_kernels(dc_ctx* ctx, int32_t which);

/* Human-readable detail of the last error on this context; owned by the context. */
const char* dc_last_error(const dc_ctx* ctx);

/* Timing hooks for benchmarks: average milliseconds per launch of each kernel family
 * over the calls made since dc_profile_begin, measured with HIP events on the call's
 * stream.  names/ms receive up to `cap` entries; returns the number of families.
 * Profiling serialises nothing but adds event records; leave it off in production.    */
dc_status dc_profile_begin(dc_ctx* ctx);
int32_t dc_profile_end(dc_ctx* ctx, const char** names, float* total_ms, int32_t* launches, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* DISCO_H_ */

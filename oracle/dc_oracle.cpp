// TEST INFRASTRUCTURE ONLY -- plain, slow, single-threaded CPU oracle for the
// fusion-candidate evaluator.  It shares no code with the HIP library and is
// never called by it; only the tests, the smoke check and the benchmark's CPU
// baseline leg may load this file.
//
// What it computes, written out as the definitions themselves:
//
//  * Contraction of a base training DAG by a fusion labelling.  A fused op is
//    the set of original ops carrying one label, its internal dependencies
//    disappear and the dependencies that cross groups become the edges of the
//    candidate module (Sec. 3.3: a fused op is a subgraph whose nodes are the
//    original ops and whose edges are their dependencies).  A fused gradient
//    tensor has the sum of its members' sizes (Sec. 2.3); every feature
//    column is summed the same way.  The adjacency is 0/1 (Sec. 3.3.1 input
//    (2)), so parallel edges collapse and self loops are dropped.
//    Numbering is a choice of this build: groups are numbered by ascending
//    smallest member index; neighbour lists are ascending.
//
//  * The estimator's forward pass in the fixed architecture of this build:
//    per layer, the mean over predecessors and the mean over successors
//    (neighbourhood encoding, Sec. 3.3.1 first equation, with uniform
//    coefficients and separate weights per direction and for the node
//    itself), a linear map plus bias and ReLU; a sum over all nodes of the
//    graph (Sec. 3.3.1 second equation); then fully connected layers with
//    ReLU and a scalar output (Sec. 3.3.2).
//
//  * The same forward pass with the neighbourhood encoding of Sec. 3.3.1 taken with
//    attention coefficients (orc_gnn_forward_attn).  The paper names K heads, a
//    coefficient gamma^k_ij per neighbour j of i (i included) and one weight
//    matrix W^k per head, but prints no formula for gamma; this build reads it
//    the way graph attention networks do (a reading, labelled as such):
//        z_j = W e'_j,   u^k_ij = LeakyReLU_0.2(a_src^k . z^k_i + a_dst^k . z^k_j),
//        gamma^k_ij = softmax over j in N_i of u^k_ij,
//        e^k_i = ReLU(sum_j gamma^k_ij z^k_j + b^k),
//    heads being contiguous blocks of H/K columns.  N_i is the list
//    (i, predecessors ascending, successors ascending); a node that is both a
//    predecessor and a successor counts twice.
//
//  * End-to-end time of a candidate module by list scheduling (orc_simulate, Sec. 3.4):
//    computation ops run one at a time on one device in the order of a FIFO ready queue
//    (an op enters the tail when its last dependency clears; it starts when the device is
//    free and its predecessors are done); all-reduce instructions run one at a time on a
//    communication channel, in the order in which their tensors are produced, each
//    starting when its tensor is produced (all its predecessors done) and the channel is
//    clear, for T = C x + D (Sec. 3.1, Profiler) with x the tensor size; they overlap with
//    computation.  The result is the later of the two ends.  Choices of this build where
//    the text is silent: the queue starts with the source ops in ascending index; an
//    all-reduce is put on the channel the moment its last predecessor is processed (before
//    the next op is taken from the queue), ties in ascending index; successors of a node
//    are released in ascending index; a module whose graph has a cycle (an invalid fusion)
//    costs +infinity.  All arithmetic in fp64.
//
//  * Cost(H) as the paper composes it (Sec. 3.1, Simulator; Sec. 3.3; Sec. 3.4): the
//    estimator is applied to every fused op, i.e. to the subgraph of its original ops with
//    the dependencies among them (orc_fused_op_batch builds these subgraphs, the forward
//    pass above runs on them as a batch of small graphs); single ops take their profiled
//    time, a (fused) gradient tensor the sum of its members' sizes (orc_module_times);
//    orc_simulate then gives the end-to-end time.  Choices of this build: an estimate is
//    clamped at zero; a group that mixes ops and tensors gets an infinite time.
//
// Numerics: values are stored as fp32, every sum and dot product is
// accumulated in fp64 and rounded once.  With bf16 != 0 the storage points
// that the bf16 device path rounds (contracted features, all activations,
// both means, the layer and head matrices) are rounded to bfloat16
// (round-to-nearest-even); accumulation stays fp64.
//
// Parity pins (tests, CPU only): identity / single-group partitions, the
// dense quotient  [P^T A P > 0] - diag  over all partitions of tiny graphs,
// conservation of feature sums, label-bijection and node-permutation
// invariance, a dense-adjacency float64 forward pass on <= 16 nodes, zero
// weights (bias-only closed form), identity self-weights (readout equals
// column sums), edgeless graphs, and one hand-worked example.  Agreement with
// the paper's *trained* estimator: parity unpinned (no weights or data exist).
// Attention variant: zero attention vectors (closed form: plain mean over N_i),
// a dense masked-softmax float64 formulation on small graphs, a single-node graph,
// invariance to a shift of all scores of a node, and one hand-worked example;
// that gamma has this form in the paper's own code: parity unpinned.
// Simulator: a chain (sum of times), ops only (sum of times whatever the graph), one
// all-reduce behind a chain, two buckets that queue on the channel, overlap of
// communication with computation, the ring closed form for C, a brute-force event
// simulation on random DAGs, cyclic graphs, and one hand-worked example.
// Cost composition: the all-singleton partition (profiled data only), every fused op
// rebuilt on its own from a dense adjacency restricted to its members and evaluated by the
// dense float64 forward pass, closed forms with a constant estimator (bias-only head), the
// clamp, a fused tensor behind one op, mixed groups, label-bijection invariance, and one
// hand-worked example.
#include <cstdint>
#include <cstring>
#include <cmath>
#include <set>
#include <utility>
#include <vector>

namespace {

float round_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) return x;  // inf / nan unchanged
  u += 0x7FFFu + ((u >> 16) & 1u);
  u &= 0xFFFF0000u;
  std::memcpy(&x, &u, 4);
  return x;
}

inline float store(double v, int bf16) {
  float f = static_cast<float>(v);
  return bf16 ? round_bf16(f) : f;
}

// One candidate.  rowptr/col describe the base graph (n nodes), label[v] is
// an arbitrary integer in [0, n).  Outputs use local numbering 0..G-1.
// Returns 0, or 3 when a label is out of range.
int contract_one(int n, const int32_t* rowptr, const int32_t* col, const float* X, int F,
                 const int32_t* label, int bf16,
                 std::vector<int32_t>& new_id, int& G,
                 std::vector<int32_t>& out_rowptr, std::vector<int32_t>& out_col,
                 std::vector<int32_t>& in_rowptr, std::vector<int32_t>& in_col,
                 std::vector<float>& Xc, std::vector<int32_t>& cnt) {
  for (int v = 0; v < n; ++v)
    if (label[v] < 0 || label[v] >= n) return 3;
  // groups numbered in order of first appearance when scanning v upwards
  std::vector<int32_t> id_of_label(n, -1);
  new_id.assign(n, 0);
  G = 0;
  for (int v = 0; v < n; ++v) {
    if (id_of_label[label[v]] < 0) id_of_label[label[v]] = G++;
    new_id[v] = id_of_label[label[v]];
  }
  // feature sums and member counts
  std::vector<double> acc(static_cast<size_t>(G) * F, 0.0);
  cnt.assign(G, 0);
  for (int v = 0; v < n; ++v) {
    cnt[new_id[v]] += 1;
    for (int f = 0; f < F; ++f) acc[static_cast<size_t>(new_id[v]) * F + f] += X[static_cast<size_t>(v) * F + f];
  }
  Xc.resize(static_cast<size_t>(G) * F);
  for (size_t i = 0; i < Xc.size(); ++i) Xc[i] = store(acc[i], bf16);
  // edge set of the quotient graph
  std::set<std::pair<int32_t, int32_t>> fwd, bwd;
  for (int u = 0; u < n; ++u)
    for (int e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      int32_t a = new_id[u], b = new_id[col[e]];
      if (a != b) {
        fwd.insert({a, b});
        bwd.insert({b, a});
      }
    }
  out_rowptr.assign(G + 1, 0);
  in_rowptr.assign(G + 1, 0);
  out_col.clear();
  in_col.clear();
  for (const auto& p : fwd) {
    out_rowptr[p.first + 1] += 1;
    out_col.push_back(p.second);
  }
  for (const auto& p : bwd) {
    in_rowptr[p.first + 1] += 1;
    in_col.push_back(p.second);
  }
  for (int g = 0; g < G; ++g) {
    out_rowptr[g + 1] += out_rowptr[g];
    in_rowptr[g + 1] += in_rowptr[g];
  }
  return 0;
}

// Sum over the nodes of each graph (Sec. 3.3.1, second equation) and the fully connected
// layers with ReLU and a scalar output (Sec. 3.3.2).
void readout_and_head(int n_cand, const int32_t* node_off, const float* h, int H, int bf16, const float* head,
                      float* pred, float* readout) {
  const size_t HH = static_cast<size_t>(H) * H;
  std::vector<float> hd(head, head + 2 * HH + 3 * H + 1);
  if (bf16) {
    for (size_t i = 0; i < HH; ++i) hd[i] = round_bf16(hd[i]);                     // W1
    for (size_t i = 0; i < HH; ++i) hd[HH + H + i] = round_bf16(hd[HH + H + i]);   // W2
    for (int i = 0; i < H; ++i) hd[2 * HH + 2 * H + i] = round_bf16(hd[2 * HH + 2 * H + i]);  // w3
  }
  const float* W1 = hd.data();
  const float* b1 = W1 + HH;
  const float* W2 = b1 + H;
  const float* b2 = W2 + HH;
  const float* w3 = b2 + H;
  const float* b3 = w3 + H;
  std::vector<double> r(H), z1(H), z2(H);
  std::vector<float> rf(H), z1f(H), z2f(H);
  for (int c = 0; c < n_cand; ++c) {
    for (int j = 0; j < H; ++j) r[j] = 0.0;
    for (int64_t v = node_off[c]; v < node_off[c + 1]; ++v)
      for (int j = 0; j < H; ++j) r[j] += h[static_cast<size_t>(v) * H + j];
    for (int j = 0; j < H; ++j) rf[j] = static_cast<float>(r[j]);
    if (readout) std::memcpy(readout + static_cast<size_t>(c) * H, rf.data(), H * sizeof(float));
    for (int j = 0; j < H; ++j) z1[j] = b1[j];
    for (int k = 0; k < H; ++k)
      for (int j = 0; j < H; ++j) z1[j] += static_cast<double>(rf[k]) * W1[static_cast<size_t>(k) * H + j];
    for (int j = 0; j < H; ++j) z1f[j] = static_cast<float>(z1[j] > 0.0 ? z1[j] : 0.0);
    for (int j = 0; j < H; ++j) z2[j] = b2[j];
    for (int k = 0; k < H; ++k)
      for (int j = 0; j < H; ++j) z2[j] += static_cast<double>(z1f[k]) * W2[static_cast<size_t>(k) * H + j];
    for (int j = 0; j < H; ++j) z2f[j] = static_cast<float>(z2[j] > 0.0 ? z2[j] : 0.0);
    double t = b3[0];
    for (int j = 0; j < H; ++j) t += static_cast<double>(z2f[j]) * w3[j];
    pred[c] = static_cast<float>(t);
  }
}

}  // namespace

extern "C" {

// Rounds x[0..n) to bfloat16 values in place (still stored as fp32).
void orc_round_bf16(float* x, int64_t n) {
  for (int64_t i = 0; i < n; ++i) x[i] = round_bf16(x[i]);
}

// Contracts every candidate and lays the results out block-diagonally:
// candidate c owns nodes [node_off[c], node_off[c+1]) and edges
// [edge_off[c], edge_off[c+1]); rowptr entries are global edge positions and
// col entries are global node numbers.  Base graph b occupies rows
// [g_node_off[b], g_node_off[b+1]) of X, its rowptr (n_b+1 entries starting
// at 0) starts at g_node_off[b] + b and its col at g_edge_off[b].
// cnt (optional) receives the member count per contracted node.
// Capacities: new_id has cand_off[C] entries; node arrays cap_nodes (+1 for
// rowptr), edge arrays cap_edges.  Returns 0, 3 (bad label), 4 (capacity).
int orc_contract_batch(int n_graphs, const int32_t* g_node_off, const int32_t* g_edge_off,
                       const int32_t* rowptr, const int32_t* col, const float* X, int F,
                       int n_cand, const int32_t* cand_graph, const int64_t* cand_off,
                       const int32_t* label, int bf16,
                       int64_t cap_nodes, int64_t cap_edges,
                       int32_t* node_off, int32_t* edge_off, int32_t* new_id,
                       int32_t* out_rowptr, int32_t* out_col, int32_t* in_rowptr, int32_t* in_col,
                       float* Xc, int32_t* cnt) {
  (void)n_graphs;
  int64_t nt = 0, et = 0;
  node_off[0] = 0;
  edge_off[0] = 0;
  std::vector<int32_t> nid, orp, oc, irp, ic, ct;
  std::vector<float> xc;
  for (int c = 0; c < n_cand; ++c) {
    int b = cand_graph[c];
    int n = g_node_off[b + 1] - g_node_off[b];
    int G = 0;
    int rc = contract_one(n, rowptr + g_node_off[b] + b, col + g_edge_off[b],
                          X + static_cast<size_t>(g_node_off[b]) * F, F, label + cand_off[c], bf16,
                          nid, G, orp, oc, irp, ic, xc, ct);
    if (rc) return rc;
    int64_t E = static_cast<int64_t>(oc.size());
    if (nt + G > cap_nodes || et + E > cap_edges) return 4;
    for (int v = 0; v < n; ++v) new_id[cand_off[c] + v] = nid[v];
    for (int g = 0; g < G; ++g) {
      out_rowptr[nt + g] = static_cast<int32_t>(et + orp[g]);
      in_rowptr[nt + g] = static_cast<int32_t>(et + irp[g]);
      if (cnt) cnt[nt + g] = ct[g];
    }
    for (int64_t e = 0; e < E; ++e) {
      out_col[et + e] = static_cast<int32_t>(nt + oc[e]);
      in_col[et + e] = static_cast<int32_t>(nt + ic[e]);
    }
    std::memcpy(Xc + static_cast<size_t>(nt) * F, xc.data(), xc.size() * sizeof(float));
    nt += G;
    et += E;
    node_off[c + 1] = static_cast<int32_t>(nt);
    edge_off[c + 1] = static_cast<int32_t>(et);
  }
  out_rowptr[nt] = static_cast<int32_t>(et);
  in_rowptr[nt] = static_cast<int32_t>(et);
  return 0;
}

// Forward pass over a block-diagonal batch (layout as produced above).
//   W_layers: concat over l of W^l, row-major [3d, H], d = F for l = 0 else H;
//             rows [0,d) multiply the node's own vector, [d,2d) the mean over
//             predecessors, [2d,3d) the mean over successors.
//   b_layers: concat of b^l [H].
//   head:     W1[H,H] | b1[H] | W2[H,H] | b2[H] | w3[H] | b3[1]; W row-major [in,out].
//   pred[c]:  predicted time of candidate c.
//   h_last (optional, [Ntot,H]) and readout (optional, [C,H]) receive the last
//   layer's activations and the per-graph sums.
void orc_gnn_forward(int n_cand, const int32_t* node_off,
                     const int32_t* out_rowptr, const int32_t* out_col,
                     const int32_t* in_rowptr, const int32_t* in_col,
                     const float* Xc, int F, int H, int L, int bf16,
                     const float* W_layers, const float* b_layers, const float* head,
                     float* pred, float* h_last, float* readout) {
  const int64_t Ntot = node_off[n_cand];
  // weights as the device path stores them
  size_t wlen = 0;
  for (int l = 0; l < L; ++l) wlen += static_cast<size_t>(3) * (l == 0 ? F : H) * H;
  std::vector<float> W(W_layers, W_layers + wlen);
  if (bf16)
    for (auto& w : W) w = round_bf16(w);

  int dmax = F > H ? F : H;
  std::vector<float> h(static_cast<size_t>(Ntot) * dmax), hn(static_cast<size_t>(Ntot) * dmax);
  std::vector<float> hin(static_cast<size_t>(Ntot) * dmax), hout(static_cast<size_t>(Ntot) * dmax);
  for (int64_t v = 0; v < Ntot; ++v)
    for (int k = 0; k < F; ++k) h[v * F + k] = bf16 ? round_bf16(Xc[v * F + k]) : Xc[v * F + k];

  std::vector<double> acc(dmax > H ? dmax : H);
  const float* Wl = W.data();
  const float* bl = b_layers;
  int d = F;
  for (int l = 0; l < L; ++l) {
    // mean over predecessors / successors; an empty neighbourhood gives 0
    for (int64_t v = 0; v < Ntot; ++v) {
      for (int dir = 0; dir < 2; ++dir) {
        const int32_t* rp = dir == 0 ? in_rowptr : out_rowptr;
        const int32_t* ci = dir == 0 ? in_col : out_col;
        float* dst = (dir == 0 ? hin.data() : hout.data()) + v * d;
        int deg = rp[v + 1] - rp[v];
        for (int k = 0; k < d; ++k) acc[k] = 0.0;
        for (int e = rp[v]; e < rp[v + 1]; ++e)
          for (int k = 0; k < d; ++k) acc[k] += h[static_cast<int64_t>(ci[e]) * d + k];
        for (int k = 0; k < d; ++k) dst[k] = deg ? store(acc[k] / deg, bf16) : 0.0f;
      }
    }
    // h' = ReLU([h | h_in | h_out] W + b)
    for (int64_t v = 0; v < Ntot; ++v) {
      for (int j = 0; j < H; ++j) acc[j] = bl[j];
      const float* parts[3] = {h.data() + v * d, hin.data() + v * d, hout.data() + v * d};
      for (int p = 0; p < 3; ++p)
        for (int k = 0; k < d; ++k) {
          double a = parts[p][k];
          const float* wrow = Wl + (static_cast<size_t>(p) * d + k) * H;
          for (int j = 0; j < H; ++j) acc[j] += a * wrow[j];
        }
      for (int j = 0; j < H; ++j) hn[v * H + j] = store(acc[j] > 0.0 ? acc[j] : 0.0, bf16);
    }
    h.swap(hn);
    Wl += static_cast<size_t>(3) * d * H;
    bl += H;
    d = H;
  }
  if (h_last) std::memcpy(h_last, h.data(), static_cast<size_t>(Ntot) * H * sizeof(float));
  readout_and_head(n_cand, node_off, h.data(), H, bf16, head, pred, readout);
}

// Forward pass with attention coefficients (see the header of this file).
//   W_layers: concat over l of W^l, row-major [d_l, H] (d_0 = F, else H).
//   att:      concat over l of a_src^l [H] | a_dst^l [H] (head k owns columns k*H/K ..).
//   b_layers: concat of b^l [H].
void orc_gnn_forward_attn(int n_cand, const int32_t* node_off,
                          const int32_t* out_rowptr, const int32_t* out_col,
                          const int32_t* in_rowptr, const int32_t* in_col,
                          const float* Xc, int F, int H, int L, int K, int bf16,
                          const float* W_layers, const float* att, const float* b_layers, const float* head,
                          float* pred, float* h_last, float* readout) {
  const int64_t Ntot = node_off[n_cand];
  const int Dh = H / K;
  size_t wlen = 0;
  for (int l = 0; l < L; ++l) wlen += static_cast<size_t>(l == 0 ? F : H) * H;
  std::vector<float> W(W_layers, W_layers + wlen);
  if (bf16)
    for (auto& w : W) w = round_bf16(w);
  const int dmax = F > H ? F : H;
  std::vector<float> h(static_cast<size_t>(Ntot) * dmax), hn(static_cast<size_t>(Ntot) * H);
  std::vector<float> z(static_cast<size_t>(Ntot) * H), sc_src(static_cast<size_t>(Ntot) * K),
      sc_dst(static_cast<size_t>(Ntot) * K);
  for (int64_t v = 0; v < Ntot; ++v)
    for (int k = 0; k < F; ++k) h[v * F + k] = bf16 ? round_bf16(Xc[v * F + k]) : Xc[v * F + k];
  std::vector<double> acc(H), u, wgt;
  std::vector<int64_t> nb;
  const float* Wl = W.data();
  const float* al = att;
  const float* bl = b_layers;
  int d = F;
  for (int l = 0; l < L; ++l) {
    // z = W e' per node, then the two score terms per node and head
    for (int64_t v = 0; v < Ntot; ++v) {
      for (int j = 0; j < H; ++j) acc[j] = 0.0;
      for (int k = 0; k < d; ++k) {
        const double a = h[v * d + k];
        const float* wrow = Wl + static_cast<size_t>(k) * H;
        for (int j = 0; j < H; ++j) acc[j] += a * wrow[j];
      }
      for (int j = 0; j < H; ++j) z[v * H + j] = store(acc[j], bf16);
      for (int k = 0; k < K; ++k) {
        double ss = 0.0, tt = 0.0;
        for (int c = k * Dh; c < (k + 1) * Dh; ++c) {
          ss += static_cast<double>(al[c]) * z[v * H + c];
          tt += static_cast<double>(al[H + c]) * z[v * H + c];
        }
        sc_src[v * K + k] = static_cast<float>(ss);
        sc_dst[v * K + k] = static_cast<float>(tt);
      }
    }
    for (int64_t v = 0; v < Ntot; ++v) {
      nb.clear();
      nb.push_back(v);
      for (int e = in_rowptr[v]; e < in_rowptr[v + 1]; ++e) nb.push_back(in_col[e]);
      for (int e = out_rowptr[v]; e < out_rowptr[v + 1]; ++e) nb.push_back(out_col[e]);
      u.resize(nb.size());
      wgt.resize(nb.size());
      for (int k = 0; k < K; ++k) {
        double m = -INFINITY;
        for (size_t i = 0; i < nb.size(); ++i) {
          double x = static_cast<double>(sc_src[v * K + k]) + static_cast<double>(sc_dst[nb[i] * K + k]);
          x = x > 0.0 ? x : 0.2 * x;
          u[i] = x;
          if (x > m) m = x;
        }
        double den = 0.0;
        for (size_t i = 0; i < nb.size(); ++i) {
          wgt[i] = std::exp(u[i] - m);
          den += wgt[i];
        }
        for (int c = k * Dh; c < (k + 1) * Dh; ++c) {
          double o = 0.0;
          for (size_t i = 0; i < nb.size(); ++i) o += wgt[i] / den * z[nb[i] * H + c];
          o += bl[c];
          hn[v * H + c] = store(o > 0.0 ? o : 0.0, bf16);
        }
      }
    }
    h.assign(hn.begin(), hn.end());
    Wl += static_cast<size_t>(d) * H;
    al += 2 * H;
    bl += H;
    d = H;
  }
  if (h_last) std::memcpy(h_last, h.data(), static_cast<size_t>(Ntot) * H * sizeof(float));
  readout_and_head(n_cand, node_off, h.data(), H, bf16, head, pred, readout);
}

// List-scheduling estimate of the per-iteration time of each candidate module (see the
// header).  op_time[v]: execution time of computation node v; ar_size[v]: tensor size of
// all-reduce node v, negative for computation nodes.  cost[c] = +inf if graph c has a cycle.
void orc_simulate(int n_cand, const int32_t* node_off,
                  const int32_t* out_rowptr, const int32_t* out_col,
                  const int32_t* in_rowptr, const int32_t* /*in_col*/,
                  const float* op_time, const float* ar_size, float ar_c, float ar_d, float* cost) {
  std::vector<int> indeg;
  std::vector<double> ready;
  std::vector<int64_t> q, aq;
  for (int c = 0; c < n_cand; ++c) {
    const int64_t n0 = node_off[c], n1 = node_off[c + 1], G = n1 - n0;
    indeg.assign(G, 0);
    ready.assign(G, 0.0);
    q.clear();
    aq.clear();
    for (int64_t v = 0; v < G; ++v) {
      indeg[v] = in_rowptr[n0 + v + 1] - in_rowptr[n0 + v];
      if (indeg[v] == 0) (ar_size[n0 + v] >= 0.0f ? aq : q).push_back(v);
    }
    size_t qh = 0, ah = 0;
    int64_t processed = 0;
    double dev = 0.0, chan = 0.0;
    while (ah < aq.size() || qh < q.size()) {
      int64_t u;
      double done;
      if (ah < aq.size()) {               // tensors already produced go on the channel first
        u = aq[ah++];
        const double start = ready[u] > chan ? ready[u] : chan;
        done = start + (static_cast<double>(ar_c) * static_cast<double>(ar_size[n0 + u]) + static_cast<double>(ar_d));
        chan = done;
      } else {
        u = q[qh++];
        const double start = ready[u] > dev ? ready[u] : dev;
        done = start + static_cast<double>(op_time[n0 + u]);
        dev = done;
      }
      ++processed;
      for (int e = out_rowptr[n0 + u]; e < out_rowptr[n0 + u + 1]; ++e) {
        const int64_t w = out_col[e] - n0;
        if (done > ready[w]) ready[w] = done;
        if (--indeg[w] == 0) (ar_size[n0 + w] >= 0.0f ? aq : q).push_back(w);
      }
    }
    cost[c] = processed == G ? static_cast<float>(dev > chan ? dev : chan) : INFINITY;
  }
}

// The fused ops of every candidate as a batch of small graphs (Sec. 3.3: a fused op is the
// subgraph of the model graph whose nodes are its original ops and whose edges are the
// dependencies among them; the estimator predicts its execution time from that subgraph).
// A contracted node is a fused op when it has at least two members and all of them are
// computation ops (ar_size_base < 0).  Order: candidates ascending, within a candidate
// contracted nodes ascending; the rows of a fused op are its members in ascending base
// index with their own feature rows (rounded like every stored feature); its edges are the
// base edges with both ends in the group, 0/1 adjacency, lists ascending.  Layout as for
// orc_contract_batch with one graph per fused op.  fo_cnode[k] is the contracted node
// (global number) of fused op k, fo_member[r] the base node (local number) of row r.
// new_id / c_node_off are the outputs of orc_contract_batch for the same candidates.
// Returns the number of fused ops, or -4 when a capacity is exceeded.
int64_t orc_fused_op_batch(const int32_t* g_node_off, const int32_t* g_edge_off, const int32_t* rowptr,
                           const int32_t* col, const float* X, int F, const float* ar_size_base, int n_cand,
                           const int32_t* cand_graph, const int64_t* cand_off, const int32_t* new_id,
                           const int32_t* c_node_off, int bf16, int64_t cap_graphs, int64_t cap_nodes,
                           int64_t cap_edges, int32_t* fo_node_off, int32_t* fo_edge_off, int32_t* fo_cnode,
                           int32_t* fo_member, int32_t* out_rowptr, int32_t* out_col, int32_t* in_rowptr,
                           int32_t* in_col, float* Xf) {
  int64_t K = 0, nt = 0, et = 0;
  fo_node_off[0] = 0;
  fo_edge_off[0] = 0;
  for (int c = 0; c < n_cand; ++c) {
    const int b = cand_graph[c];
    const int n = g_node_off[b + 1] - g_node_off[b];
    const int32_t* rp = rowptr + g_node_off[b] + b;
    const int32_t* ci = col + g_edge_off[b];
    const int32_t* nid = new_id + cand_off[c];
    const int G = c_node_off[c + 1] - c_node_off[c];
    std::vector<std::vector<int32_t>> members(G);
    for (int v = 0; v < n; ++v) members[nid[v]].push_back(v);      // ascending by construction
    for (int g = 0; g < G; ++g) {
      const std::vector<int32_t>& m = members[g];
      bool ops_only = true;
      for (int32_t v : m) ops_only = ops_only && ar_size_base[g_node_off[b] + v] < 0.0f;
      if (m.size() < 2 || !ops_only) continue;
      std::set<std::pair<int32_t, int32_t>> fwd, bwd;             // (row, neighbour) in member positions
      for (size_t i = 0; i < m.size(); ++i)
        for (int e = rp[m[i]]; e < rp[m[i] + 1]; ++e) {
          const int32_t w = ci[e];
          if (nid[w] != g || w == m[i]) continue;
          size_t j = 0;
          while (m[j] != w) ++j;
          fwd.insert({static_cast<int32_t>(i), static_cast<int32_t>(j)});
          bwd.insert({static_cast<int32_t>(j), static_cast<int32_t>(i)});
        }
      const int64_t sz = static_cast<int64_t>(m.size()), E = static_cast<int64_t>(fwd.size());
      if (K + 1 > cap_graphs || nt + sz > cap_nodes || et + E > cap_edges) return -4;
      std::vector<int32_t> orp(sz + 1, 0), irp(sz + 1, 0);
      int64_t k = 0;
      for (const auto& p : fwd) {
        orp[p.first + 1] += 1;
        out_col[et + k++] = static_cast<int32_t>(nt + p.second);
      }
      k = 0;
      for (const auto& p : bwd) {
        irp[p.first + 1] += 1;
        in_col[et + k++] = static_cast<int32_t>(nt + p.second);
      }
      for (int64_t i = 0; i < sz; ++i) {
        orp[i + 1] += orp[i];
        irp[i + 1] += irp[i];
        out_rowptr[nt + i] = static_cast<int32_t>(et + orp[i]);
        in_rowptr[nt + i] = static_cast<int32_t>(et + irp[i]);
        fo_member[nt + i] = m[i];
        for (int f = 0; f < F; ++f)
          Xf[static_cast<size_t>(nt + i) * F + f] =
              store(static_cast<double>(X[static_cast<size_t>(g_node_off[b] + m[i]) * F + f]), bf16);
      }
      fo_cnode[K] = c_node_off[c] + g;
      nt += sz;
      et += E;
      ++K;
      fo_node_off[K] = static_cast<int32_t>(nt);
      fo_edge_off[K] = static_cast<int32_t>(et);
    }
  }
  out_rowptr[nt] = static_cast<int32_t>(et);
  in_rowptr[nt] = static_cast<int32_t>(et);
  return K;
}

// What the simulator is given for every node of the candidate modules (Sec. 3.1, Simulator:
// profiled data for individual ops, the estimator for fused ops, the linear model for
// all-reduce instructions on the size of the - possibly fused - tensor; Sec. 2.3: the size of
// a fused tensor is the sum of its members' sizes).  Per contracted node:
//   all members all-reduce tensors: ar_size = sum of their sizes (fp64, ascending member
//                                   index, rounded once), op_time = 0 (unused)
//   one op:                         op_time = its profiled time, ar_size = -1
//   two or more ops:                op_time = max(0, estimator output) (the regression network
//                                   ends in a ReLU, Sec. 3.3.2: a time is never negative),
//                                   taken from fo_pred through fo_cnode; ar_size = -1
//   ops and tensors mixed:          not a fusion the strategies produce (Sec. 3.2): op_time =
//                                   +infinity, which makes the module cost +infinity
void orc_module_times(const int32_t* g_node_off, const float* op_time_base, const float* ar_size_base, int n_cand,
                      const int32_t* cand_graph, const int64_t* cand_off, const int32_t* new_id,
                      const int32_t* c_node_off, int64_t K, const int32_t* fo_cnode, const float* fo_pred,
                      float* op_time, float* ar_size) {
  for (int c = 0; c < n_cand; ++c) {
    const int b = cand_graph[c];
    const int n = g_node_off[b + 1] - g_node_off[b];
    const int32_t* nid = new_id + cand_off[c];
    const int G = c_node_off[c + 1] - c_node_off[c];
    std::vector<int> n_op(G, 0), n_ar(G, 0);
    std::vector<double> size_sum(G, 0.0);
    std::vector<float> single(G, 0.0f);
    for (int v = 0; v < n; ++v) {
      const float x = ar_size_base[g_node_off[b] + v];
      if (x >= 0.0f) {
        n_ar[nid[v]] += 1;
        size_sum[nid[v]] += static_cast<double>(x);
      } else {
        n_op[nid[v]] += 1;
        single[nid[v]] = op_time_base[g_node_off[b] + v];
      }
    }
    for (int g = 0; g < G; ++g) {
      const int64_t o = c_node_off[c] + g;
      if (n_op[g] == 0) {
        op_time[o] = 0.0f;
        ar_size[o] = static_cast<float>(size_sum[g]);
      } else if (n_ar[g] == 0) {
        op_time[o] = n_op[g] == 1 ? single[g] : 0.0f;      // fused ops are filled in below
        ar_size[o] = -1.0f;
      } else {
        op_time[o] = INFINITY;
        ar_size[o] = -1.0f;
      }
    }
  }
  for (int64_t k = 0; k < K; ++k) op_time[fo_cnode[k]] = fo_pred[k] > 0.0f ? fo_pred[k] : 0.0f;
}

}  // extern "C"

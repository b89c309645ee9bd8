// C2T tree-construction ORACLE — test infrastructure, not product code.
//
// A plain, slow, single-threaded CPU statement of what one draft phase of C2T
// computes (arXiv 2502.13652): Algorithm 1 with Eq. 1 (joint probability),
// Eq. 2 (entropy; first line = full vocabulary, second line = top-M variant),
// Eq. 3 (classifier confidence), the two prunings of Sec. 4.2 and the emission
// of the verification inputs (tree mask, position ids, parent links) that tree
// attention (Sec. 2.2) consumes.  All real arithmetic is fp64 unless a comment
// says otherwise; nothing is blocked, fused or reordered.  Only tests, the
// smoke check and the benchmark's cpu_baseline leg may call this file; the HIP
// library shares no code with it.
//
// Readings taken where the paper is silent (each is listed in the design notes):
//  * H_i is the entropy of the distribution node i was drawn from (Sec. 4.1:
//    "the distribution in which each node resides"), natural logarithm, 0 log 0 = 0.
//  * C = sigmoid(z); "keep iff C > beta" (Alg. 1 loop guard, strict) is decided
//    as z > logit(beta) with logit(beta) rounded once to fp32.
//  * The classifier is evaluated in fp32 with a fixed fused-multiply-add order
//    (the precision the decisions are taken in); features are the fp64 results
//    rounded once to fp32; P_child = P_parent * p is one fp32 multiply (Eq. 1 as
//    a running product).
//  * depth feature d = layer index (0 for the root's children), position id = d+1.
//  * Second pruning keeps the `max_frontier` best survivors ranked by
//    (z desc, token id asc, parent slot asc); the node budget (EAGLE-2's N,
//    Sec. 2.2, root excluded) admits min(max_frontier, budget - |T|) per layer.
//  * NaN, +inf or an all -inf row yields no candidates and sets status bit 0.
//
// parity pins: tests/test_oracle_*.py (closed forms, invariants, library
// routines, brute force, the paper's tree-size and overhead arithmetic).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

enum { DT_F32 = 0, DT_BF16 = 1 };

inline double load_logit(const void* row, int dtype, int64_t j) {
  if (dtype == DT_F32) return (double)((const float*)row)[j];
  uint32_t bits = (uint32_t)((const uint16_t*)row)[j] << 16;  // bf16 -> fp32 is exact widening
  float f;
  std::memcpy(&f, &bits, 4);
  return (double)f;
}

struct RowResult {
  bool bad = false;       // NaN / +inf present, or no finite element
  double m = 0, Z = 0, S = 0, H = 0;
  std::vector<int32_t> top_id;   // K ids, (logit desc, id asc)
  std::vector<double> top_x;     // their logits
  std::vector<double> top_p;     // e^{x-m}/Z
};

// Softmax normaliser, entropy (Eq. 2, first line) and the K most probable
// tokens of one logits row (Sec. 4.2.2, purpose 1 of TopK).
RowResult row_definition(const void* row, int dtype, int V, int K) {
  RowResult r;
  std::vector<double> x((size_t)V);
  double m = -std::numeric_limits<double>::infinity();
  for (int j = 0; j < V; ++j) {
    x[j] = load_logit(row, dtype, j);
    if (std::isnan(x[j]) || x[j] == std::numeric_limits<double>::infinity()) r.bad = true;
    if (x[j] > m) m = x[j];
  }
  if (V <= 0 || m == -std::numeric_limits<double>::infinity()) r.bad = true;
  if (r.bad) return r;
  double Z = 0.0, S = 0.0;
  for (int j = 0; j < V; ++j) {
    double e = std::exp(x[j] - m);
    Z += e;
    if (e > 0.0) S += (x[j] - m) * e;       // 0 * log 0 := 0
  }
  r.m = m; r.Z = Z; r.S = S;
  r.H = std::log(Z) - S / Z;                // = -sum p ln p with p = e^{x-m}/Z
  std::vector<int32_t> idx((size_t)V);
  for (int j = 0; j < V; ++j) idx[j] = j;
  int k = std::min(K, V);
  std::partial_sort(idx.begin(), idx.begin() + k, idx.end(), [&](int32_t a, int32_t b) {
    if (x[a] != x[b]) return x[a] > x[b];
    return a < b;
  });
  for (int c = 0; c < k; ++c) {
    r.top_id.push_back(idx[c]);
    r.top_x.push_back(x[idx[c]]);
    r.top_p.push_back(std::exp(x[idx[c]] - m) / Z);
  }
  return r;
}

// Eq. 2, second line: entropy over the M most probable tokens only, using the
// probabilities of the full softmax (not renormalised), as the equation writes it.
double entropy_top_m(const void* row, int dtype, int V, int M) {
  RowResult full = row_definition(row, dtype, V, std::min(M, V));
  if (full.bad) return std::numeric_limits<double>::quiet_NaN();
  double H = 0.0;
  for (double p : full.top_p)
    if (p > 0.0) H -= p * std::log(p);
  return H;
}

// Eq. 3: two-layer FFN on (P, H, d), ReLU hidden layer; returns the pre-sigmoid
// logit z.  fp32, one fixed order of fused multiply-adds.
float mlp_logit(int h, const float* W1, const float* b1, const float* w2, float b2,
                float P, float H, float d) {
  float z = b2;
  for (int j = 0; j < h; ++j) {
    float a = std::fmaf(W1[3 * j + 0], P, b1[j]);
    a = std::fmaf(W1[3 * j + 1], H, a);
    a = std::fmaf(W1[3 * j + 2], d, a);
    a = a > 0.0f ? a : 0.0f;
    z = std::fmaf(w2[j], a, z);
  }
  return z;
}

struct Node {
  int32_t token, parent, depth;   // parent = node index, -1 for a child of the root
  float P, H, z, p;
};

struct Cand {
  int32_t token, slot;
  float p, P, H, z;
  int32_t kept;      // 0 dropped, 1 kept
};

// Every candidate that was given a confidence, in the order it was scored (layer by layer, within a
// layer by frontier slot, then by rank in the row); s = smallest classifier logit on the path from
// the root's child down to the candidate (itself included).
struct HistCand {
  int32_t token, parent, depth;   // parent = index into the history, -1 for a child of the root
  float P, H, z, s;
};

struct Seq {
  std::vector<HistCand> hist;
  std::vector<int32_t> node_hist;       // history index of each tree node
  std::vector<Node> nodes;
  std::vector<int32_t> frontier;        // node indices; -1 = root
  std::vector<int32_t> frontier_slot;   // slot of each frontier node's parent in the previous frontier
  std::vector<Cand> last_cands;
  uint32_t status = 0;
  int64_t scored = 0;
  double min_thr_margin = std::numeric_limits<double>::infinity();
  double min_rank_gap = std::numeric_limits<double>::infinity();
};

struct Tree {
  int B, V, F, K, D, N, h, dtype;
  float beta, z_beta;
  int entropy_top_m = 0;     // 0 = full-vocabulary entropy
  std::vector<float> W1, b1, w2;
  float b2 = 0;
  bool have_cls = false;
  int layer = 0;
  std::vector<Seq> seq;
};

void reset_seq(Seq& s) {
  s.hist.clear();
  s.node_hist.clear();
  s.nodes.clear();
  s.frontier.assign(1, -1);
  s.frontier_slot.assign(1, 0);
  s.last_cands.clear();
  s.status = 0;
  s.scored = 0;
  s.min_thr_margin = std::numeric_limits<double>::infinity();
  s.min_rank_gap = std::numeric_limits<double>::infinity();
}

// One iteration of the while-loop of Algorithm 1 for one sequence.
void expand_seq(Tree& t, Seq& s, const char* logits_seq, int64_t row_stride_elems) {
  const int esz = t.dtype == DT_F32 ? 4 : 2;
  std::vector<Cand> cand;
  const int nf = (int)s.frontier.size();
  for (int f = 0; f < nf; ++f) {
    const void* row = logits_seq + (int64_t)f * row_stride_elems * esz;
    RowResult r = row_definition(row, t.dtype, t.V, t.K);
    if (r.bad) { s.status |= 1u; continue; }
    double Hd = r.H;
    if (t.entropy_top_m > 0) Hd = entropy_top_m(row, t.dtype, t.V, t.entropy_top_m);
    const float H32 = (float)Hd;
    const int32_t parent = s.frontier[f];
    const float Pparent = parent < 0 ? 1.0f : s.nodes[parent].P;
    for (size_t c = 0; c < r.top_id.size(); ++c) {
      Cand q;
      q.token = r.top_id[c];
      q.slot = f;
      q.p = (float)r.top_p[c];
      q.P = Pparent * q.p;                       // Eq. 1, running product in fp32
      q.H = H32;
      q.z = mlp_logit(t.h, t.W1.data(), t.b1.data(), t.w2.data(), t.b2, q.P, q.H, (float)t.layer);
      q.kept = 0;
      cand.push_back(q);
    }
  }
  s.scored += (int64_t)cand.size();
  const int32_t hist_base = (int32_t)s.hist.size();
  for (const Cand& q : cand) {
    HistCand hc;
    const int32_t parent_node = s.frontier[q.slot];
    hc.token = q.token; hc.depth = t.layer; hc.P = q.P; hc.H = q.H; hc.z = q.z;
    hc.parent = parent_node < 0 ? -1 : s.node_hist[parent_node];
    hc.s = hc.parent < 0 ? q.z : std::min(s.hist[hc.parent].s, q.z);
    s.hist.push_back(hc);
  }
  // first pruning: keep iff C > beta  <=>  z > logit(beta)
  std::vector<int> surv;
  for (int i = 0; i < (int)cand.size(); ++i) {
    if (cand[i].z > t.z_beta) surv.push_back(i);
    if (std::isfinite(t.z_beta)) {
      double mg = std::fabs((double)cand[i].z - (double)t.z_beta);
      if (mg < s.min_thr_margin) s.min_thr_margin = mg;
    }
  }
  // second pruning + budget: rank, keep the first min(F, N - |T|)
  std::stable_sort(surv.begin(), surv.end(), [&](int a, int b) {
    if (cand[a].z != cand[b].z) return cand[a].z > cand[b].z;
    if (cand[a].token != cand[b].token) return cand[a].token < cand[b].token;
    return cand[a].slot < cand[b].slot;
  });
  int room = t.N - (int)s.nodes.size();
  int n_keep = std::min(std::min(t.F, room), (int)surv.size());
  if (n_keep < 0) n_keep = 0;
  // audit: smallest gap between neighbours in the ranking that a decision or the
  // output order depends on (positions 0..n_keep), exact ties excluded
  for (int i = 0; i + 1 < (int)surv.size() && i < n_keep; ++i) {
    double g = (double)cand[surv[i]].z - (double)cand[surv[i + 1]].z;
    if (g > 0 && g < s.min_rank_gap) s.min_rank_gap = g;
  }
  std::vector<int32_t> new_frontier, new_slot;
  for (int i = 0; i < n_keep; ++i) {
    Cand& q = cand[surv[i]];
    q.kept = 1;
    Node n;
    n.token = q.token;
    n.parent = s.frontier[q.slot];
    n.depth = t.layer;
    n.P = q.P; n.H = q.H; n.z = q.z; n.p = q.p;
    new_frontier.push_back((int32_t)s.nodes.size());
    new_slot.push_back(q.slot);
    s.nodes.push_back(n);
    s.node_hist.push_back(hist_base + surv[i]);
  }
  s.frontier.swap(new_frontier);
  s.frontier_slot.swap(new_slot);
  s.last_cands.swap(cand);
}

}  // namespace

extern "C" {

// ---- single-row entry points (used by pins and by row-level parity) ----
int c2t_ref_row(const void* row, int dtype, int vocab, int top_k, double* m, double* Z, double* S,
                double* H, int32_t* top_ids, double* top_logits, double* top_p) {
  RowResult r = row_definition(row, dtype, vocab, top_k);
  if (r.bad) return 1;
  *m = r.m; *Z = r.Z; *S = r.S; *H = r.H;
  for (size_t c = 0; c < r.top_id.size(); ++c) {
    top_ids[c] = r.top_id[c];
    if (top_logits) top_logits[c] = r.top_x[c];
    if (top_p) top_p[c] = r.top_p[c];
  }
  return 0;
}

double c2t_ref_entropy_top_m(const void* row, int dtype, int vocab, int M) {
  return entropy_top_m(row, dtype, vocab, M);
}

float c2t_ref_mlp_logit(int h, const float* W1, const float* b1, const float* w2, float b2,
                        float P, float H, float d) {
  return mlp_logit(h, W1, b1, w2, b2, P, H, d);
}

float c2t_ref_logit_of_beta(float beta) {
  if (beta <= 0.0f) return -std::numeric_limits<float>::infinity();
  return (float)std::log((double)beta / (1.0 - (double)beta));
}

// ---- tree object: reset -> expand_layer x D -> finalize ----
void* c2t_ref_create(int B, int V, int F, int K, int D, int N, int h, int dtype, float beta) {
  if (B <= 0 || V <= 0 || F <= 0 || K <= 0 || D <= 0 || N <= 0 || h <= 0) return nullptr;
  if (!(beta >= 0.0f && beta < 1.0f)) return nullptr;
  if (dtype != DT_F32 && dtype != DT_BF16) return nullptr;
  Tree* t = new Tree;
  t->B = B; t->V = V; t->F = F; t->K = K; t->D = D; t->N = N; t->h = h; t->dtype = dtype;
  t->beta = beta;
  t->z_beta = c2t_ref_logit_of_beta(beta);
  t->seq.resize((size_t)B);
  for (Seq& s : t->seq) reset_seq(s);
  return t;
}

void c2t_ref_destroy(void* tp) { delete (Tree*)tp; }

void c2t_ref_set_entropy_top_m(void* tp, int M) { ((Tree*)tp)->entropy_top_m = M; }

void c2t_ref_set_classifier(void* tp, const float* W1, const float* b1, const float* w2, float b2) {
  Tree* t = (Tree*)tp;
  t->W1.assign(W1, W1 + 3 * t->h);
  t->b1.assign(b1, b1 + t->h);
  t->w2.assign(w2, w2 + t->h);
  t->b2 = b2;
  t->have_cls = true;
}

void c2t_ref_reset(void* tp) {
  Tree* t = (Tree*)tp;
  t->layer = 0;
  for (Seq& s : t->seq) reset_seq(s);
}

// logits: host memory [B][F][row_stride] of the configured dtype; row f of
// sequence b belongs to frontier slot f; only rows f < n_frontier[b] are read.
// Processes sequences [b0, b1) of the current layer (sequences are independent,
// so a harness may call disjoint ranges from several threads) ...
int c2t_ref_expand_layer_range(void* tp, const void* logits, int64_t row_stride_elems, int b0, int b1) {
  Tree* t = (Tree*)tp;
  if (!t->have_cls || t->layer >= t->D || row_stride_elems < t->V) return -1;
  const int esz = t->dtype == DT_F32 ? 4 : 2;
  for (int b = b0; b < b1; ++b) {
    const char* base = (const char*)logits + (int64_t)b * t->F * row_stride_elems * esz;
    expand_seq(*t, t->seq[b], base, row_stride_elems);
  }
  return 0;
}
// ... and this closes the layer (d <- d + 1 in Algorithm 1).
void c2t_ref_end_layer(void* tp) { ((Tree*)tp)->layer += 1; }

int c2t_ref_expand_layer(void* tp, const void* logits, int64_t row_stride_elems) {
  Tree* t = (Tree*)tp;
  int rc = c2t_ref_expand_layer_range(tp, logits, row_stride_elems, 0, t->B);
  if (rc == 0) c2t_ref_end_layer(tp);
  return rc;
}

int c2t_ref_layer(void* tp) { return ((Tree*)tp)->layer; }

// frontier after the last expand: tokens/parent_slot [B][F] (unused entries -1), n_frontier [B]
void c2t_ref_get_frontier(void* tp, int32_t* tokens, int32_t* parent_slot, int32_t* n_frontier) {
  Tree* t = (Tree*)tp;
  for (int b = 0; b < t->B; ++b) {
    Seq& s = t->seq[b];
    bool root = s.frontier.size() == 1 && s.frontier[0] < 0;
    n_frontier[b] = (int32_t)s.frontier.size();
    for (int f = 0; f < t->F; ++f) {
      bool v = f < (int)s.frontier.size();
      tokens[(int64_t)b * t->F + f] = (v && !root) ? s.nodes[s.frontier[f]].token : -1;
      parent_slot[(int64_t)b * t->F + f] = v ? s.frontier_slot[f] : -1;
    }
  }
}

// candidates scored in the last expanded layer, per sequence, in (slot, rank-in-row) order:
// arrays are [B][F*K]; n_cand [B]
void c2t_ref_get_candidates(void* tp, int32_t* n_cand, int32_t* token, int32_t* slot, float* p,
                            float* P, float* H, float* z, int32_t* kept) {
  Tree* t = (Tree*)tp;
  const int64_t FK = (int64_t)t->F * t->K;
  for (int b = 0; b < t->B; ++b) {
    Seq& s = t->seq[b];
    n_cand[b] = (int32_t)s.last_cands.size();
    for (size_t i = 0; i < s.last_cands.size(); ++i) {
      const Cand& q = s.last_cands[i];
      int64_t o = b * FK + (int64_t)i;
      token[o] = q.token; slot[o] = q.slot; p[o] = q.p; P[o] = q.P; H[o] = q.H; z[o] = q.z;
      kept[o] = q.kept;
    }
  }
}

// conditioning audit: smallest |z - logit(beta)| and smallest positive gap between ranked
// neighbours that the kept set or its order depends on, over all layers so far; plus the
// number of candidates given a confidence.  Arrays [B].
void c2t_ref_get_audit(void* tp, double* min_thr_margin, double* min_rank_gap, int64_t* scored) {
  Tree* t = (Tree*)tp;
  for (int b = 0; b < t->B; ++b) {
    min_thr_margin[b] = t->seq[b].min_thr_margin;
    min_rank_gap[b] = t->seq[b].min_rank_gap;
    scored[b] = t->seq[b].scored;
  }
}

// Verification inputs.  Arrays: tokens/parent/position [B][N] int32 (unused -1/-1/0),
// conf/joint_prob/entropy [B][N] float (unused 0), n_nodes [B], mask [B][N][N] uint8,
// status [B] uint32.  mask[i][j] = 1 iff j == i or j is an ancestor of i; the root is
// not a slot (every candidate attends to it implicitly); position = depth + 1.
void c2t_ref_finalize(void* tp, int32_t* tokens, int32_t* parent, int32_t* position, float* conf,
                      float* joint_prob, float* entropy, int32_t* n_nodes, uint8_t* mask,
                      uint32_t* status) {
  Tree* t = (Tree*)tp;
  const int N = t->N;
  for (int b = 0; b < t->B; ++b) {
    Seq& s = t->seq[b];
    const int n = (int)s.nodes.size();
    n_nodes[b] = n;
    status[b] = s.status;
    uint8_t* mk = mask + (int64_t)b * N * N;
    std::memset(mk, 0, (size_t)N * N);
    for (int i = 0; i < N; ++i) {
      int64_t o = (int64_t)b * N + i;
      if (i < n) {
        const Node& nd = s.nodes[i];
        tokens[o] = nd.token; parent[o] = nd.parent; position[o] = nd.depth + 1;
        conf[o] = (float)(1.0 / (1.0 + std::exp(-(double)nd.z)));
        joint_prob[o] = nd.P; entropy[o] = nd.H;
        for (int j = i; j >= 0; j = s.nodes[j].parent) mk[(int64_t)i * N + j] = 1;
      } else {
        tokens[o] = -1; parent[o] = -1; position[o] = 0;
        conf[o] = 0; joint_prob[o] = 0; entropy[o] = 0;
      }
    }
  }
}

// EAGLE-2-style reranking (Sec. 2.2: "reranks all candidate nodes, selecting the top N"): over every
// candidate scored in any layer, kept by the prunings or not, the n_out best by s, the smallest
// classifier logit on the candidate's path.  s never increases along a path, so with the order
// (s desc, depth asc, scoring order asc) every selected candidate's parent is selected before it:
// the result is a tree for any classifier, and for a classifier that is monotone along paths
// (EAGLE-2's value = joint probability) it is the plain top-n_out by confidence.
// Outputs as c2t_ref_finalize with N replaced by n_out; nodes in selection order.
void c2t_ref_finalize_rerank(void* tp, int n_out, int32_t* tokens, int32_t* parent, int32_t* position, float* conf,
                             float* joint_prob, float* entropy, float* path_min_z, int32_t* n_nodes, uint8_t* mask,
                             uint32_t* status) {
  Tree* t = (Tree*)tp;
  const int N = n_out;
  for (int b = 0; b < t->B; ++b) {
    Seq& s = t->seq[b];
    std::vector<int32_t> order(s.hist.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
      if (s.hist[x].s != s.hist[y].s) return s.hist[x].s > s.hist[y].s;
      if (s.hist[x].depth != s.hist[y].depth) return s.hist[x].depth < s.hist[y].depth;
      return x < y;
    });
    const int n = std::min(N, (int)order.size());
    std::vector<int32_t> out_pos(s.hist.size(), -1);
    for (int i = 0; i < n; ++i) out_pos[order[i]] = i;
    n_nodes[b] = n;
    status[b] = s.status;
    uint8_t* mk = mask + (int64_t)b * N * N;
    std::memset(mk, 0, (size_t)N * N);
    for (int i = 0; i < N; ++i) {
      int64_t o = (int64_t)b * N + i;
      if (i < n) {
        const HistCand& c = s.hist[order[i]];
        tokens[o] = c.token; parent[o] = c.parent < 0 ? -1 : out_pos[c.parent]; position[o] = c.depth + 1;
        conf[o] = (float)(1.0 / (1.0 + std::exp(-(double)c.z)));
        joint_prob[o] = c.P; entropy[o] = c.H; path_min_z[o] = c.s;
        for (int32_t j = order[i]; j >= 0; j = s.hist[j].parent) mk[(int64_t)i * N + out_pos[j]] = 1;
      } else {
        tokens[o] = -1; parent[o] = -1; position[o] = 0;
        conf[o] = 0; joint_prob[o] = 0; entropy[o] = 0; path_min_z[o] = 0;
      }
    }
  }
}

// per-node generation probability p and pre-sigmoid logit z (for invariant tests)
void c2t_ref_get_node_extras(void* tp, float* p, float* z) {
  Tree* t = (Tree*)tp;
  for (int b = 0; b < t->B; ++b)
    for (size_t i = 0; i < t->seq[b].nodes.size(); ++i) {
      p[(int64_t)b * t->N + i] = t->seq[b].nodes[i].p;
      z[(int64_t)b * t->N + i] = t->seq[b].nodes[i].z;
    }
}

}  // extern "C"

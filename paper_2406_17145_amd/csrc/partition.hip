// Pipeline stage partitioner (paper section 5, Alg. 1): series-parallel structure of the operator graph,
// a dynamic programme over it whose value is the smallest number of in-flight samples at the first
// stages of a sub-graph under a bound on every stage's time per sample, and a binary search on that
// bound.  The states carry the schedule configurations of Alg. 1 -- (b, k) of the first stage(s) of a
// sub-graph and (i, b, k) of the stage(s) it feeds -- so that stages may run at different micro-batch sizes
// and kFkB group sizes; gpp_partition is the search with one candidate of each (the default configuration
// of section 6).  Host code; no kernels.  The cost model and the readings of what the paper leaves open
// are stated with gpp_partition and gpp_partition_search in the header.
#include <algorithm>
#include <cstdint>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/gpp.h"

namespace gpp {
gpp_status_t report_error(gpp_status_t st, const std::string &msg);
}
using gpp::report_error;

namespace {

// ---- series-parallel structure (operators are nodes) ---------------------------------------------------
enum Kind : int { LEAF, BLOCK, SERIES, PARALLEL };
struct TNode {
  int kind = LEAF;
  std::vector<int> kids;     // SERIES / PARALLEL: child nodes, in graph order / by smallest operator
  std::vector<int> ops;      // all operators below
  // prefix sums over the children (index c: children [0, c)); for LEAF / BLOCK one entry pair [0, total];
  // pt holds one such row per candidate micro-batch size (the time per sample depends on it)
  std::vector<double> pt, pw, pa;
};

struct Bits {               // set of operators
  std::vector<uint64_t> w;
  explicit Bits(int n = 0) : w((n + 63) / 64, 0) {}
  void set(int i) { w[i >> 6] |= 1ull << (i & 63); }
  bool has(int i) const { return (w[i >> 6] >> (i & 63)) & 1; }
  void or_with(const Bits &o) { for (size_t k = 0; k < w.size(); ++k) w[k] |= o.w[k]; }
  int count_and(const Bits &o) const {
    int c = 0;
    for (size_t k = 0; k < w.size(); ++k) c += __builtin_popcountll(w[k] & o.w[k]);
    return c;
  }
};

struct Builder {
  int n;
  std::vector<std::vector<int>> succ, nbr;
  std::vector<Bits> desc, anc;
  std::vector<TNode> nodes;

  bool closure() {          // descendants by reverse topological order; false on a cycle
    std::vector<int> indeg(n, 0), order;
    for (int u = 0; u < n; ++u) for (int v : succ[u]) ++indeg[v];
    for (int u = 0; u < n; ++u) if (!indeg[u]) order.push_back(u);
    for (size_t q = 0; q < order.size(); ++q)
      for (int v : succ[order[q]]) if (--indeg[v] == 0) order.push_back(v);
    if ((int)order.size() != n) return false;
    desc.assign(n, Bits(n));
    anc.assign(n, Bits(n));
    for (int q = n - 1; q >= 0; --q) {
      const int u = order[q];
      for (int v : succ[u]) {
        desc[u].set(v);
        desc[u].or_with(desc[v]);
      }
    }
    for (int u = 0; u < n; ++u)
      for (int v = 0; v < n; ++v) if (desc[u].has(v)) anc[v].set(u);
    return true;
  }

  int build(std::vector<int> ops) {   // ops sorted ascending
    const int id = (int)nodes.size();
    nodes.emplace_back();
    nodes[id].ops = ops;
    if (ops.size() == 1) return id;
    Bits in(n);
    for (int o : ops) in.set(o);
    // weakly connected parts, each found from its smallest operator
    std::vector<std::vector<int>> parts;
    {
      std::vector<char> seen(n, 0);
      for (int start : ops) {
        if (seen[start]) continue;
        std::vector<int> comp{start}, todo{start};
        seen[start] = 1;
        while (!todo.empty()) {
          const int u = todo.back();
          todo.pop_back();
          for (int v : nbr[u])
            if (in.has(v) && !seen[v]) {
              seen[v] = 1;
              comp.push_back(v);
              todo.push_back(v);
            }
        }
        std::sort(comp.begin(), comp.end());
        parts.push_back(comp);
      }
    }
    if (parts.size() > 1) {
      nodes[id].kind = PARALLEL;
      for (auto &c : parts) {
        const int k = build(c);
        nodes[id].kids.push_back(k);
      }
      return id;
    }
    // operators related to every other operator of the set, in graph order
    std::vector<std::pair<int, int>> cuts;   // (ancestors inside the set, operator)
    for (int v : ops) {
      const int na = anc[v].count_and(in), nd = desc[v].count_and(in);
      if (na + nd + 1 == (int)ops.size()) cuts.push_back({na, v});
    }
    if (cuts.empty()) {
      nodes[id].kind = BLOCK;
      return id;
    }
    std::sort(cuts.begin(), cuts.end());
    std::vector<int> kids;
    Bits before(n);
    for (auto &cv : cuts) {
      const int v = cv.second;
      std::vector<int> seg;
      for (int o : ops) if (anc[v].has(o) && !before.has(o)) seg.push_back(o);
      if (!seg.empty()) kids.push_back(build(seg));
      kids.push_back(build({v}));
      for (int o : seg) before.set(o);
      before.set(v);
    }
    std::vector<int> rest;
    for (int o : ops) if (!before.has(o)) rest.push_back(o);
    if (!rest.empty()) kids.push_back(build(rest));
    nodes[id].kind = SERIES;     // at least two children: a cut operator and something on one side of it
    nodes[id].kids = kids;
    return id;
  }
};

// ---- the dynamic programme ---------------------------------------------------------------------------
// A state is DP(G, c_f, c_b, d) of Alg. 1: G = children [lo, hi) of a tree node; c_f = (b_f, k_f), the
// configuration of the first stage(s) of G; c_b = (i_b, b_b, k_b), the configuration of the stage(s) G feeds
// (none: G ends the graph); d devices.  Its value is the smallest number of in-flight samples at the first
// stage(s) of G such that every stage's time per sample is within the bound and fits its memory.
constexpr int64_t INF = INT64_MAX / 4;
struct Choice {
  int64_t i_f = INF;     // in-flight samples at the first stages of the sub-graph (the DP value)
  int split = 0;         // 0: one stage; else children [lo, split) and [split, hi)
  int d_right = 0;       // devices of the right part
  int bm = 0, km = 0;    // series split: configuration c_m of the first stage(s) of the right part
};
struct Key {
  int32_t node, lo, hi, d, bf, kf, bb, kb;     // bb < 0: no successor
  int64_t ib;
  bool operator==(const Key &o) const {
    return node == o.node && lo == o.lo && hi == o.hi && d == o.d && bf == o.bf && kf == o.kf && bb == o.bb && kb == o.kb && ib == o.ib;
  }
};
struct KeyHash {
  size_t operator()(const Key &k) const {
    uint64_t h = 1469598103934665603ull;
    for (uint64_t v : {(uint64_t)k.node, (uint64_t)k.lo, (uint64_t)k.hi, (uint64_t)k.d, (uint64_t)k.bf, (uint64_t)k.kf,
                       (uint64_t)(k.bb + 1), (uint64_t)k.kb, (uint64_t)k.ib})
      h = (h ^ v) * 1099511628211ull;
    return (size_t)h;
  }
};

struct Search {
  const std::vector<TNode> &T;
  std::vector<int64_t> bs, ks;           // candidate micro-batch sizes and group sizes
  double memory, sync, t_max = 0;
  int64_t mini_batch;
  double link_latency = 0, link_spb = 0;
  // operator edges and their bytes per sample (transfer cost); child index of every operator per node
  const std::vector<std::pair<int, int>> *edges = nullptr;
  const double *x = nullptr;
  std::vector<std::vector<int>> child_of;     // [node][operator] -> child index in that node, -1 outside
  std::unordered_map<Key, Choice, KeyHash> memo;
  std::unordered_map<uint64_t, std::pair<int, double>> cut_memo;
  int64_t states = 0;

  // operator edges with exactly one end in children [lo, hi) of `node`: (count, bytes per sample)
  std::pair<int, double> cut(int node, int lo, int hi) {
    if (!edges || (link_latency == 0 && link_spb == 0)) return {0, 0.0};
    const uint64_t k = ((uint64_t)node << 32) | ((uint64_t)lo << 16) | (uint64_t)hi;
    auto it = cut_memo.find(k);
    if (it != cut_memo.end()) return it->second;
    const std::vector<int> &c = child_of[node];
    int n = 0;
    double by = 0;
    for (size_t e = 0; e < edges->size(); ++e) {
      const int cu = c[(*edges)[e].first], cv = c[(*edges)[e].second];
      const bool in_u = cu >= lo && cu < hi, in_v = cv >= lo && cv < hi;
      if (in_u != in_v) {
        ++n;
        by += x ? x[e] : 0.0;
      }
    }
    return cut_memo.emplace(k, std::make_pair(n, by)).first->second;
  }
  double stage_time(double t, double w, int d, int n_cut, double cut_bytes, int64_t b) const {
    double v = t / d;
    if (d > 1) v += 2.0 * (d - 1) / d * w * sync / (double)mini_batch;
    return v + n_cut * link_latency / (double)b + cut_bytes * link_spb;
  }
  const Choice &solve(int node, int lo, int hi, int bf, int kf, int64_t ib, int bb, int kb, int d) {
    const TNode &N = T[node];
    if (N.kind >= SERIES && hi - lo == 1) {
      const int c = N.kids[lo];
      return solve(c, 0, T[c].kind >= SERIES ? (int)T[c].kids.size() : 1, bf, kf, ib, bb, kb, d);
    }
    const Key k{node, lo, hi, d, bf, kf, bb, kb, ib};
    auto it = memo.find(k);
    if (it != memo.end()) return it->second;
    ++states;
    Choice best;
    const size_t row = (size_t)bf * N.pw.size();      // pt: a row of prefix sums per candidate micro-batch size
    const double t = N.pt[row + hi] - N.pt[row + lo];
    const double w = N.pw[hi] - N.pw[lo], a = N.pa[hi] - N.pa[lo];
    // one stage: its in-flight samples follow from the two configurations (appendix table)
    {
      int64_t i_x = ks[kf] * bs[bf];
      if (bb >= 0) gpp_compute_in_flight(ks[kf], bs[bf], ks[kb], bs[bb], ib, &i_x);
      const std::pair<int, double> c = cut(node, lo, hi);
      if (stage_time(t, w, d, c.first, c.second, bs[bf]) <= t_max && w + (double)i_x / d * a <= memory) best.i_f = i_x;
    }
    if (N.kind >= SERIES && d >= 2) {
      for (int s = lo + 1; s < hi; ++s)
        for (int d2 = 1; d2 < d; ++d2) {
          if (N.kind == SERIES) {
            // the later part first, for every configuration c_m of its first stage(s); what it returns is the
            // successor's in-flight count for the earlier part
            for (int bm = 0; bm < (int)bs.size(); ++bm)
              for (int km = 0; km < (int)ks.size(); ++km) {
                const int64_t mid = solve(node, s, hi, bm, km, ib, bb, kb, d2).i_f;
                if (mid >= INF) continue;
                const int64_t val = solve(node, lo, s, bf, kf, mid, bm, km, d - d2).i_f;
                if (val < best.i_f) {
                  best.i_f = val;
                  best.split = s;
                  best.d_right = d2;
                  best.bm = bm;
                  best.km = km;
                }
              }
          } else {
            // both parts start with c_f and feed c_b; the producer in front has to cover the larger count
            const int64_t l = solve(node, lo, s, bf, kf, ib, bb, kb, d - d2).i_f;
            if (l >= INF) continue;
            const int64_t r = solve(node, s, hi, bf, kf, ib, bb, kb, d2).i_f;
            const int64_t val = std::max(l, r);
            if (val < best.i_f) {
              best.i_f = val;
              best.split = s;
              best.d_right = d2;
            }
          }
        }
    }
    return memo.emplace(k, best).first->second;
  }
};

struct Stage {
  std::vector<int> ops;
  int d;
  int64_t in_flight, b, k;
};
void collect(Search &S, int node, int lo, int hi, int bf, int kf, int64_t ib, int bb, int kb, int d, std::vector<Stage> &out) {
  const TNode &N = S.T[node];
  if (N.kind >= SERIES && hi - lo == 1) {
    const int c = N.kids[lo];
    return collect(S, c, 0, S.T[c].kind >= SERIES ? (int)S.T[c].kids.size() : 1, bf, kf, ib, bb, kb, d, out);
  }
  const Choice c = S.solve(node, lo, hi, bf, kf, ib, bb, kb, d);
  if (c.split == 0) {
    Stage st;
    if (N.kind >= SERIES) for (int q = lo; q < hi; ++q) st.ops.insert(st.ops.end(), S.T[N.kids[q]].ops.begin(), S.T[N.kids[q]].ops.end());
    else st.ops = N.ops;
    st.d = d;
    st.in_flight = c.i_f;
    st.b = S.bs[bf];
    st.k = S.ks[kf];
    out.push_back(st);
    return;
  }
  if (N.kind == SERIES) {
    const int64_t mid = S.solve(node, c.split, hi, c.bm, c.km, ib, bb, kb, c.d_right).i_f;
    collect(S, node, lo, c.split, bf, kf, mid, c.bm, c.km, d - c.d_right, out);
    collect(S, node, c.split, hi, c.bm, c.km, ib, bb, kb, c.d_right, out);
  } else {
    collect(S, node, lo, c.split, bf, kf, ib, bb, kb, d - c.d_right, out);
    collect(S, node, c.split, hi, bf, kf, ib, bb, kb, c.d_right, out);
  }
}

}  // namespace

extern "C" gpp_status_t gpp_partition_search(int32_t n_ops, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                                             int32_t n_b, const int64_t *b_values, const double *t, const double *w,
                                             const double *a, int32_t n_k, const int64_t *k_values, const double *x,
                                             double link_latency, double link_seconds_per_byte, int32_t n_devices,
                                             double memory_bytes, double sync_seconds_per_byte, int64_t mini_batch,
                                             double eps_rel, int32_t *stage_of_op, int32_t *n_stages, int32_t *stage_devices,
                                             int64_t *stage_in_flight, int64_t *stage_b, int64_t *stage_k, double *bottleneck,
                                             int64_t *dp_states) {
  if (n_ops <= 0 || n_edges < 0 || (n_edges > 0 && (!edge_from || !edge_to)) || !t || !w || !a || !stage_of_op || !n_stages ||
      !stage_devices || !stage_in_flight || !b_values || !k_values)
    return report_error(GPP_ERR_INVALID_ARG, "partition: null argument or empty graph");
  if (n_devices <= 0 || n_devices > 60000 || mini_batch <= 0 || !(eps_rel > 0) || !(memory_bytes > 0) || sync_seconds_per_byte < 0 ||
      link_latency < 0 || link_seconds_per_byte < 0)
    return report_error(GPP_ERR_INVALID_ARG, "partition: devices, mini-batch, memory and eps must be positive, costs non-negative");
  if (n_b <= 0 || n_b > 64 || n_k <= 0 || n_k > 64) return report_error(GPP_ERR_INVALID_ARG, "partition: 1 to 64 candidate micro-batch sizes and group sizes");
  for (int j = 0; j < n_b; ++j)
    if (b_values[j] <= 0 || b_values[j] > (1ll << 30)) return report_error(GPP_ERR_INVALID_ARG, "partition: micro-batch sizes must be positive");
  for (int j = 0; j < n_k; ++j)
    if (k_values[j] <= 0 || k_values[j] > (1ll << 30)) return report_error(GPP_ERR_INVALID_ARG, "partition: group sizes must be positive");
  if (n_ops > 30000) return report_error(GPP_ERR_UNSUPPORTED, "partition: more than 30000 operators");
  Builder B;
  B.n = n_ops;
  B.succ.assign(n_ops, {});
  B.nbr.assign(n_ops, {});
  std::vector<std::pair<int, int>> edges;
  for (int e = 0; e < n_edges; ++e) {
    const int u = edge_from[e], v = edge_to[e];
    if (u < 0 || u >= n_ops || v < 0 || v >= n_ops || u == v) return report_error(GPP_ERR_INVALID_ARG, "partition: edge endpoint out of range");
    if (x && !(x[e] >= 0)) return report_error(GPP_ERR_INVALID_ARG, "partition: edge bytes must be non-negative");
    B.succ[u].push_back(v);
    B.nbr[u].push_back(v);
    B.nbr[v].push_back(u);
    edges.push_back({u, v});
  }
  for (int o = 0; o < n_ops; ++o) {
    if (!(w[o] >= 0) || !(a[o] >= 0)) return report_error(GPP_ERR_INVALID_ARG, "partition: costs must be non-negative");
    for (int j = 0; j < n_b; ++j)
      if (!(t[(size_t)o * n_b + j] >= 0)) return report_error(GPP_ERR_INVALID_ARG, "partition: costs must be non-negative");
  }
  if (!B.closure()) return report_error(GPP_ERR_BAD_GRAPH, "partition: the operator graph has a cycle");
  std::vector<int> all(n_ops);
  for (int o = 0; o < n_ops; ++o) all[o] = o;
  const int root = B.build(all);
  std::vector<std::vector<int>> child_of(B.nodes.size());
  for (size_t id = 0; id < B.nodes.size(); ++id) {
    TNode &N = B.nodes[id];
    if (N.kind >= SERIES && N.kids.size() > 250) return report_error(GPP_ERR_UNSUPPORTED, "partition: more than 250 parts in one series or parallel composition");
    const size_t m = N.kind >= SERIES ? N.kids.size() : 1;
    // pt: one row of prefix sums per candidate micro-batch size, rows of m + 1 entries (the stride is pw's length)
    N.pt.assign((size_t)n_b * (m + 1), 0.0);
    N.pw.assign(m + 1, 0.0);
    N.pa.assign(m + 1, 0.0);
    const bool charged = link_latency > 0 || link_seconds_per_byte > 0;      // the cut of a stage is only needed then
    if (charged) child_of[id].assign(n_ops, -1);
    for (size_t c = 0; c < m; ++c) {
      double sw = 0, sa = 0;
      std::vector<double> st(n_b, 0.0);
      for (int o : (N.kind >= SERIES ? B.nodes[N.kids[c]].ops : N.ops)) {
        sw += w[o], sa += a[o];
        if (charged) child_of[id][o] = (int)c;
        for (int j = 0; j < n_b; ++j) st[j] += t[(size_t)o * n_b + j];
      }
      for (int j = 0; j < n_b; ++j) N.pt[(size_t)j * (m + 1) + c + 1] = N.pt[(size_t)j * (m + 1) + c] + st[j];
      N.pw[c + 1] = N.pw[c] + sw;
      N.pa[c + 1] = N.pa[c] + sa;
    }
  }
  const TNode &R = B.nodes[root];
  const int r_hi = R.kind >= SERIES ? (int)R.kids.size() : 1;
  Search S{B.nodes};
  S.bs.assign(b_values, b_values + n_b);
  S.ks.assign(k_values, k_values + n_k);
  S.memory = memory_bytes;
  S.sync = sync_seconds_per_byte;
  S.mini_batch = mini_batch;
  S.link_latency = link_latency;
  S.link_spb = link_seconds_per_byte;
  S.edges = &edges;
  S.x = x;
  S.child_of = child_of;
  // a bound no stage can exceed: everything on one device at its slowest micro-batch size, the dearest
  // synchronisation, every edge cut at the smallest micro-batch size
  double total_t = 0, total_w = 0, total_x = 0;
  for (int o = 0; o < n_ops; ++o) {
    double worst = 0;
    for (int j = 0; j < n_b; ++j) worst = std::max(worst, t[(size_t)o * n_b + j]);
    total_t += worst, total_w += w[o];
  }
  for (int e = 0; e < n_edges; ++e) total_x += x ? x[e] : 0.0;
  const int64_t b_min = *std::min_element(S.bs.begin(), S.bs.end());
  double t_r = total_t + 2.0 * total_w * sync_seconds_per_byte / (double)mini_batch + n_edges * link_latency / (double)b_min +
               total_x * link_seconds_per_byte;
  double t_l = 0.0;
  int64_t states = 0;
  // SearchStageGraph: every configuration of the first stage(s); the better result holds fewer in-flight samples
  int best_b = 0, best_k = 0;
  auto feasible = [&](double bound) {
    S.t_max = bound;
    S.memo.clear();
    int64_t best = INF;
    for (int bf = 0; bf < n_b; ++bf)
      for (int kf = 0; kf < n_k; ++kf) {
        const int64_t v = S.solve(root, 0, r_hi, bf, kf, 0, -1, 0, n_devices).i_f;
        if (v < best) best = v, best_b = bf, best_k = kf;
      }
    states += S.states;
    S.states = 0;
    return best < INF;
  };
  *n_stages = 0;
  if (bottleneck) *bottleneck = 0.0;
  if (!feasible(t_r)) {          // no stage graph fits the memory: not an error, there is simply no strategy
    if (dp_states) *dp_states = states;
    return GPP_OK;
  }
  while (t_r - t_l > eps_rel * t_r) {
    const double t_m = 0.5 * (t_l + t_r);
    if (feasible(t_m)) t_r = t_m;
    else t_l = t_m;
  }
  feasible(t_r);
  std::vector<Stage> stages;
  collect(S, root, 0, r_hi, best_b, best_k, 0, -1, 0, n_devices, stages);
  double worst = 0.0;
  for (size_t s = 0; s < stages.size(); ++s) {
    double st = 0, sw = 0;
    int bj = 0;
    for (int j = 0; j < n_b; ++j) if (S.bs[j] == stages[s].b) bj = j;
    Bits in(n_ops);
    for (int o : stages[s].ops) {
      stage_of_op[o] = (int32_t)s;
      st += t[(size_t)o * n_b + bj];
      sw += w[o];
      in.set(o);
    }
    int n_cut = 0;
    double cut_bytes = 0;
    for (int e = 0; e < n_edges; ++e)
      if (in.has(edges[e].first) != in.has(edges[e].second)) ++n_cut, cut_bytes += x ? x[e] : 0.0;
    stage_devices[s] = stages[s].d;
    stage_in_flight[s] = stages[s].in_flight;
    if (stage_b) stage_b[s] = stages[s].b;
    if (stage_k) stage_k[s] = stages[s].k;
    worst = std::max(worst, S.stage_time(st, sw, stages[s].d, n_cut, cut_bytes, stages[s].b));
  }
  *n_stages = (int32_t)stages.size();
  if (bottleneck) *bottleneck = worst;
  if (dp_states) *dp_states = states;
  return GPP_OK;
}

// the default schedule configuration of section 6: one micro-batch size, 1F1B everywhere, tensors between
// stages not charged
extern "C" gpp_status_t gpp_partition(int32_t n_ops, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                                      const double *t, const double *w, const double *a, int32_t n_devices, int64_t b,
                                      double memory_bytes, double sync_seconds_per_byte, int64_t mini_batch,
                                      double eps_rel, int32_t *stage_of_op, int32_t *n_stages, int32_t *stage_devices,
                                      int64_t *stage_in_flight, double *bottleneck, int64_t *dp_states) {
  if (b <= 0) return report_error(GPP_ERR_INVALID_ARG, "partition: devices, micro-batch size, mini-batch, memory and eps must be positive");
  const int64_t one = 1;
  return gpp_partition_search(n_ops, n_edges, edge_from, edge_to, 1, &b, t, w, a, 1, &one, nullptr, 0.0, 0.0, n_devices,
                              memory_bytes, sync_seconds_per_byte, mini_batch, eps_rel, stage_of_op, n_stages, stage_devices,
                              stage_in_flight, nullptr, nullptr, bottleneck, dp_states);
}

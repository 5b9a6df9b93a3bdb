// Pipeline stage partitioner (paper section 5, Alg. 1): series-parallel structure of the operator graph,
// a dynamic programme over it whose value is the smallest number of in-flight samples at the first
// stages of a sub-graph under a bound on every stage's time per sample, and a binary search on that
// bound.  Host code; no kernels.  The cost model and the readings of what the paper leaves open are
// stated with gpp_partition in the header.
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
  // prefix sums over the children (index c: children [0, c)); for LEAF / BLOCK one entry pair [0, total]
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
constexpr int64_t INF = INT64_MAX / 4;
struct Choice {
  int64_t i_f = INF;     // in-flight samples at the first stages of the sub-graph (the DP value)
  int split = 0;         // 0: one stage; else children [lo, split) and [split, hi)
  int d_right = 0;       // devices of the right part
};

struct Search {
  const std::vector<TNode> &T;
  int64_t b;
  double memory, sync, t_max = 0;
  int64_t mini_batch;
  std::unordered_map<uint64_t, Choice> memo;
  int64_t states = 0;

  static uint64_t key(int node, int lo, int hi, int64_t ib, int d) {
    return ((uint64_t)node << 48) | ((uint64_t)lo << 40) | ((uint64_t)hi << 32) | ((uint64_t)ib << 16) | (uint64_t)d;
  }
  double stage_time(double t, double w, int d) const {
    const double compute = t / d;
    return d == 1 ? compute : compute + 2.0 * (d - 1) / d * w * sync / (double)mini_batch;
  }
  // children [lo, hi) of `node` (a leaf or block: lo = 0, hi = 1), successor stages hold ib * b samples
  // (0: no successor), d devices
  const Choice &solve(int node, int lo, int hi, int64_t ib, int d) {
    const TNode &N = T[node];
    if (N.kind >= SERIES && hi - lo == 1) return solve(N.kids[lo], 0, T[N.kids[lo]].kind >= SERIES ? (int)T[N.kids[lo]].kids.size() : 1, ib, d);
    const uint64_t k = key(node, lo, hi, ib, d);
    auto it = memo.find(k);
    if (it != memo.end()) return it->second;
    ++states;
    Choice best;
    const double t = N.pt[hi] - N.pt[lo], w = N.pw[hi] - N.pw[lo], a = N.pa[hi] - N.pa[lo];
    // one stage: 1F1B in front of 1F1B at the same micro-batch size adds one micro-batch (appendix table)
    {
      int64_t i_x = b;
      if (ib > 0) gpp_compute_in_flight(1, b, 1, b, ib * b, &i_x);
      if (stage_time(t, w, d) <= t_max && w + (double)i_x / d * a <= memory) best.i_f = i_x;
    }
    if (N.kind >= SERIES && d >= 2) {
      for (int s = lo + 1; s < hi; ++s)
        for (int d2 = 1; d2 < d; ++d2) {
          int64_t val;
          if (N.kind == SERIES) {
            const int64_t mid = solve(node, s, hi, ib, d2).i_f;       // the later part first: its first stages
            if (mid >= INF) continue;                                  // are what the earlier part feeds
            val = solve(node, lo, s, mid / b, d - d2).i_f;
          } else {
            const int64_t l = solve(node, lo, s, ib, d - d2).i_f;
            if (l >= INF) continue;
            const int64_t r = solve(node, s, hi, ib, d2).i_f;
            val = std::max(l, r);                                      // the producer in front holds the larger
          }
          if (val < best.i_f) {
            best.i_f = val;
            best.split = s;
            best.d_right = d2;
          }
        }
    }
    return memo.emplace(k, best).first->second;
  }
};

struct Stage {
  std::vector<int> ops;
  int d;
  int64_t in_flight;
};
void collect(Search &S, int node, int lo, int hi, int64_t ib, int d, std::vector<Stage> &out) {
  const TNode &N = S.T[node];
  if (N.kind >= SERIES && hi - lo == 1) {
    const int c = N.kids[lo];
    return collect(S, c, 0, S.T[c].kind >= SERIES ? (int)S.T[c].kids.size() : 1, ib, d, out);
  }
  const Choice c = S.solve(node, lo, hi, ib, d);
  if (c.split == 0) {
    Stage st;
    if (N.kind >= SERIES) for (int q = lo; q < hi; ++q) st.ops.insert(st.ops.end(), S.T[N.kids[q]].ops.begin(), S.T[N.kids[q]].ops.end());
    else st.ops = N.ops;
    st.d = d;
    st.in_flight = c.i_f;
    out.push_back(st);
    return;
  }
  if (N.kind == SERIES) {
    const int64_t mid = S.solve(node, c.split, hi, ib, c.d_right).i_f;
    collect(S, node, lo, c.split, mid / S.b, d - c.d_right, out);
    collect(S, node, c.split, hi, ib, c.d_right, out);
  } else {
    collect(S, node, lo, c.split, ib, d - c.d_right, out);
    collect(S, node, c.split, hi, ib, c.d_right, out);
  }
}

}  // namespace

extern "C" gpp_status_t gpp_partition(int32_t n_ops, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                                      const double *t, const double *w, const double *a, int32_t n_devices, int64_t b,
                                      double memory_bytes, double sync_seconds_per_byte, int64_t mini_batch,
                                      double eps_rel, int32_t *stage_of_op, int32_t *n_stages, int32_t *stage_devices,
                                      int64_t *stage_in_flight, double *bottleneck, int64_t *dp_states) {
  if (n_ops <= 0 || n_edges < 0 || (n_edges > 0 && (!edge_from || !edge_to)) || !t || !w || !a || !stage_of_op || !n_stages ||
      !stage_devices || !stage_in_flight)
    return report_error(GPP_ERR_INVALID_ARG, "partition: null argument or empty graph");
  if (n_devices <= 0 || n_devices > 60000 || b <= 0 || mini_batch <= 0 || !(eps_rel > 0) || !(memory_bytes > 0) || sync_seconds_per_byte < 0)
    return report_error(GPP_ERR_INVALID_ARG, "partition: devices, micro-batch size, mini-batch, memory and eps must be positive");
  if (n_ops > 30000) return report_error(GPP_ERR_UNSUPPORTED, "partition: more than 30000 operators");
  Builder B;
  B.n = n_ops;
  B.succ.assign(n_ops, {});
  B.nbr.assign(n_ops, {});
  for (int e = 0; e < n_edges; ++e) {
    const int u = edge_from[e], v = edge_to[e];
    if (u < 0 || u >= n_ops || v < 0 || v >= n_ops || u == v) return report_error(GPP_ERR_INVALID_ARG, "partition: edge endpoint out of range");
    B.succ[u].push_back(v);
    B.nbr[u].push_back(v);
    B.nbr[v].push_back(u);
  }
  for (int o = 0; o < n_ops; ++o)
    if (!(t[o] >= 0) || !(w[o] >= 0) || !(a[o] >= 0)) return report_error(GPP_ERR_INVALID_ARG, "partition: costs must be non-negative");
  if (!B.closure()) return report_error(GPP_ERR_BAD_GRAPH, "partition: the operator graph has a cycle");
  std::vector<int> all(n_ops);
  for (int o = 0; o < n_ops; ++o) all[o] = o;
  const int root = B.build(all);
  for (TNode &N : B.nodes) {
    if (N.kind >= SERIES && N.kids.size() > 250) return report_error(GPP_ERR_UNSUPPORTED, "partition: more than 250 parts in one series or parallel composition");
    const size_t m = N.kind >= SERIES ? N.kids.size() : 1;
    N.pt.assign(m + 1, 0.0);
    N.pw.assign(m + 1, 0.0);
    N.pa.assign(m + 1, 0.0);
    for (size_t c = 0; c < m; ++c) {
      double st = 0, sw = 0, sa = 0;
      for (int o : (N.kind >= SERIES ? B.nodes[N.kids[c]].ops : N.ops)) st += t[o], sw += w[o], sa += a[o];
      N.pt[c + 1] = N.pt[c] + st;
      N.pw[c + 1] = N.pw[c] + sw;
      N.pa[c + 1] = N.pa[c] + sa;
    }
  }
  const TNode &R = B.nodes[root];
  const int r_hi = R.kind >= SERIES ? (int)R.kids.size() : 1;
  Search S{B.nodes, b, memory_bytes, sync_seconds_per_byte, 0.0, mini_batch, {}, 0};
  // a bound no stage can exceed: everything on one device, plus the dearest synchronisation
  double total_t = 0, total_w = 0;
  for (int o = 0; o < n_ops; ++o) total_t += t[o], total_w += w[o];
  double t_r = total_t + 2.0 * total_w * sync_seconds_per_byte / (double)mini_batch, t_l = 0.0;
  int64_t states = 0;
  auto feasible = [&](double bound) {
    S.t_max = bound;
    S.memo.clear();
    const bool ok = S.solve(root, 0, r_hi, 0, n_devices).i_f < INF;
    states += S.states;
    S.states = 0;
    return ok;
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
  collect(S, root, 0, r_hi, 0, n_devices, stages);
  double worst = 0.0;
  for (size_t s = 0; s < stages.size(); ++s) {
    double st = 0, sw = 0;
    for (int o : stages[s].ops) {
      stage_of_op[o] = (int32_t)s;
      st += t[o];
      sw += w[o];
    }
    stage_devices[s] = stages[s].d;
    stage_in_flight[s] = stages[s].in_flight;
    worst = std::max(worst, S.stage_time(st, sw, stages[s].d));
  }
  *n_stages = (int32_t)stages.size();
  if (bottleneck) *bottleneck = worst;
  if (dp_states) *dp_states = states;
  return GPP_OK;
}

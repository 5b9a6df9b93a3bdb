// Static micro-batch scheduler of a stage graph (paper section 6, Alg. 2, and the appendix
// "Generalized Per-stage kFkB Schedule"): in-flight sample counts, the choice of k per stage, and
// the order of forward and backward passes of one stage.  Integer host code; no kernels.
#include <algorithm>
#include <string>
#include <vector>

#include "../../include/gpp.h"

namespace gpp {
gpp_status_t report_error(gpp_status_t st, const std::string &msg);

// The appendix table, organised by how the group sizes X = k_x b_x and Y = k_y b_y compare; every
// branch names the table rows it stands for (rows counted from the top).
static int64_t in_flight(int64_t kx, int64_t bx, int64_t ky, int64_t by, int64_t iy) {
  const int64_t X = kx * bx, Y = ky * by, m = std::max(bx, by);
  if (X < Y) {
    if (m < X) return iy + 2 * m;              // row 1
    if (m == X) return iy + m;                 // row 2
    return iy + by;                            // row 9: b_x <= X < b_y <= Y
  }
  if (X == Y) return m == Y ? iy + Y : iy + 2 * m;   // rows 7 and 8
  // X > Y
  if (bx > Y) return iy + X - Y + bx;          // row 10: b_y <= Y < b_x <= X
  if (m == Y) return iy + X;                   // rows 4 and 6
  return iy + X - Y + 2 * m;                   // rows 3 and 5
}

static bool fits(int64_t a, int64_t b) { return a > 0 && b > 0 && a <= (int64_t)1 << 30 && b <= (int64_t)1 << 30; }
}  // namespace gpp

using namespace gpp;

extern "C" {

gpp_status_t gpp_compute_in_flight(int64_t k_x, int64_t b_x, int64_t k_y, int64_t b_y, int64_t i_y, int64_t *i_x) {
  if (!i_x) return report_error(GPP_ERR_INVALID_ARG, "i_x is null");
  if (!fits(k_x, b_x) || !fits(k_y, b_y) || i_y <= 0 || i_y > (int64_t)1 << 60)
    return report_error(GPP_ERR_INVALID_ARG, "k, b and i must be positive (k, b at most 2^30)");
  *i_x = in_flight(k_x, b_x, k_y, b_y, i_y);
  return GPP_OK;
}

gpp_status_t gpp_assign_schedules(int32_t n_stages, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                                  const int64_t *b, const int32_t *k_begin, const int64_t *k_values, int64_t *i_out,
                                  int64_t *k_out) {
  if (n_stages <= 0 || n_edges < 0 || !b || !k_begin || !k_values || !i_out || !k_out || (n_edges > 0 && (!edge_from || !edge_to)))
    return report_error(GPP_ERR_INVALID_ARG, "assign_schedules: null argument or empty stage graph");
  std::vector<std::vector<int>> succ(n_stages);
  std::vector<int> pending(n_stages, 0);   // successors not yet scheduled
  std::vector<std::vector<int>> pred(n_stages);
  for (int e = 0; e < n_edges; ++e) {
    const int x = edge_from[e], y = edge_to[e];
    if (x < 0 || x >= n_stages || y < 0 || y >= n_stages) return report_error(GPP_ERR_INVALID_ARG, "assign_schedules: edge endpoint out of range");
    succ[x].push_back(y);
    pred[y].push_back(x);
    ++pending[x];
  }
  for (int x = 0; x < n_stages; ++x) {
    if (b[x] <= 0 || b[x] > (int64_t)1 << 30) return report_error(GPP_ERR_INVALID_ARG, "assign_schedules: micro-batch sizes must be positive");
    if (k_begin[x + 1] <= k_begin[x]) return report_error(GPP_ERR_INVALID_ARG, "assign_schedules: a stage has no candidate k");
    for (int c = k_begin[x]; c < k_begin[x + 1]; ++c)
      if (k_values[c] <= 0 || k_values[c] > (int64_t)1 << 30) return report_error(GPP_ERR_INVALID_ARG, "assign_schedules: k must be positive");
  }
  // last stages first, then against the direction of the edges
  std::vector<int> ready;
  for (int x = 0; x < n_stages; ++x)
    if (pending[x] == 0) ready.push_back(x);
  int done = 0;
  while (!ready.empty()) {
    const int x = ready.back();
    ready.pop_back();
    ++done;
    std::vector<int64_t> ks(k_values + k_begin[x], k_values + k_begin[x + 1]);
    std::sort(ks.begin(), ks.end());       // equal counts: the smallest k
    int64_t best_i = -1, best_k = 0;
    for (int64_t kx : ks) {
      int64_t worst = succ[x].empty() ? kx * b[x] : 0;
      for (int y : succ[x]) worst = std::max(worst, in_flight(kx, b[x], k_out[y], b[y], i_out[y]));
      if (best_i < 0 || worst < best_i) best_i = worst, best_k = kx;
    }
    i_out[x] = best_i;
    k_out[x] = best_k;
    for (int p : pred[x])
      if (--pending[p] == 0) ready.push_back(p);
  }
  if (done != n_stages) return report_error(GPP_ERR_BAD_GRAPH, "assign_schedules: the stage graph has a cycle");
  return GPP_OK;
}

gpp_status_t gpp_schedule_tasks(int64_t n_micro, int64_t i, int64_t k, int64_t b, int32_t *tasks) {
  if (n_micro < 0 || n_micro > (int64_t)1 << 30 || i <= 0 || k <= 0 || b <= 0) return report_error(GPP_ERR_INVALID_ARG, "schedule_tasks: n >= 0 and i, k, b > 0");
  if (n_micro > 0 && !tasks) return report_error(GPP_ERR_INVALID_ARG, "tasks is null");
  const int64_t cap = std::max<int64_t>(1, i / b);
  // kFkB written as runs: warm-up, then groups of backward and forward passes, then cool-down
  const int64_t warm = std::min(cap, n_micro), group = std::min(k, warm);
  int64_t f = 0, r = 0, t = 0;
  for (; f < warm; ++f) tasks[t++] = (int32_t)(f + 1);
  while (f < n_micro) {
    for (int64_t e = std::min(r + group, f); r < e; ++r) tasks[t++] = (int32_t)-(r + 1);
    for (int64_t e = std::min(f + group, n_micro); f < e; ++f) tasks[t++] = (int32_t)(f + 1);
  }
  for (; r < n_micro; ++r) tasks[t++] = (int32_t)-(r + 1);
  return GPP_OK;
}

}  // extern "C"

// Host-side rules of the pruning search: how many filters to prune given the structure of
// the program chosen for a layer (Section 3.5), and the order in which tasks are tried
// (Section 3.3).  No device work.
#include "common.hpp"

#include <algorithm>
#include <numeric>
#include <vector>

namespace cprune {
namespace {

// Smallest slice of a box of filters with side lengths f[0..n): product / largest side.
// Returns 0 on invalid input or overflow.
int64_t min_prunable(const int64_t* f, int n) {
  if (!f || n < 1) return 0;
  int64_t prod = 1, largest = 0;
  for (int i = 0; i < n; ++i) {
    if (f[i] < 1) return 0;
    if (prod > INT64_MAX / f[i]) return 0;
    prod *= f[i];
    largest = std::max(largest, f[i]);
  }
  return prod / largest;
}

}  // namespace
}  // namespace cprune

using namespace cprune;

extern "C" int cprune_lcm_step(const int64_t* l1, int n1, const int64_t* l2, int n2, int64_t* step_out) {
  if (!step_out) return CPRUNE_ERR_INVALID_ARG;
  const int64_t a = min_prunable(l1, n1), b = min_prunable(l2, n2);
  if (a < 1 || b < 1) return CPRUNE_ERR_INVALID_ARG;
  const int64_t g = std::gcd(a, b);
  if (a / g > INT64_MAX / b) return CPRUNE_ERR_UNSUPPORTED;
  *step_out = a / g * b;
  return CPRUNE_OK;
}

extern "C" int cprune_prune_count(int c_out, int64_t step, int* count_out) {
  if (!count_out || c_out < 1 || step < 1) return CPRUNE_ERR_INVALID_ARG;
  const int64_t keep = ((int64_t)c_out - 1) / step * step;
  *count_out = keep >= 1 ? (int)(c_out - keep) : 0;
  return CPRUNE_OK;
}

extern "C" int cprune_variant_filter_splits(int v, int c_out, int64_t* main_loop, int64_t* epilogue,
                                            int* unit_out) {
  if (v < 0 || v >= num_variants() || c_out < 1 || !main_loop || !epilogue || !unit_out) return CPRUNE_ERR_INVALID_ARG;
  const TileVariant& tv = variant(v);
  const int tile_m = tv.tile_m();
  const int unit = tv.blk32 ? 32 : 16;   // rows of the MFMA block the variant is built on
  const int64_t tiles = (c_out + tile_m - 1) / tile_m;
  const int64_t blocks = std::min<int64_t>(tile_m / unit, (c_out + unit - 1) / unit);
  // the reduction loop walks (tile, MFMA row block of the tile); the store loop walks the same
  // blocks (inside a block the rows are the MFMA result layout, not a loop)
  main_loop[0] = tiles; main_loop[1] = blocks;
  epilogue[0] = tiles; epilogue[1] = blocks;
  *unit_out = unit;
  return CPRUNE_OK;
}

extern "C" int cprune_variant_prune_step(int v, int c_out, int64_t* step_out) {
  if (!step_out) return CPRUNE_ERR_INVALID_ARG;
  int64_t ml[2], ep[2];
  int unit = 0;
  int rc = cprune_variant_filter_splits(v, c_out, ml, ep, &unit);
  if (rc != CPRUNE_OK) return rc;
  int64_t blocks = 0;
  rc = cprune_lcm_step(ml, 2, ep, 2, &blocks);
  if (rc != CPRUNE_OK) return rc;
  *step_out = blocks * unit;
  return CPRUNE_OK;
}

extern "C" int cprune_order_tasks(const double* exec_time, const int* n_subgraphs, int n_tasks, int* order_out,
                                  double* impact_out) {
  if (!exec_time || !n_subgraphs || !order_out || n_tasks < 0) return CPRUNE_ERR_INVALID_ARG;
  std::vector<double> impact(n_tasks);
  for (int i = 0; i < n_tasks; ++i) {
    if (!(exec_time[i] >= 0.0) || n_subgraphs[i] < 0) return CPRUNE_ERR_INVALID_ARG;
    impact[i] = exec_time[i] * (double)n_subgraphs[i];
  }
  std::vector<int> order(n_tasks);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return impact[a] > impact[b]; });
  for (int i = 0; i < n_tasks; ++i) {
    order_out[i] = order[i];
    if (impact_out) impact_out[i] = impact[i];
  }
  return CPRUNE_OK;
}

// ---- Algorithm 1 (Section 3.2) as a state machine over reported measurements ---------------
// The caller owns models, tuning, latency measurement and accuracy; this object owns the
// decisions: which task is tried next, whether a measured candidate passes the latency
// gate, whether its accuracy keeps it, which tasks are out for good, and when the search
// ends.  Between cprune_search_next_task and the matching report the object waits for
// exactly one of: exhausted, latency (then, if the gate passed, accuracy).
namespace {

enum SearchWait { kIdle = 0, kWaitCandidate = 1, kWaitAccuracy = 2 };

struct LogEntry { int64_t task; double l_m, l_t, a_s; int verdict; };

}  // namespace

struct cprune_search {
  double a_goal, alpha, beta;
  int64_t max_passes;
  bool started = false, finished = false;
  double l_t = 0.0, a_p = 0.0;
  std::vector<int64_t> todo;        // tasks still in play, by descending impact of the accepted model
  std::vector<int64_t> out;         // tasks that left the search for good
  std::vector<int64_t> pass;        // the list as it stood when the current pass began
  size_t cursor = 0;
  bool in_pass = false, progress = false;
  int64_t passes = 0;
  int wait = kIdle;
  int64_t current = 0;
  double current_l_m = 0.0;
  std::vector<LogEntry> log;
};

static bool is_out(const cprune_search* s, int64_t t) {
  return std::find(s->out.begin(), s->out.end(), t) != s->out.end();
}

static void drop_task(cprune_search* s, int64_t t) {
  s->todo.erase(std::remove(s->todo.begin(), s->todo.end(), t), s->todo.end());
  if (!is_out(s, t)) s->out.push_back(t);
  s->progress = true;
}

extern "C" int cprune_search_create(double a_goal, double alpha, double beta, int64_t max_passes,
                                    cprune_search** out) {
  if (!out || !(alpha >= 0.0) || !(beta > 0.0) || max_passes < 0 || a_goal != a_goal) return CPRUNE_ERR_INVALID_ARG;
  cprune_search* s = new cprune_search();
  s->a_goal = a_goal; s->alpha = alpha; s->beta = beta; s->max_passes = max_passes;
  *out = s;
  return CPRUNE_OK;
}

extern "C" int cprune_search_start(cprune_search* s, const int64_t* tasks_by_impact, int n_tasks, double l_m,
                                   double a_p) {
  if (!s || s->started || n_tasks < 0 || (n_tasks > 0 && !tasks_by_impact) || !(l_m >= 0.0)) return CPRUNE_ERR_INVALID_ARG;
  s->todo.assign(tasks_by_impact, tasks_by_impact + n_tasks);
  s->l_t = s->beta * l_m;
  s->a_p = a_p;
  s->started = true;
  return CPRUNE_OK;
}

extern "C" int cprune_search_next_task(cprune_search* s, int64_t* task_out, int* done_out) {
  if (!s || !task_out || !done_out || !s->started || s->wait != kIdle) return CPRUNE_ERR_INVALID_ARG;
  *done_out = 0;
  for (;;) {
    if (s->finished) { *done_out = 1; return CPRUNE_OK; }
    if (!s->in_pass) {
      if (!(s->a_p > s->a_goal) || s->todo.empty() || s->passes >= s->max_passes) { s->finished = true; continue; }
      s->pass = s->todo; s->cursor = 0; s->progress = false; s->in_pass = true; ++s->passes;
    }
    if (s->cursor < s->pass.size()) {
      s->current = s->pass[s->cursor++];
      s->wait = kWaitCandidate;
      *task_out = s->current;
      return CPRUNE_OK;
    }
    s->in_pass = false;                       // the pass tried every task of its list
    if (!s->progress) s->finished = true;     // and changed nothing: another pass would repeat it
  }
}

extern "C" int cprune_search_report_exhausted(cprune_search* s) {
  if (!s || s->wait != kWaitCandidate) return CPRUNE_ERR_INVALID_ARG;
  const double nan = __builtin_nan("");
  s->log.push_back(LogEntry{s->current, nan, s->l_t, nan, CPRUNE_SEARCH_EXHAUSTED});
  drop_task(s, s->current);
  s->wait = kIdle;
  return CPRUNE_OK;
}

extern "C" int cprune_search_report_latency(cprune_search* s, double l_m, int* needs_accuracy_out) {
  if (!s || !needs_accuracy_out || s->wait != kWaitCandidate) return CPRUNE_ERR_INVALID_ARG;
  if (l_m < s->l_t) {
    s->current_l_m = l_m;
    s->wait = kWaitAccuracy;
    *needs_accuracy_out = 1;
    return CPRUNE_OK;
  }
  s->log.push_back(LogEntry{s->current, l_m, s->l_t, __builtin_nan(""), CPRUNE_SEARCH_SLOW});
  s->wait = kIdle;
  *needs_accuracy_out = 0;
  return CPRUNE_OK;
}

extern "C" int cprune_search_report_accuracy(cprune_search* s, double a_s, const int64_t* tasks_by_impact,
                                             int n_tasks, int* accepted_out) {
  if (!s || !accepted_out || s->wait != kWaitAccuracy || n_tasks < 0 || (n_tasks > 0 && !tasks_by_impact))
    return CPRUNE_ERR_INVALID_ARG;
  s->wait = kIdle;
  if (a_s < s->alpha * s->a_p) {
    s->log.push_back(LogEntry{s->current, s->current_l_m, s->l_t, a_s, CPRUNE_SEARCH_INACCURATE});
    drop_task(s, s->current);
    *accepted_out = 0;
    return CPRUNE_OK;
  }
  s->log.push_back(LogEntry{s->current, s->current_l_m, s->l_t, a_s, CPRUNE_SEARCH_ACCEPTED});
  s->todo.clear();
  for (int i = 0; i < n_tasks; ++i)
    if (!is_out(s, tasks_by_impact[i])) s->todo.push_back(tasks_by_impact[i]);
  s->l_t = s->beta * s->current_l_m;
  s->a_p = a_s;
  s->progress = true;
  s->in_pass = false;          // the next pass walks the accepted model's list from its head
  *accepted_out = 1;
  return CPRUNE_OK;
}

extern "C" int cprune_search_log_size(const cprune_search* s) { return s ? (int)s->log.size() : 0; }

extern "C" int cprune_search_log_entry(const cprune_search* s, int index, int64_t* task_out, double* l_m_out,
                                       double* l_t_out, double* a_s_out, int* verdict_out) {
  if (!s || index < 0 || index >= (int)s->log.size() || !task_out || !l_m_out || !l_t_out || !a_s_out || !verdict_out)
    return CPRUNE_ERR_INVALID_ARG;
  const LogEntry& e = s->log[index];
  *task_out = e.task; *l_m_out = e.l_m; *l_t_out = e.l_t; *a_s_out = e.a_s; *verdict_out = e.verdict;
  return CPRUNE_OK;
}

extern "C" int cprune_search_destroy(cprune_search* s) {
  if (!s) return CPRUNE_ERR_INVALID_ARG;
  delete s;
  return CPRUNE_OK;
}

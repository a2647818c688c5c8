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

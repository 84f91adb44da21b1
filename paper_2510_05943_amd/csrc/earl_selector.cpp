// Parallelism-selector table (Section 2 of the paper, "Parallelism Selector"; Equation 1 in
// Section 3.1): host code only.  The reading of the paper that fixes every rule below is stated in
// earl_selector.h.
#include "earl_selector.h"

#include <cmath>
#include <new>
#include <vector>

struct earl_selector {
  std::vector<int64_t> lengths;    // measured context lengths, ascending
  std::vector<int32_t> best;       // per measured length: best feasible configuration or -1
  std::vector<int32_t> range_of;   // per measured length: index of its range
  std::vector<int64_t> range_hi;   // per range: largest measured length in it
  std::vector<int32_t> range_cfg;  // per range: configuration
  double hysteresis = 0.0;
  int32_t current_cfg = -1;
  int32_t current_range = -1;
};

namespace {

inline bool feasible(double tgs) { return std::isfinite(tgs) && tgs > 0.0; }

// Range of an averaged context length: the first measured length that is >= x, else the last.
int32_t range_of_length(const earl_selector& s, double x) {
  size_t lo = 0, hi = s.lengths.size();   // first j with lengths[j] >= x
  while (lo < hi) {
    const size_t mid = (lo + hi) / 2;
    if ((double)s.lengths[mid] >= x) hi = mid; else lo = mid + 1;
  }
  if (lo == s.lengths.size()) lo = s.lengths.size() - 1;
  return s.range_of[lo];
}

}  // namespace

extern "C" {

double earl_speedup_percent(double tgs_a, double tgs_b) { return (tgs_b - tgs_a) / tgs_a * 100.0; }

int32_t earl_selector_build(const int64_t* context_lengths, int32_t n_lengths, int32_t n_configs,
                            const double* tgs, double hysteresis, int32_t initial_config,
                            earl_selector** out) {
  if (!context_lengths || !tgs || !out) return EARL_INVALID_ARG;
  if (n_lengths < 1 || n_lengths > EARL_SELECTOR_MAX_LENGTHS) return EARL_INVALID_ARG;
  if (n_configs < 1 || n_configs > EARL_SELECTOR_MAX_CONFIGS) return EARL_INVALID_ARG;
  if (!std::isfinite(hysteresis) || hysteresis < 0.0) return EARL_INVALID_ARG;
  if (initial_config < -1 || initial_config >= n_configs) return EARL_INVALID_ARG;
  for (int32_t j = 0; j < n_lengths; ++j) {
    if (context_lengths[j] < 1) return EARL_INVALID_ARG;
    if (j > 0 && context_lengths[j] <= context_lengths[j - 1]) return EARL_INVALID_ARG;
  }
  earl_selector* s = new (std::nothrow) earl_selector;
  if (!s) return EARL_CAPACITY;
  s->lengths.assign(context_lengths, context_lengths + n_lengths);
  s->hysteresis = hysteresis;
  s->current_cfg = initial_config;
  s->best.resize(n_lengths);
  s->range_of.resize(n_lengths);
  for (int32_t j = 0; j < n_lengths; ++j) {
    int32_t arg = -1;
    double top = 0.0;
    for (int32_t k = 0; k < n_configs; ++k) {
      const double v = tgs[(size_t)j * n_configs + k];
      if (feasible(v) && (arg < 0 || v > top)) { arg = k; top = v; }
    }
    s->best[j] = arg;
    if (j == 0 || arg != s->best[j - 1]) {
      s->range_hi.push_back(context_lengths[j]);
      s->range_cfg.push_back(arg);
    } else {
      s->range_hi.back() = context_lengths[j];
    }
    s->range_of[j] = (int32_t)s->range_cfg.size() - 1;
  }
  *out = s;
  return EARL_OK;
}

int32_t earl_selector_n_ranges(const earl_selector* sel, int32_t* out) {
  if (!sel || !out) return EARL_INVALID_ARG;
  *out = (int32_t)sel->range_cfg.size();
  return EARL_OK;
}

int32_t earl_selector_get_ranges(const earl_selector* sel, int64_t* range_hi, int32_t* config) {
  if (!sel) return EARL_INVALID_ARG;
  for (size_t t = 0; t < sel->range_cfg.size(); ++t) {
    if (range_hi) range_hi[t] = sel->range_hi[t];
    if (config) config[t] = sel->range_cfg[t];
  }
  return EARL_OK;
}

int32_t earl_selector_best_at(const earl_selector* sel, int32_t j, int32_t* config) {
  if (!sel || !config || j < 0 || (size_t)j >= sel->best.size()) return EARL_INVALID_ARG;
  *config = sel->best[j];
  return EARL_OK;
}

int32_t earl_selector_observe(earl_selector* sel, double avg_context_length, int32_t* config,
                              int32_t* switched) {
  if (!sel || !config || !switched) return EARL_INVALID_ARG;
  if (!std::isfinite(avg_context_length) || avg_context_length <= 0.0) return EARL_INVALID_ARG;
  int32_t t = range_of_length(*sel, avg_context_length);
  if (sel->current_range >= 0 && t < sel->current_range) {
    // a shorter range: only as far down as the inflated average allows
    const int32_t t_infl = range_of_length(*sel, avg_context_length * (1.0 + sel->hysteresis));
    t = t_infl < sel->current_range ? t_infl : sel->current_range;
  }
  const int32_t cfg = sel->range_cfg[t];
  if (cfg < 0) {
    *config = -1;
    *switched = 0;
    return EARL_NO_FEASIBLE_CONFIG;
  }
  *config = cfg;
  *switched = cfg != sel->current_cfg ? 1 : 0;
  sel->current_cfg = cfg;
  sel->current_range = t;
  return EARL_OK;
}

int32_t earl_selector_current_range(const earl_selector* sel, int32_t* range) {
  if (!sel || !range) return EARL_INVALID_ARG;
  *range = sel->current_range;
  return EARL_OK;
}

int32_t earl_selector_destroy(earl_selector* sel) {
  delete sel;
  return EARL_OK;
}

}  // extern "C"

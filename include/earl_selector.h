/*
 * earl_selector.h - C ABI of the parallelism-selector table (host only, no GPU work).
 *
 * Section 2 of the paper, "Parallelism Selector": at the start of training the throughput of every
 * candidate parallelism configuration is measured at several context lengths, and the best
 * configuration is kept for every context-length range; during training the averaged context
 * length of the generated sequences is monitored, and when it enters another range the system
 * switches to that range's configuration before the next Rollout stage.  Section 3.1, "Metrics":
 * throughput is tokens per GPU per second (TGS), and Equation 1 defines the relative speedup of
 * one configuration over another.
 *
 * The paper gives no further rule; this library's reading:
 *   - the table is measured at context lengths l_0 < l_1 < ... < l_{M-1}; a measurement that is
 *     not a positive finite number marks a configuration that failed there (out of memory,
 *     Section 3.2) and is never chosen for that length;
 *   - the best configuration at l_j is the feasible one with the largest TGS, the lowest index
 *     among equals;
 *   - an averaged context length x belongs to the first measured length that is >= x (what was
 *     measured to fit l_j fits anything shorter), and to l_{M-1} when it exceeds all of them;
 *   - neighbouring measured lengths with the same best configuration form one range;
 *   - moving to a longer range takes effect at once; moving to a shorter one only when
 *     x*(1 + hysteresis) also lies in a shorter range, and then only as far down as that inflated
 *     value allows (hysteresis = 0 is the paper's plain rule).
 *
 * All pointers are host pointers; the caller owns every array it passes.  Functions return an
 * earl_status (earl_dispatch.h) and never throw; calls on one selector must come from one thread
 * at a time.
 */
#ifndef EARL_SELECTOR_H_
#define EARL_SELECTOR_H_

#include <stdint.h>

#include "earl_dispatch.h"

#ifdef __cplusplus
extern "C" {
#endif

#define EARL_SELECTOR_MAX_LENGTHS 4096
#define EARL_SELECTOR_MAX_CONFIGS 4096

typedef struct earl_selector earl_selector;

/*
 * Equation 1 of the paper: relative speedup, in percent, of switching from a configuration with
 * throughput tgs_a to one with throughput tgs_b: (tgs_b - tgs_a) / tgs_a * 100.  Positive when b
 * is faster.  No argument checks: the IEEE result for tgs_a == 0 is the caller's.
 */
double earl_speedup_percent(double tgs_a, double tgs_b);

/*
 * Builds the table.
 *   context_lengths[n_lengths]   strictly ascending, >= 1, 1 <= n_lengths <= EARL_SELECTOR_MAX_LENGTHS.
 *   tgs[n_lengths * n_configs]   row-major: tgs[j*n_configs + k] = throughput of configuration k at
 *                                context_lengths[j]; zero, negative, infinite or NaN = failed.
 *   hysteresis                   >= 0, finite.
 *   initial_config               configuration in use before the first observation, in
 *                                [0, n_configs), or -1 for none.
 * EARL_INVALID_ARG for anything else.  A length at which every configuration failed is allowed:
 * its range reports configuration -1.
 */
int32_t earl_selector_build(const int64_t* context_lengths, int32_t n_lengths, int32_t n_configs,
                            const double* tgs, double hysteresis, int32_t initial_config,
                            earl_selector** out);

/* Number of ranges (1 <= n <= n_lengths). */
int32_t earl_selector_n_ranges(const earl_selector* sel, int32_t* out);

/*
 * Range t covers averaged context lengths in (range_hi[t-1], range_hi[t]] (range 0 from 0; the
 * last range has no upper end and reports the largest measured length).  Both arrays have
 * earl_selector_n_ranges entries; either may be NULL.
 */
int32_t earl_selector_get_ranges(const earl_selector* sel, int64_t* range_hi, int32_t* config);

/* Best configuration at measured length j alone, before ranges are merged (-1 = none feasible). */
int32_t earl_selector_best_at(const earl_selector* sel, int32_t j, int32_t* config);

/*
 * One monitoring step before a Rollout stage: the averaged context length of the last step's
 * sequences (> 0, finite).  Writes the configuration to use now and whether it differs from the
 * one in use before the call.  If the range has no feasible configuration the call returns
 * EARL_NO_FEASIBLE_CONFIG, writes -1 and 0, and keeps the state unchanged.
 */
int32_t earl_selector_observe(earl_selector* sel, double avg_context_length, int32_t* config,
                              int32_t* switched);

/* Range the selector is in (-1 before the first observation). */
int32_t earl_selector_current_range(const earl_selector* sel, int32_t* range);

int32_t earl_selector_destroy(earl_selector* sel);

#ifdef __cplusplus
}
#endif
#endif /* EARL_SELECTOR_H_ */

"""CPU oracle for the parallelism-selector table.

TEST INFRASTRUCTURE ONLY: imported by the tests alone; the product path never imports it and it
imports nothing from the product.

What it follows.  Section 2 of the paper ("Parallelism Selector"): throughput is measured at the
start of training for every candidate parallelism configuration at several context lengths, the
best configuration is remembered for every context-length range, the averaged context length is
monitored during training, and the configuration of the range it falls into is switched to
before the next Rollout stage.  Section 3.1 ("Metrics", Equation 1) defines the relative speedup
of one configuration over another from their tokens-per-GPU-per-second (TGS); Section 3.2
reports that a configuration can fail with out-of-memory at a length where another still runs.

The paper states no tie-break, no rule for lengths between two measured ones and no
hysteresis; the rules below are this project's reading (the same sentences as in the library's
header, written out here as plain loops):
  * a measurement that is not a positive finite number is a failed run and is never chosen;
  * best configuration at a measured length = largest TGS, lowest index among equals, -1 if
    every run failed;
  * an averaged length x belongs to the first measured length >= x, to the last one if none;
  * neighbouring measured lengths with the same best configuration are one range;
  * a move to a longer range is immediate; a move to a shorter one goes only as far down as
    the range of x*(1+h) allows (h = 0: no hysteresis).

Pins (tests/test_selector.py): Equation 1 against the percentages the paper's text quotes for
its Figure 3, the switch points the text describes for 32 responses, the out-of-memory case for
128 responses, brute-force checks of the range rule on small tables.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple


def speedup_percent(tgs_a: float, tgs_b: float) -> float:
    """Equation 1: relative speedup in percent of switching from a to b."""
    return (tgs_b - tgs_a) / tgs_a * 100.0


def is_feasible(tgs: float) -> bool:
    return math.isfinite(tgs) and tgs > 0.0


def best_configs(tgs: Sequence[Sequence[float]]) -> List[int]:
    """Per measured length (row of the table): index of the fastest feasible configuration."""
    best = []
    for row in tgs:
        arg, top = -1, 0.0
        for k, v in enumerate(row):
            if is_feasible(v) and (arg < 0 or v > top):
                arg, top = k, v
        best.append(arg)
    return best


def ranges(context_lengths: Sequence[int], tgs: Sequence[Sequence[float]]) -> Tuple[List[int], List[int]]:
    """(range_hi, config): maximal runs of measured lengths with one best configuration."""
    best = best_configs(tgs)
    range_hi: List[int] = []
    config: List[int] = []
    for j, length in enumerate(context_lengths):
        if j > 0 and best[j] == best[j - 1]:
            range_hi[-1] = int(length)
        else:
            range_hi.append(int(length))
            config.append(best[j])
    return range_hi, config


def range_of(range_hi: Sequence[int], x: float) -> int:
    """First range whose upper end is >= x; the last range has no upper end."""
    for t, hi in enumerate(range_hi):
        if x <= hi:
            return t
    return len(range_hi) - 1


class Selector:
    """The online part: one `observe` per training step, before the Rollout stage."""

    def __init__(self, context_lengths: Sequence[int], tgs: Sequence[Sequence[float]],
                 hysteresis: float = 0.0, initial_config: int = -1):
        self.range_hi, self.config = ranges(context_lengths, tgs)
        self.h = float(hysteresis)
        self.current_config = int(initial_config)
        self.current_range = -1

    def observe(self, x: float) -> Tuple[Optional[int], bool]:
        """Returns (configuration to use, whether it differs from the one in use); (None, False)
        and no state change if the range has no feasible configuration."""
        t = range_of(self.range_hi, x)
        if self.current_range >= 0 and t < self.current_range:
            t = min(self.current_range, range_of(self.range_hi, x * (1.0 + self.h)))
        cfg = self.config[t]
        if cfg < 0:
            return None, False
        switched = cfg != self.current_config
        self.current_config, self.current_range = cfg, t
        return cfg, switched

"""Parallelism-selector table (Section 2 "Parallelism Selector", Equation 1): the oracle against
what the paper's text and the mathematics fix, then the C-ABI library against the oracle.  Host
code only: nothing here needs a GPU."""
import json
import math
import os

import numpy as np
import pytest

from oracle import selector_oracle as SO
from paper_2510_05943_amd import binding as B
from paper_2510_05943_amd import selector as S

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def gold():
    with open(os.path.join(GOLD, "selector_section32.json")) as f:
        return json.load(f)


def nan_table(rows):
    return [[float("nan") if v is None else float(v) for v in row] for row in rows]


# ------------------------------------------------------------------ pins of the oracle

def test_equation_1_closed_forms():
    assert SO.speedup_percent(5.0, 5.0) == 0.0
    assert SO.speedup_percent(2.0, 4.0) == 100.0
    assert SO.speedup_percent(4.0, 2.0) == -50.0
    assert SO.speedup_percent(8.0, 9.0) == 12.5
    rng = np.random.default_rng(0)
    for a, b in rng.uniform(0.1, 1e4, size=(200, 2)):
        s_ab, s_ba = SO.speedup_percent(a, b), SO.speedup_percent(b, a)
        # going there and back multiplies the throughput by one
        assert math.isclose((1 + s_ab / 100) * (1 + s_ba / 100), 1.0, rel_tol=1e-12)
        assert (s_ab > 0) == (b > a)


def test_percentages_quoted_in_section_3_2():
    g = gold()
    small, long_ = g["tgs_32_responses"][0], g["tgs_32_responses"][1]
    assert math.isclose(SO.speedup_percent(small[1], small[0]),
                        g["speedup_percent_tp8_to_tp4_small_context"], rel_tol=1e-12)
    assert math.isclose(SO.speedup_percent(long_[0], long_[1]),
                        g["speedup_percent_tp4_to_tp8_long_context"], rel_tol=1e-12)
    # the figure's sign convention: Speedup(4, 8) is negative where TP=4 is the faster one
    assert SO.speedup_percent(small[0], small[1]) < 0 < SO.speedup_percent(long_[0], long_[1])


def test_switch_points_described_in_section_3_2():
    g = gold()
    hi, cfg = SO.ranges(g["context_lengths"], g["tgs_32_responses"])
    assert hi == g["expected_range_hi"] and cfg == g["expected_range_config"]
    sel = SO.Selector(g["context_lengths"], g["tgs_32_responses"], initial_config=0)
    got = [sel.observe(x) for x in g["observed_avg_context"]]
    assert [c for c, _ in got] == g["expected_config"]
    assert [s for _, s in got] == g["expected_switched"]


def test_out_of_memory_configuration_is_never_chosen():
    g = gold()
    table = nan_table(g["tgs_32_responses"][:2] + [g["tgs_128_responses_32k_row"]])
    assert SO.best_configs(table)[2] == g["expected_config_128_responses_32k"]
    # even a much faster measurement elsewhere does not bring the failed one back
    for bad in (float("nan"), 0.0, -3.0, float("inf")):
        assert SO.best_configs([[bad, 1e-9]]) == [1]
    assert SO.best_configs([[float("nan"), 0.0]]) == [-1]
    sel = SO.Selector([100, 200], [[1.0, 2.0], [0.0, float("nan")]], initial_config=1)
    assert sel.observe(50.0) == (1, False)
    assert sel.observe(150.0) == (None, False)
    assert sel.current_range == 0 and sel.current_config == 1


def test_range_rule_against_direct_lookup():
    """For every integer length: the configuration of a fresh selector equals numpy's first
    arg-max of the row of the first measured length that is not shorter (the last row beyond)."""
    rng = np.random.default_rng(1)
    for _ in range(60):
        m, c = int(rng.integers(1, 7)), int(rng.integers(1, 5))
        lengths = np.cumsum(rng.integers(1, 6, size=m))
        table = rng.integers(1, 5, size=(m, c)).astype(float)   # many ties
        hi, cfg = SO.ranges(lengths, table)
        assert hi[-1] == lengths[-1] and all(a != b for a, b in zip(cfg, cfg[1:]))
        for x in range(1, int(lengths[-1]) + 4):
            j = min(int(np.searchsorted(lengths, x, side="left")), m - 1)
            want = int(np.argmax(table[j]))
            assert cfg[SO.range_of(hi, float(x))] == want
            assert SO.Selector(lengths, table).observe(float(x)) == (want, True)
            assert SO.Selector(lengths, table, initial_config=want).observe(float(x)) == (want, False)


def test_hysteresis_hand_worked():
    # ranges: (0,100] -> 0, (100,200] -> 1, (200,inf) -> 2
    lengths, table = [100, 200, 300], [[3, 2, 1], [1, 3, 2], [1, 2, 3]]
    sel = SO.Selector(lengths, table, hysteresis=0.25)
    assert sel.observe(250.0) == (2, True)
    assert sel.observe(190.0) == (2, False)    # 190*1.25 = 237.5 still in the long range
    assert sel.observe(160.0) == (1, True)     # 200 exactly: in the middle range
    assert sel.observe(90.0) == (1, False)     # 112.5: not yet in the short range
    assert sel.observe(80.0) == (0, True)      # 100 exactly
    assert sel.observe(101.0) == (1, True)     # upwards: at once
    assert sel.observe(500.0) == (2, True)
    assert sel.observe(70.0) == (0, True)      # 87.5: two ranges down in one step
    plain = SO.Selector(lengths, table)
    assert [plain.observe(x)[0] for x in (250.0, 190.0, 90.0)] == [2, 1, 0]


MUTANTS = {
    "tie_goes_to_highest_index": ("best_configs", lambda tgs: [
        max((k for k, v in enumerate(r) if SO.is_feasible(v)),
            key=lambda k: (r[k], k), default=-1) for r in tgs]),
    "length_belongs_to_last_measured_below": ("range_of", lambda hi, x: max(
        [t for t, h in enumerate(hi) if (hi[t - 1] if t else 0) <= x] or [0])),
    "failed_runs_compete": ("is_feasible", lambda v: not math.isnan(v)),
}


@pytest.mark.parametrize("mutant", sorted(MUTANTS))
def test_pins_catch_planted_mistake(mutant, monkeypatch):
    name, fn = MUTANTS[mutant]
    monkeypatch.setattr(SO, name, fn)
    failed = 0
    for pin in (test_switch_points_described_in_section_3_2,
                test_out_of_memory_configuration_is_never_chosen,
                test_range_rule_against_direct_lookup, test_hysteresis_hand_worked):
        try:
            pin()
        except AssertionError:
            failed += 1
    assert failed > 0


# ------------------------------------------------------------------ the library against the oracle

def test_header_functions_are_exported():
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "earl_selector.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(earl_[a-z_]+)\s*\(", text)))
    assert set(names) == set(S.EXPORTED)
    lib = B.load_library()
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.earl_status_string(S.EARL_NO_FEASIBLE_CONFIG).decode().startswith("no feasible")


def test_library_speedup_is_bit_equal():
    rng = np.random.default_rng(2)
    for a, b in rng.uniform(1e-3, 1e6, size=(500, 2)):
        assert S.speedup_percent(a, b) == SO.speedup_percent(a, b)


def random_table(rng, m, c):
    table = rng.integers(1, 6, size=(m, c)).astype(float) * rng.choice([1.0, 0.5, 1e3])
    bad = rng.random((m, c)) < 0.25
    table[bad] = rng.choice([float("nan"), 0.0, -1.0, float("inf")], size=int(bad.sum()))
    return table


@pytest.mark.parametrize("seed", range(8))
def test_library_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(40):
        m, c = int(rng.integers(1, 12)), int(rng.integers(1, 6))
        lengths = np.cumsum(rng.integers(1, 2000, size=m))
        table = random_table(rng, m, c)
        h = float(rng.choice([0.0, 0.1, 0.5, 2.0]))
        init = int(rng.integers(-1, c))
        sel = S.selector_build(lengths, table, h, init)
        ref = SO.Selector(lengths, table, h, init)
        assert S.selector_get_ranges(sel) == (ref.range_hi, ref.config)
        assert [S.selector_best_at(sel, j) for j in range(m)] == SO.best_configs(table)
        assert S.selector_current_range(sel) == -1
        for x in rng.uniform(0.5, float(lengths[-1]) * 1.3, size=50):
            x = float(np.round(x)) if rng.random() < 0.3 else float(x)
            want = ref.observe(x)
            if want[0] is None:
                with pytest.raises(B.EarlError) as e:
                    S.selector_observe(sel, x)
                assert e.value.status == S.EARL_NO_FEASIBLE_CONFIG
            else:
                assert S.selector_observe(sel, x) == want
            assert S.selector_current_range(sel) == ref.current_range
        S.selector_destroy(sel)


def test_library_reproduces_section_3_2():
    g = gold()
    sel = S.selector_build(g["context_lengths"], g["tgs_32_responses"], 0.0, 0)
    assert S.selector_get_ranges(sel) == (g["expected_range_hi"], g["expected_range_config"])
    got = [S.selector_observe(sel, x) for x in g["observed_avg_context"]]
    assert [c for c, _ in got] == g["expected_config"]
    assert [s for _, s in got] == g["expected_switched"]
    S.selector_destroy(sel)


def test_library_rejects_bad_arguments():
    ok_l, ok_t = [10, 20], [[1.0, 2.0], [2.0, 1.0]]
    bad = [
        ([], np.zeros((0, 2)), 0.0, -1),
        ([20, 10], ok_t, 0.0, -1),
        ([10, 10], ok_t, 0.0, -1),
        ([0, 10], ok_t, 0.0, -1),
        (ok_l, ok_t, -0.1, -1),
        (ok_l, ok_t, float("nan"), -1),
        (ok_l, ok_t, 0.0, 2),
        (ok_l, ok_t, 0.0, -2),
        (ok_l, np.zeros((2, 0)), 0.0, -1),
    ]
    for lengths, table, h, init in bad:
        with pytest.raises(B.EarlError) as e:
            S.selector_build(lengths, table, h, init)
        assert e.value.status == B.EARL_INVALID_ARG
    sel = S.selector_build(ok_l, ok_t)
    for x in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(B.EarlError) as e:
            S.selector_observe(sel, x)
        assert e.value.status == B.EARL_INVALID_ARG
    with pytest.raises(B.EarlError):
        S.selector_best_at(sel, 2)
    S.selector_destroy(sel)

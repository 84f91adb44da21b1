"""Pins for the CPU oracle (no GPU).

The paper (Section 2, "Data Dispatcher") prints no worked dispatch, so the oracle is pinned
to things other than itself: hand-worked fixtures (tests/golden), closed forms and bounds of
list scheduling, brute force over all assignments on tiny inputs, library routines in special
cases (cumsum, array_split, identity), a checker that reads a result through its own
metadata only (tests/checkers.py), round trips, and structural invariants on all five
workloads.  The last block plants mistakes in the oracle and requires the pins to fail.
"""
import itertools
import json
import os

import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

import checkers
from oracle import earl_oracle as O
from paper_2510_05943_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


def plan_of(w, **over):
    kw = dict(n_groups=w.n_groups, replication=w.replication, seq_group=w.seq_group,
              dp=w.dp, sp=w.sp, zigzag=w.zigzag, pad_multiple=w.pad_multiple,
              mb_token_budget=w.mb_token_budget)
    kw.update(over)
    return O.build_plan(w.lengths, **kw)


def result_of(plan, with_pos=True):
    res = dict(n_seq=plan.n_seq, n_mb=plan.n_mb, seq_ids=plan.seq_ids, rank=plan.rank,
               mb_seq_start=plan.mb_seq_start, mb_row_start=plan.mb_row_start,
               cu_seqlens=plan.cu_seqlens, shard_rows=plan.shard_rows, dst_row=plan.dst_row,
               a2a_counts=plan.a2a_counts, seq_shard=plan.seq_shard)
    if with_pos:
        res["position_ids"] = [O.position_ids_shard(plan, q) for q in range(plan.D * plan.C)]
    return res


def shard_bufs(w, field):
    """Per shard-buffer arrays: every replica of a group holds the group's bytes."""
    groups = [w.group_buffer(field, g) for g in range(w.n_groups)]
    return groups, [groups[s // w.replication] for s in range(w.n_shards)]


# ---------------------------------------------------------------------------------------
# hand-worked fixtures
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["lpt_two_ranks.json", "lpt_ties_three_ranks.json"])
def test_lpt_hand_worked(name):
    g = gold(name)
    rank, load = O.lpt_ranks(g["Lp"], g["D"])
    assert rank.tolist() == g["rank"]
    assert load.tolist() == g["load"]


def test_zigzag_hand_worked_L13():
    g = gold("zigzag_L13.json")
    K, m, Lp, loc = O.padded_geometry([g["L"]], g["C"], g["zigzag"], g["P"])
    assert (K, int(m[0]), int(Lp[0]), int(loc[0])) == (g["K"], g["m"], g["Lp"], g["loc"])
    plan = O.build_plan([g["L"]], n_groups=1, dp=1, sp=g["C"], zigzag=1, pad_multiple=1,
                        mb_token_budget=1 << 20)
    src = [np.arange(100, 100 + g["L"], dtype=np.uint32).reshape(-1, 1)]
    for c in range(g["C"]):
        pos = O.position_ids_shard(plan, c)
        assert pos.tolist() == g["position_ids"][c]
        out = O.dispatch_field_shard(plan, c, src, np.uint32, 1, 7)
        want = [100 + p if real else 7 for p, real in zip(g["position_ids"][c], g["is_real"][c])]
        assert out.ravel().tolist() == want


def test_zigzag_hand_worked_pad64():
    g = gold("zigzag_pad64.json")
    K, m, Lp, loc = O.padded_geometry([g["L"]], g["C"], g["zigzag"], g["P"])
    assert (K, int(m[0]), int(Lp[0]), int(loc[0])) == (g["K"], g["m"], g["Lp"], g["loc"])
    plan = O.build_plan([g["L"]], n_groups=1, dp=1, sp=2, zigzag=1, pad_multiple=64,
                        mb_token_budget=1 << 20)
    for c in range(2):
        pos = O.position_ids_shard(plan, c)
        assert [int(pos[0]), int(pos[64])] == g["first_position_of_each_local_half"][c]
        assert int(plan.a2a_counts[:, c].sum()) == g["real_rows_per_sp_rank"][c]


def test_next_fit_hand_worked():
    g = gold("next_fit.json")
    plan = O.build_plan(g["Lp"], n_groups=1, dp=1, sp=1, zigzag=0, pad_multiple=1,
                        mb_token_budget=g["B"])
    assert plan.mb.tolist() == g["mb"]
    assert plan.mb_seq_start.tolist() == g["mb_seq_start"]
    assert plan.mb_row_start.tolist() == g["mb_row_start"]
    assert plan.cu_seqlens.tolist() == g["cu_seqlens"]


def test_quadratic_lpt_hand_worked():
    g = gold("lpt_quadratic_two_ranks.json")
    rank, load = O.lpt_ranks(g["Lp"], g["D"])
    assert rank.tolist() == g["rank_linear"] and load.tolist() == g["load_linear"]
    rank, load = O.lpt_ranks(g["Lp"], g["D"], quadratic=True)
    assert rank.tolist() == g["rank_quadratic"] and load.tolist() == g["load_quadratic"]
    plan = O.build_plan(g["Lp"], n_groups=1, dp=g["D"], sp=1, zigzag=0, pad_multiple=1,
                        mb_token_budget=1 << 20, balance_policy=2)
    assert plan.rank.tolist() == g["rank_quadratic"]
    assert plan.rank_load.tolist() == g["token_load_quadratic"]   # reported in tokens


def test_equal_mb_hand_worked():
    g = gold("equal_mb_two_ranks.json")
    for key, flag in (("plain", 0), ("equal", 1)):
        plan = O.build_plan(g["L"], n_groups=1, dp=g["D"], sp=1, zigzag=0, pad_multiple=1,
                            mb_token_budget=g["B"], equal_mb=flag)
        assert plan.rank.tolist() == g["rank"] and plan.mb.tolist() == g["mb"]
        for name, want in g[key].items():
            assert getattr(plan, name).tolist() == want, (key, name)


def test_replica_choice_hand_worked():
    g = gold("replica_choice.json")
    _, seq_shard, seq_row, _, seq_k = O.source_layout([3] * g["N"], g["G"], g["R"])
    assert seq_k.tolist() == [0, 1, 2, 3, 4, 0, 1, 2, 3, 4]
    assert seq_shard.tolist() == g["seq_shard"]
    assert seq_row.tolist() == [0, 3, 6, 9, 12, 0, 3, 6, 9, 12]


# ---------------------------------------------------------------------------------------
# list-scheduling bounds and brute-force optimum
# ---------------------------------------------------------------------------------------
def test_lpt_against_brute_force_optimum():
    rng = np.random.default_rng(5)
    for trial in range(60):
        D = int(rng.integers(2, 4))
        N = int(rng.integers(1, 9))
        Lp = rng.integers(1, 40, size=N).tolist()
        rank, load = O.lpt_ranks(Lp, D)
        best = min(max(sum(Lp[i] for i in range(N) if a[i] == d) for d in range(D))
                   for a in itertools.product(range(D), repeat=N))
        assert load.max() * 3 * D <= (4 * D - 1) * best, (Lp, D)
        assert load.tolist() == [sum(Lp[i] for i in range(N) if rank[i] == d) for d in range(D)]
        if N >= D:
            assert load.max() - load.min() <= max(Lp)
        assert load.max() <= sum(Lp) / D + (1 - 1 / D) * max(Lp) + 1e-9


def test_quadratic_lpt_against_brute_force_optimum():
    """The same list-scheduling guarantees, on the squared lengths."""
    rng = np.random.default_rng(6)
    for trial in range(60):
        D = int(rng.integers(2, 4))
        N = int(rng.integers(1, 9))
        Lp = rng.integers(1, 40, size=N).tolist()
        cost = [x * x for x in Lp]
        rank, load = O.lpt_ranks(Lp, D, quadratic=True)
        best = min(max(sum(cost[i] for i in range(N) if a[i] == d) for d in range(D))
                   for a in itertools.product(range(D), repeat=N))
        assert max(load) * 3 * D <= (4 * D - 1) * best, (Lp, D)
        assert load.tolist() == [sum(cost[i] for i in range(N) if rank[i] == d) for d in range(D)]
        if N >= D:
            assert max(load) - min(load) <= max(cost)
    # equal lengths: both costs give the round-robin deal
    assert O.lpt_ranks([9] * 12, 4, quadratic=True)[0].tolist() == [i % 4 for i in range(12)]
    # squares are exact beyond 2^53 (no floating point on the way)
    big = [(1 << 21) - k for k in range(6)]
    _, load = O.lpt_ranks(big, 2, quadratic=True)
    assert sum(load) == sum(x * x for x in big)


def test_equal_mb_only_appends_empty_micro_batches():
    rng = np.random.default_rng(7)
    for trial in range(40):
        N, D, C = int(rng.integers(1, 40)), int(rng.integers(1, 7)), int(rng.integers(1, 4))
        L = rng.integers(1, 300, size=N)
        kw = dict(n_groups=1, dp=D, sp=C, zigzag=int(rng.integers(0, 2)), pad_multiple=1,
                  mb_token_budget=int(rng.integers(700, 1500)),
                  balance_policy=int(rng.integers(0, 3)))
        a, b = O.build_plan(L, **kw), O.build_plan(L, equal_mb=1, **kw)
        for name in ("rank", "slot", "mb", "dst_row", "seq_ids", "shard_rows", "n_seq",
                     "seg_dst_row", "seg_src_row", "seg_n_real", "a2a_counts"):
            assert np.array_equal(getattr(a, name), getattr(b, name)), name
        most = int(a.n_mb.max())
        assert b.n_mb.tolist() == [most] * D
        pa = pb = ca = cb = 0
        for r in range(D):
            na, extra = int(a.n_mb[r]), most - int(a.n_mb[r])
            assert b.mb_seq_start[pb:pb + na + 1].tolist() == a.mb_seq_start[pa:pa + na + 1].tolist()
            assert b.mb_row_start[pb:pb + na + 1].tolist() == a.mb_row_start[pa:pa + na + 1].tolist()
            assert b.mb_seq_start[pb + na + 1:pb + most + 1].tolist() == [int(a.n_seq[r])] * extra
            assert b.mb_row_start[pb + na + 1:pb + most + 1].tolist() == \
                [int(a.shard_rows[r * C])] * extra
            la = int(a.n_seq[r]) + na
            assert b.cu_seqlens[cb:cb + la].tolist() == a.cu_seqlens[ca:ca + la].tolist()
            assert b.cu_seqlens[cb + la:cb + la + extra].tolist() == [0] * extra
            pa, pb, ca, cb = pa + na + 1, pb + most + 1, ca + la, cb + la + extra
        assert pb == len(b.mb_seq_start) and cb == len(b.cu_seqlens)


def test_lpt_equal_lengths_is_round_robin():
    for D in (1, 2, 3, 8):
        N = 6 * D
        rank, load = O.lpt_ranks([17] * N, D)
        assert rank.tolist() == [i % D for i in range(N)]
        assert len(set(load.tolist())) == 1


def test_snake_hand_worked_and_bounds():
    g = gold("snake_three_ranks.json")
    rank, load = O.snake_ranks(g["Lp"], g["D"])
    assert rank.tolist() == g["rank"] and load.tolist() == g["load"]
    rng = np.random.default_rng(8)
    for trial in range(200):
        D = int(rng.integers(1, 9))
        N = int(rng.integers(1, 60))
        Lp = rng.integers(1, 1000, size=N)
        rank, load = O.snake_ranks(Lp, D)
        counts = np.bincount(rank, minlength=D)
        assert counts.max() - counts.min() <= 1          # a deal: equal counts up to one
        assert load.tolist() == [int(Lp[rank == d].sum()) for d in range(D)]
        if N >= D:
            assert load.max() - load.min() <= Lp.max()   # round ranges telescope
    # equal lengths: boustrophedon over the index
    rank, _ = O.snake_ranks([5] * 8, 3)
    assert rank.tolist() == [0, 1, 2, 2, 1, 0, 0, 1]


def test_per_sequence_field_equals_the_repeated_per_token_field():
    """Broadcasting one row per sequence must equal dispatching the field after numpy.repeat has
    expanded it to one row per token."""
    for case in small_cases()[:12]:
        f = synth.per_sequence_field("adv", 4)
        w = synth.custom_workload(case["L"], n_groups=case["G"], replication=case["R"],
                                  seq_group=case["grp"], dp=case["D"], sp=case["C"], zigzag=case["z"],
                                  pad_multiple=case["P"], mb_token_budget=case["B"], fields=(f,),
                                  seed=case["seed"])
        plan = plan_of(w)
        per_seq = [w.group_buffer(f, s // w.replication) for s in range(w.n_shards)]
        per_tok = []
        for s in range(w.n_shards):
            members = w.group_members(s // w.replication)
            assert per_seq[s].shape[0] == len(members)
            per_tok.append(np.repeat(per_seq[s], w.lengths[members], axis=0))
        a = O.dispatch_field(plan, per_seq, f.np_dtype, 1, 0x7F, per_sequence=True)
        b = O.dispatch_field(plan, per_tok, f.np_dtype, 1, 0x7F)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_nonzero_counts_against_the_dispatched_field():
    """Two other routes to the same numbers: a plain count on the zero-padded dispatched shard,
    micro-batch by micro-batch; and the sum over everything equals the non-zeros of the source
    (every real token lands on exactly one shard and micro-batch)."""
    rng = np.random.default_rng(11)
    for trial in range(25):
        N, D, C = int(rng.integers(1, 30)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        L = rng.integers(1, 200, size=N)
        G, R = int(rng.integers(1, 4)), int(rng.integers(1, 3))
        plan = O.build_plan(L, n_groups=G, replication=R, dp=D, sp=C, zigzag=int(rng.integers(0, 2)),
                            pad_multiple=int(rng.choice([1, 8])),
                            mb_token_budget=int(rng.integers(700, 2000)),
                            equal_mb=int(rng.integers(0, 2)))
        width = int(rng.choice([1, 1, 3]))
        # one buffer per group, identical over its replicas; sequences packed in index order
        grp = (np.arange(N) * G) // N
        bufs = []
        for g in range(G):
            rows = int(L[grp == g].sum())
            buf = (rng.random((rows, width)) < 0.6).astype(np.uint8) * rng.integers(1, 255)
            bufs.extend([buf.astype(np.uint8)] * R)
        got = O.nonzero_counts(plan, bufs, width)
        assert got.shape == (D * C, int(plan.n_mb.max()))
        total = 0
        tbl = 0
        for r in range(D):
            nmb = int(plan.n_mb[r])
            starts = plan.mb_row_start[tbl:tbl + nmb + 1]
            tbl += nmb + 1
            for c in range(C):
                q = r * C + c
                # padded with zeros, the padding rows add nothing to a plain count of the shard
                out = O.dispatch_field_shard(plan, q, bufs, np.uint8, width, 0)
                for b in range(nmb):
                    lo, hi = int(starts[b]), int(starts[b + 1])
                    want = int(np.count_nonzero(out[lo:hi]))
                    assert got[q, b] == want, (trial, q, b)
                    total += want
                assert not got[q, nmb:].any()
        assert total == int(got.sum()) == sum(int(np.count_nonzero(bufs[g * R])) for g in range(G))


def test_nonzero_counts_hand_worked():
    # one rank, two SP ranks (contiguous halves), B=8: sequences of 4 and 4 fill micro-batch 0,
    # the sequence of 6 is micro-batch 1.  mask rows: seq0 = 1,1,0,1  seq1 = 0,0,0,1  seq2 = 1,0,1,1,1,0
    L = [4, 4, 6]
    mask = np.array([1, 1, 0, 1, 0, 0, 0, 1, 1, 0, 1, 1, 1, 0], np.uint8).reshape(-1, 1)
    plan = O.build_plan(L, n_groups=1, dp=1, sp=2, zigzag=0, pad_multiple=1, mb_token_budget=8)
    assert plan.mb.tolist() == [0, 0, 1]
    # SP rank 0 holds the first halves: (1,1),(0,0) | (1,0,1); SP rank 1 the second: (0,1),(0,1) | (1,1,0)
    assert O.nonzero_counts(plan, [mask]).tolist() == [[2, 2], [2, 2]]
    mask[4] = 7   # any non-zero value counts once
    assert O.nonzero_counts(plan, [mask]).tolist() == [[3, 2], [2, 2]]


def test_two_pass_gather_then_scatter_equals_direct_dispatch():
    """The single-controller pattern of Section 1 (everything gathered in one place, then
    redistributed) must produce the same training layout as the direct dispatch."""
    w = synth.make_workload("mid", seed=4, scale=0.0625)
    direct = plan_of(w)
    gather = O.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                          seq_group=w.seq_group, dp=1, sp=1, zigzag=0, pad_multiple=1,
                          mb_token_budget=1 << 40)
    scatter = O.build_plan(w.lengths, n_groups=1, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                           pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget)
    for f in w.fields:
        _, bufs = shard_bufs(w, f)
        one = O.dispatch_field(gather, bufs, f.np_dtype, f.width, f.pad_scalar)
        assert len(one) == 1 and one[0].shape[0] == w.total_tokens
        two = O.dispatch_field(scatter, one, f.np_dtype, f.width, f.pad_scalar)
        want = O.dispatch_field(direct, bufs, f.np_dtype, f.width, f.pad_scalar)
        assert all(np.array_equal(a, b) for a, b in zip(two, want))
    assert O.algorithmic_bytes(gather, [4], False) + O.algorithmic_bytes(scatter, [4], False) \
        > 1.9 * O.algorithmic_bytes(direct, [4], False)


def test_lpt_fewer_sequences_than_ranks():
    plan = O.build_plan([5, 9, 2], n_groups=1, dp=5, sp=2, zigzag=1, pad_multiple=1,
                        mb_token_budget=100)
    assert plan.rank.tolist() == [1, 0, 2]          # longest first onto the lowest empty rank
    assert plan.n_seq.tolist() == [1, 1, 1, 0, 0]
    assert plan.n_mb.tolist() == [1, 1, 1, 0, 0]
    assert plan.shard_rows.tolist() == [6, 6, 4, 4, 2, 2, 0, 0, 0, 0]
    assert plan.mb_seq_start.tolist() == [0, 1, 0, 1, 0, 1, 0, 0]


# ---------------------------------------------------------------------------------------
# special cases that reduce to library routines
# ---------------------------------------------------------------------------------------
def test_trivial_layout_is_identity():
    w = synth.custom_workload(np.random.default_rng(1).integers(1, 50, size=23))
    plan = plan_of(w)
    L = w.lengths.astype(np.int64)
    assert plan.cu_seqlens.tolist() == [0] + np.cumsum(L).tolist()
    assert O.position_ids_shard(plan, 0).tolist() == np.concatenate([np.arange(x) for x in L]).tolist()
    for f in w.fields:
        _, bufs = shard_bufs(w, f)
        out = O.dispatch_field_shard(plan, 0, bufs, f.np_dtype, f.width, 0)
        assert np.array_equal(out, bufs[0])
    assert plan.seq_row.tolist() == (np.cumsum(L) - L).tolist()


def test_contiguous_split_is_array_split():
    C = 4
    L = [8, 12, 4, 40]
    w = synth.custom_workload(L, sp=C)
    plan = plan_of(w)
    f = w.fields[0]
    _, bufs = shard_bufs(w, f)
    seqs = np.split(bufs[0], np.cumsum(L)[:-1])
    for c in range(C):
        want = np.concatenate([np.array_split(s, C)[c] for s in seqs])
        assert np.array_equal(O.dispatch_field_shard(plan, c, bufs, f.np_dtype, 1, 0), want)


def test_source_offsets_are_per_group_cumsum():
    rng = np.random.default_rng(3)
    L = rng.integers(1, 30, size=40)
    grp = rng.integers(0, 5, size=40)
    _, seq_shard, seq_row, group_rows, seq_k = O.source_layout(L, 5, 1, seq_group=grp)
    assert seq_k.tolist() == [int((grp[:i] == grp[i]).sum()) for i in range(40)]
    assert seq_row.tolist() == checkers.packed_source_rows(L, grp, 5).tolist()
    assert seq_shard.tolist() == grp.tolist()
    assert group_rows.tolist() == [int(L[grp == g].sum()) for g in range(5)]


# ---------------------------------------------------------------------------------------
# self-describing output, conservation, round trip on small random batches
# ---------------------------------------------------------------------------------------
def small_cases():
    rng = np.random.default_rng(11)
    cases = []
    for t in range(24):
        N = int(rng.integers(1, 14))
        G = int(rng.integers(1, 4))
        R = int(rng.choice([1, 1, 2, 4]))
        D = int(rng.integers(1, 4))
        C = int(rng.choice([1, 2, 3, 4]))
        z = int(rng.integers(0, 2))
        P = int(rng.choice([1, 1, 2, 8]))
        L = rng.integers(1, 60, size=N)
        K = 2 * C if (z and C > 1) else C
        worst = K * P * (-(-(-(-int(L.max()) // K)) // P))
        B = int(worst + rng.integers(0, 3 * worst))
        grp = rng.integers(0, G, size=N) if t % 2 else None
        cases.append(dict(L=L, G=G, R=R, D=D, C=C, z=z, P=P, B=B, grp=grp, seed=t))
    return cases


def all_pins_on_small_case(case, oracle=O):
    fields = (synth.F_ID, synth.F_MASK, synth.bytes_field("wide", 2, 24, 0xBEEF),
              synth.bytes_field("odd", 4, 3, 0x01020304))
    w = synth.custom_workload(case["L"], n_groups=case["G"], replication=case["R"],
                              seq_group=case["grp"], dp=case["D"], sp=case["C"], zigzag=case["z"],
                              pad_multiple=case["P"], mb_token_budget=case["B"], fields=fields,
                              seed=case["seed"])
    plan = oracle.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                             seq_group=w.seq_group, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                             pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget)
    res = dict(n_seq=plan.n_seq, n_mb=plan.n_mb, seq_ids=plan.seq_ids, rank=plan.rank,
               mb_seq_start=plan.mb_seq_start, mb_row_start=plan.mb_row_start,
               cu_seqlens=plan.cu_seqlens, shard_rows=plan.shard_rows, dst_row=plan.dst_row,
               a2a_counts=plan.a2a_counts, seq_shard=plan.seq_shard,
               position_ids=[oracle.position_ids_shard(plan, q) for q in range(w.dp * w.sp)])
    checkers.check_structure(res, w.lengths, w.dp, w.sp, plan.K, w.pad_multiple, w.mb_token_budget)
    src_row = checkers.packed_source_rows(w.lengths, w.seq_group, w.n_groups)
    for f in fields:
        groups, bufs = shard_bufs(w, f)
        dst = oracle.dispatch_field(plan, bufs, f.np_dtype, f.width, f.pad_scalar)
        pad = np.full((f.width,), f.pad_scalar & ((1 << (8 * f.scalar_bytes)) - 1), f.np_dtype)
        checkers.check_self_describing(res, w.lengths, w.dp, w.sp, groups, w.seq_group, src_row,
                                       dst, pad)
        # replica choice: each shard buffer may hold garbage outside the rows read from it
        poisoned = [np.full_like(b, 0xA5) for b in bufs]
        for i in range(w.n_seqs):
            s, r0, n = int(plan.seq_shard[i]), int(plan.seq_row[i]), int(w.lengths[i])
            poisoned[s][r0:r0 + n] = bufs[s][r0:r0 + n]
        dst2 = oracle.dispatch_field(plan, poisoned, f.np_dtype, f.width, f.pad_scalar)
        assert all(np.array_equal(a, b) for a, b in zip(dst, dst2))
        # round trip
        back = [np.full_like(b, 0x5A) for b in bufs]
        oracle.inverse_field(plan, dst, back)
        for s in range(w.n_shards):
            read = _read_rows(plan, s, back[s].shape[0])
            assert np.array_equal(back[s][read], bufs[s][read])
            assert np.all(back[s][~read] == 0x5A)
    # the row map on its own: gathering source rows through it (padding where it says -1) gives
    # the dispatched shard of every field, and it says -1 exactly on the padding rows (which the
    # trace-back above has located from the metadata alone)
    for q in range(w.dp * w.sp):
        sh, row = oracle.source_row_map_shard(plan, q)
        assert sh.shape == row.shape == (int(plan.shard_rows[q]),)
        assert np.array_equal(sh < 0, row < 0)
        assert np.array_equal(sh < 0, checkers.padding_rows_of_shard(res, w.lengths, w.dp, w.sp, q))
        for f in fields:
            _, bufs = shard_bufs(w, f)
            want = oracle.dispatch_field_shard(plan, q, bufs, f.np_dtype, f.width, f.pad_scalar)
            got = np.empty_like(want)
            got[:] = np.full((f.width,), f.pad_scalar & ((1 << (8 * f.scalar_bytes)) - 1), f.np_dtype)
            for d in np.flatnonzero(sh >= 0):
                got[d] = bufs[int(sh[d])][int(row[d])]
            assert np.array_equal(got, want)
    # segment table agrees with the per-row definition
    for q in range(w.dp * w.sp):
        sh, row = oracle.source_row_map_shard(plan, q)
        e0, e1 = int(plan.shard_seg_start[q]), int(plan.shard_seg_start[q + 1])
        cover = np.zeros(len(sh), np.int32)
        for e in range(e0, e1):
            d0, n, nr = int(plan.seg_dst_row[e]), int(plan.seg_n_rows[e]), int(plan.seg_n_real[e])
            assert int(plan.seg_dst_shard[e]) == q
            cover[d0:d0 + n] += 1
            assert np.all(sh[d0:d0 + nr] == plan.seg_src_shard[e]) and np.all(sh[d0 + nr:d0 + n] == -1)
            assert row[d0:d0 + nr].tolist() == list(range(int(plan.seg_src_row[e]),
                                                           int(plan.seg_src_row[e]) + nr))
            assert res["position_ids"][q][d0:d0 + n].tolist() == list(
                range(int(plan.seg_pos0[e]), int(plan.seg_pos0[e]) + n))
            if e > e0:
                assert plan.seg_dst_row[e] == plan.seg_dst_row[e - 1] + plan.seg_n_rows[e - 1]
        assert np.all(cover == 1)
    return plan


def _read_rows(plan, s, rows):
    sel = np.zeros(rows, bool)
    for i in range(plan.N):
        if int(plan.seq_shard[i]) == s:
            sel[int(plan.seq_row[i]): int(plan.seq_row[i]) + int(plan.L[i])] = True
    return sel


@settings(max_examples=120, deadline=None, derandomize=True,
          suppress_health_check=[HealthCheck.too_slow, HealthCheck.data_too_large])
@given(st.data())
def test_all_pins_on_drawn_batches(data):
    """The same pins on batches drawn by hypothesis (fixed seed): layouts with more ranks than
    sequences, single-row sequences, budgets that fit exactly one sequence, scattered groups."""
    n = data.draw(st.integers(1, 18), label="N")
    C = data.draw(st.sampled_from([1, 2, 3, 4, 5]), label="C")
    z = data.draw(st.integers(0, 1), label="zigzag")
    P = data.draw(st.sampled_from([1, 1, 2, 3, 8]), label="P")
    L = np.array(data.draw(st.lists(st.integers(1, 70), min_size=n, max_size=n), label="L"))
    G = data.draw(st.integers(1, 4), label="G")
    K = 2 * C if (z and C > 1) else C
    worst = K * P * (-(-(-(-int(L.max()) // K)) // P))
    case = dict(L=L, G=G, R=data.draw(st.sampled_from([1, 2, 3]), label="R"),
                D=data.draw(st.integers(1, 6), label="D"), C=C, z=z, P=P,
                B=worst + data.draw(st.integers(0, 3 * worst), label="extra budget"),
                grp=(np.array(data.draw(st.lists(st.integers(0, G - 1), min_size=n, max_size=n),
                                        label="groups")) if data.draw(st.booleans()) else None),
                seed=data.draw(st.integers(0, 1000), label="seed"))
    all_pins_on_small_case(case)


@pytest.mark.parametrize("case", small_cases(), ids=lambda c: f"case{c['seed']}")
def test_small_batches_all_pins(case):
    all_pins_on_small_case(case)


# ---------------------------------------------------------------------------------------
# the five workloads: structure, conservation, byte accounting
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", synth.CONFIG_NAMES)
def test_workload_plan_structure(name):
    w = synth.make_workload(name, seed=0)
    plan = plan_of(w)
    res = result_of(plan)
    checkers.check_structure(res, w.lengths, w.dp, w.sp, plan.K, w.pad_multiple, w.mb_token_budget)
    assert plan.total_dst_rows == int(plan.Lp.sum())
    assert int(plan.rank_load.sum()) == int(plan.Lp.sum())


@pytest.mark.parametrize("name", ["tiny", "mid", "agentic"])
def test_workload_fields_trace_back(name):
    w = synth.make_workload(name, seed=1, scale=0.25 if name != "tiny" else 1.0)
    plan = plan_of(w)
    res = result_of(plan)
    src_row = checkers.packed_source_rows(w.lengths, w.seq_group, w.n_groups)
    assert plan.seq_row.tolist() == src_row.tolist()
    for f in w.fields:
        groups, bufs = shard_bufs(w, f)
        dst = O.dispatch_field(plan, bufs, f.np_dtype, f.width, f.pad_scalar)
        checkers.check_self_describing_fast(res, w.lengths, w.dp, w.sp, groups, w.seq_group,
                                            src_row, dst, np.zeros((f.width,), f.np_dtype))


def test_agentic_replicas_each_serve_one_quarter():
    w = synth.make_workload("agentic", seed=0)
    plan = plan_of(w)
    for g in range(w.n_groups):
        members = np.nonzero(w.seq_group == g)[0]
        counts = np.bincount(plan.seq_shard[members] - g * w.replication, minlength=w.replication)
        assert counts.tolist() == [len(members) // w.replication] * w.replication
        assert np.all(np.diff(plan.seq_shard[members]) >= 0)


def test_byte_accounting_is_linear_in_tokens():
    """Table 1 of the paper: the batch volume doubles with every doubling of the context."""
    base = np.array([64, 128, 256, 512] * 4)
    row_bytes = [4, 1, 4, 4]
    sizes = []
    for mult in (1, 2, 4, 8):
        plan = O.build_plan(base * mult, n_groups=2, dp=2, sp=2, zigzag=1, pad_multiple=1,
                            mb_token_budget=1 << 30)
        sizes.append(O.algorithmic_bytes(plan, row_bytes))
    assert sizes[1] == 2 * sizes[0] and sizes[2] == 4 * sizes[0] and sizes[3] == 8 * sizes[0]
    assert sizes[0] == 13 * int(base.sum()) * 2 + 4 * int(base.sum())


def test_batch_volume_matches_the_papers_table():
    """Table 1 of the paper prints the batch volume for six context lengths.  The rows that
    leave the source workers (all-to-all counts), times the bytes per token, must give those
    sizes exactly: every real token counted once, whatever the replication of the sources and
    the padding of the destination."""
    g = gold("table1_batch_size.json")
    n, bpt = g["n_seqs"], g["bytes_per_token"]
    for ctx, mib in zip(g["context_length"], g["estimated_size_MiB"]):
        lengths = np.full((n,), ctx, dtype=np.int64)
        for n_groups, repl, sp, pad in ((8, 1, 1, 1), (2, 4, 4, 64), (1, 8, 3, 7)):
            plan = O.build_plan(lengths, n_groups=n_groups, replication=repl, dp=4, sp=sp, zigzag=1,
                                pad_multiple=pad, mb_token_budget=1 << 40)
            sent = int(plan.a2a_counts.sum()) * bpt
            assert sent == mib * (1 << 20)
            assert plan.total_real_rows * bpt == mib * (1 << 20)
            # the bytes one dispatch moves: that volume read once, and the padded layout written
            assert O.algorithmic_bytes(plan, [bpt], with_position_ids=False) == \
                sent + plan.total_dst_rows * bpt


def test_payload_per_worker_matches_section_3_3():
    """The three per-worker payloads Section 3.3 prints for its log-probability tensors: the rows
    one source worker sends (its row of the all-to-all counts) times 4 bytes, truncated to MiB."""
    g = gold("section33_payload_per_worker.json")
    lo, hi = g["n_range_that_reproduces_all_three"]
    for n in (lo - 1, lo, g["n_seqs_per_worker"], hi, hi + 1):
        got = []
        for ctx in g["context_length"]:
            # two source workers of n sequences each, consumers in a DP4 x SP2 layout
            plan = O.build_plan(np.full((2 * n,), ctx), n_groups=2, dp=4, sp=2, zigzag=1,
                                pad_multiple=1, mb_token_budget=1 << 40)
            sent = plan.a2a_counts.sum(axis=1) * g["bytes_per_token"]
            assert sent[0] == sent[1]
            got.append(int(sent[0]) >> 20)
        assert (got == g["payload_MiB_truncated"]) == (lo <= n <= hi), (n, got)


def test_plan_ignores_field_contents_and_is_deterministic():
    w = synth.make_workload("mid", seed=2, scale=0.125)
    a, b = plan_of(w), plan_of(w)
    for k, v in a.__dict__.items():
        assert np.array_equal(v, b.__dict__[k]), k


def test_errors():
    with pytest.raises(O.OracleError) as e:
        O.build_plan([10, 200], n_groups=1, dp=1, sp=2, zigzag=1, pad_multiple=1, mb_token_budget=199)
    assert e.value.status == O.SEQ_EXCEEDS_BUDGET
    for bad in (dict(L=[0, 3]), dict(L=[]), dict(dp=0), dict(sp=0), dict(pad_multiple=0),
                dict(seq_group=[0, 5])):
        kw = dict(L=[4, 4], n_groups=2, dp=1, sp=1, zigzag=0, pad_multiple=1, mb_token_budget=100)
        kw.update(bad)
        L = kw.pop("L")
        with pytest.raises(O.OracleError) as e:
            O.build_plan(L, **kw)
        assert e.value.status == O.INVALID_ARG


# ---------------------------------------------------------------------------------------
# planted mistakes: the pins above must notice each of them
# ---------------------------------------------------------------------------------------
def _mut_zigzag_not_mirrored(monkeypatch):
    monkeypatch.setattr(O, "chunk_to_sp", lambda k, C, K: (k, 0) if K == C else (k % C, k // C))


def _mut_lpt_tie_to_higher_rank(monkeypatch):
    def bad(Lp, D, quadratic=False):
        order = sorted(range(len(Lp)), key=lambda i: (-int(Lp[i]), i))
        load, rank = [0] * D, [0] * len(Lp)
        for i in order:
            r = min(range(D), key=lambda d: (load[d], -d))
            rank[i] = r
            load[r] += int(Lp[i])
        return np.array(rank, np.int32), np.array(load, np.int64)
    monkeypatch.setattr(O, "lpt_ranks", bad)


def _mut_lpt_shortest_first(monkeypatch):
    def bad(Lp, D, quadratic=False):
        order = sorted(range(len(Lp)), key=lambda i: (int(Lp[i]), i))
        load, rank = [0] * D, [0] * len(Lp)
        for i in order:
            r = min(range(D), key=lambda d: (load[d], d))
            rank[i] = r
            load[r] += int(Lp[i])
        return np.array(rank, np.int32), np.array(load, np.int64)
    monkeypatch.setattr(O, "lpt_ranks", bad)


def _mut_pad_ignores_multiple(monkeypatch):
    real = O.padded_geometry
    monkeypatch.setattr(O, "padded_geometry", lambda L, C, z, P: real(L, C, z, 1))


def _mut_budget_strict(monkeypatch):
    real = O.pack_ranks
    monkeypatch.setattr(O, "pack_ranks",
                        lambda rank, Lp, loc, D, B, **kw: real(rank, Lp, loc, D, B - 1, **kw))


def _mut_positions_restart_per_chunk(monkeypatch):
    real = O.position_ids_shard

    def bad(plan, q):
        out = real(plan, q)
        return (out % np.maximum(1, np.int32(plan.m.max()))).astype(np.int32)
    monkeypatch.setattr(O, "position_ids_shard", bad)


def _mut_replica_always_zero(monkeypatch):
    real = O.source_layout

    def bad(L, G, R, seq_group=None, seq_row=None):
        grp, shard, row, rows, k = real(L, G, R, seq_group, seq_row)
        return grp, (grp * R).astype(np.int32), row, rows, k
    monkeypatch.setattr(O, "source_layout", bad)


def _mut_quadratic_cost_is_linear(monkeypatch):
    real = O.lpt_ranks
    monkeypatch.setattr(O, "lpt_ranks", lambda Lp, D, quadratic=False: real(Lp, D))


def _mut_equal_mb_pads_to_most_plus_one(monkeypatch):
    real = O.pack_ranks

    def bad(rank, Lp, loc, D, B, equal_mb=False):
        pk = real(rank, Lp, loc, D, B, equal_mb=equal_mb)
        if equal_mb:
            for r in range(D):
                pk["n_mb"][r] += 1
                pk["mb_seq_start"][r].append(pk["mb_seq_start"][r][-1])
                pk["mb_row_start"][r].append(pk["mb_row_start"][r][-1])
        return pk
    monkeypatch.setattr(O, "pack_ranks", bad)


def _mut_row_map_forgets_chunk_offset(monkeypatch):
    real = O.source_row_map_shard

    def bad(plan, q):
        # every chunk starts at the sequence's first source row (the chunk's logical offset dropped)
        sh, row = real(plan, q)
        pos = O.position_ids_shard(plan, q).astype(np.int64)
        m_of_row = np.zeros_like(row)
        r = q // plan.C
        first = int(np.sum(plan.n_seq[:r]))
        for i in plan.seq_ids[first:first + int(plan.n_seq[r])]:
            d0, n = int(plan.dst_row[int(i)]), int(plan.loc[int(i)])
            m_of_row[d0:d0 + n] = int(plan.m[int(i)])
        return sh, np.where(row >= 0, row - (pos // np.maximum(m_of_row, 1)) * m_of_row, row)
    monkeypatch.setattr(O, "source_row_map_shard", bad)


def _mut_row_map_marks_no_padding(monkeypatch):
    real = O.source_row_map_shard

    def bad(plan, q):
        sh, row = real(plan, q)
        return np.where(sh < 0, 0, sh).astype(np.int32), np.where(row < 0, 0, row)
    monkeypatch.setattr(O, "source_row_map_shard", bad)


MUTANTS = [_mut_row_map_forgets_chunk_offset, _mut_row_map_marks_no_padding,
           _mut_quadratic_cost_is_linear, _mut_equal_mb_pads_to_most_plus_one,
           _mut_zigzag_not_mirrored, _mut_lpt_tie_to_higher_rank, _mut_lpt_shortest_first,
           _mut_pad_ignores_multiple, _mut_budget_strict, _mut_positions_restart_per_chunk,
           _mut_replica_always_zero]


def _run_fixture_pins():
    test_lpt_hand_worked("lpt_two_ranks.json")
    test_lpt_hand_worked("lpt_ties_three_ranks.json")
    test_zigzag_hand_worked_L13()
    test_zigzag_hand_worked_pad64()
    test_next_fit_hand_worked()
    test_replica_choice_hand_worked()
    test_quadratic_lpt_hand_worked()
    test_equal_mb_hand_worked()
    test_lpt_against_brute_force_optimum()
    test_lpt_equal_lengths_is_round_robin()
    for case in small_cases():
        all_pins_on_small_case(case)


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda m: m.__name__)
def test_pins_catch_planted_mistake(mutant, monkeypatch):
    mutant(monkeypatch)
    with pytest.raises(AssertionError):
        _run_fixture_pins()

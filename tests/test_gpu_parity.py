"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit.

Everything here is integer or byte work, so the bar is exact equality on every output: plan
arrays, segment table, all-to-all counts, every destination shard of every field, position ids
and cu_seqlens.  Sizes span several 64 KiB tiles per shard and ragged tails; edge cases cover
empty ranks, single-row sequences, odd row widths, explicit source offsets, replicated
sources, large label counts and the error paths.
"""
import numpy as np
import pytest

import checkers
from oracle import earl_oracle as O
from paper_2510_05943_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the GPU parity tests need a real MI355X")
    import gpu_harness
    return gpu_harness


def oracle_plan(w, seq_row=None, balance_policy=0, equal_mb=0):
    return O.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                        seq_group=w.seq_group, seq_row=seq_row, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                        pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget,
                        balance_policy=balance_policy, equal_mb=equal_mb)


PLAN_KEYS = ("rank", "slot", "mb", "dst_row", "seq_shard", "seq_row", "seq_ids", "mb_seq_start",
             "mb_row_start", "cu_seqlens", "n_seq", "n_mb", "shard_rows", "a2a_counts",
             "rank_load")
SEG_KEYS = ("src_shard", "src_row", "dst_shard", "dst_row", "n_real", "n_rows", "pos0")


def assert_plan_equal(res, plan):
    for k in PLAN_KEYS:
        want = getattr(plan, k)
        got = res[k]
        assert got.shape == np.asarray(want).shape, (k, got.shape, np.asarray(want).shape)
        assert np.array_equal(got, want), k
    for k in SEG_KEYS:
        assert np.array_equal(res["segments"][k], getattr(plan, "seg_" + k)), "seg_" + k
    assert np.array_equal(res["segments"]["shard_seg_start"], plan.shard_seg_start)
    assert res["total_real_rows"] == plan.total_real_rows
    assert res["total_dst_rows"] == plan.total_dst_rows
    assert res["n_segments"] == plan.N * plan.K
    assert res["n_mb_max"] == int(plan.n_mb.max())
    assert res["cu_seqlens_len"] == len(plan.cu_seqlens)
    assert res["mb_table_len"] == len(plan.mb_seq_start)
    assert res["rank_load_min"] == int(plan.rank_load.min())
    assert res["rank_load_max"] == int(plan.rank_load.max())
    need = np.zeros(plan.S, np.int64)
    for i in range(plan.N):
        s = int(plan.seq_shard[i])
        need[s] = max(need[s], int(plan.seq_row[i]) + int(plan.L[i]))
    assert np.array_equal(res["src_rows_needed"], need)


def assert_dispatch_equal(w, plan, out, shards_host, fields):
    for q in range(plan.D * plan.C):
        assert np.array_equal(out["position_ids"][q], O.position_ids_shard(plan, q)), ("pos", q)
    assert np.array_equal(out["cu_seqlens"], plan.cu_seqlens)
    for f in fields:
        for q in range(plan.D * plan.C):
            want = O.dispatch_field_shard(plan, q, shards_host[f.name], f.np_dtype, f.width,
                                          f.pad_scalar, per_sequence=f.per_sequence)
            got = out["fields"][f.name][q]
            assert got.shape == want.shape, (f.name, q)
            assert np.array_equal(got, want), (f.name, q)


# ---------------------------------------------------------------------------------------
# the five workloads
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("kernel", ["default", "general"])
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("name", synth.CONFIG_NAMES)
def test_plan_parity_full_size(H, name, seed, kernel, monkeypatch):
    if kernel == "general":
        monkeypatch.setenv("EARL_PLAN_KERNEL", "general")
    w = synth.make_workload(name, seed=seed)
    plan = H.build_plan(w)
    res = H.plan_result(plan)
    assert_plan_equal(res, oracle_plan(w))
    H.B.plan_destroy(plan)


@pytest.mark.parametrize("name,seed,scale", [
    ("tiny", 0, 1.0), ("tiny", 1, 1.0), ("tiny", 2, 1.0),
    ("mid", 0, 1.0), ("mid", 1, 0.25),
    ("agentic", 0, 1.0), ("agentic", 2, 0.25),
    ("heavy", 0, 0.01), ("heavy", 1, 0.02),
    ("longctx", 0, 0.04),
])
def test_dispatch_parity(H, name, seed, scale):
    w = synth.make_workload(name, seed=seed, scale=scale)
    oplan = oracle_plan(w)
    plan = H.build_plan(w)
    assert_plan_equal(H.plan_result(plan), oplan)
    groups, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.plan_destroy(plan)


def test_dispatch_is_deterministic_and_field_order_free(H):
    w = synth.make_workload("mid", seed=3, scale=0.25)
    plan = H.build_plan(w)
    _, shards = H.host_sources(w, w.fields)
    a = H.run_dispatch(w, plan, w.fields, src_host=shards)
    b = H.run_dispatch(w, plan, tuple(reversed(w.fields)), src_host=shards)
    one = H.run_dispatch(w, plan, w.fields[:1], src_host=shards, want_position_ids=False,
                         want_cu=False)
    for f in w.fields:
        for x, y in zip(a["fields"][f.name], b["fields"][f.name]):
            assert np.array_equal(x, y)
    for x, y in zip(a["fields"][w.fields[0].name], one["fields"][w.fields[0].name]):
        assert np.array_equal(x, y)
    H.B.plan_destroy(plan)


def test_replicas_are_read_only_where_the_plan_says(H):
    """Rows of a replica outside its share are poisoned; the result must not change."""
    w = synth.make_workload("agentic", seed=1, scale=0.25)
    oplan = oracle_plan(w)
    plan = H.build_plan(w)
    _, shards = H.host_sources(w, w.fields)
    poisoned = {}
    for f in w.fields:
        bufs = [np.full_like(b, 0xA5) for b in shards[f.name]]
        for i in range(w.n_seqs):
            s, r0, n = int(oplan.seq_shard[i]), int(oplan.seq_row[i]), int(w.lengths[i])
            bufs[s][r0:r0 + n] = shards[f.name][s][r0:r0 + n]
        poisoned[f.name] = bufs
    out = H.run_dispatch(w, plan, w.fields, src_host=poisoned)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.plan_destroy(plan)


# ---------------------------------------------------------------------------------------
# small random batches: odd widths, every layout option, trace-back check and inverse
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


ODD_FIELDS = (synth.F_ID, synth.F_MASK, synth.bytes_field("wide", 2, 24, 0xBEEF),
              synth.bytes_field("odd", 4, 3, 0x01020304), synth.bytes_field("b8", 8, 1, 0x1122334455667788),
              synth.bytes_field("b6", 2, 3, 0x7777), synth.bytes_field("row16", 4, 4, 0xABCD0123),
              synth.bytes_field("bf16x64", 2, 64, 0x3F80))


@pytest.mark.parametrize("case", small_cases(), ids=lambda c: f"case{c['seed']}")
def test_small_batches(H, case):
    w = synth.custom_workload(case["L"], n_groups=case["G"], replication=case["R"],
                              seq_group=case["grp"], dp=case["D"], sp=case["C"], zigzag=case["z"],
                              pad_multiple=case["P"], mb_token_budget=case["B"], fields=ODD_FIELDS,
                              seed=case["seed"])
    oplan = oracle_plan(w)
    plan = H.build_plan(w, explicit_groups=bool(case["seed"] % 4 == 1))
    res = H.plan_result(plan)
    assert_plan_equal(res, oplan)
    groups, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    # the result explains itself: every row traces back to its source token
    res["position_ids"] = out["position_ids"]
    res["cu_seqlens"] = out["cu_seqlens"]
    checkers.check_structure(res, w.lengths, w.dp, w.sp, oplan.K, w.pad_multiple, w.mb_token_budget)
    src_row = checkers.packed_source_rows(w.lengths, w.seq_group, w.n_groups)
    for f in w.fields:
        pad = np.full((f.width,), f.pad_scalar & ((1 << (8 * f.scalar_bytes)) - 1), f.np_dtype)
        checkers.check_self_describing(res, w.lengths, w.dp, w.sp, groups[f.name], w.seq_group,
                                       src_row, out["fields"][f.name], pad)
    # inverse: back to the rollout layout, untouched where nothing was read
    import torch
    back = {f.name: [torch.full_like(t, 0x5A) for t in out["src_dev"][f.name]] for f in w.fields}
    bfields = [H.B.Field(f.scalar_bytes, f.width, f.pad_scalar, back[f.name], out["dev"][f.name])
               for f in w.fields]
    H.B.dispatch_inverse(plan, bfields, workspace=out["workspace"])
    torch.cuda.synchronize()
    for f in w.fields:
        want = [np.full_like(b, 0x5A) for b in shards[f.name]]
        O.inverse_field(oplan, out["fields"][f.name], want)
        for s in range(w.n_shards):
            got = back[f.name][s].cpu().numpy().view(f.np_dtype).reshape(-1, f.width)
            assert np.array_equal(got, want[s]), (f.name, s)
    H.B.plan_destroy(plan)


def _dispatch_and_inverse_equal_oracle(H, w):
    import torch
    oplan = oracle_plan(w)
    plan = H.build_plan(w)
    assert_plan_equal(H.plan_result(plan), oplan)
    _, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    back = {f.name: [torch.full_like(t, 0x5A) for t in out["src_dev"][f.name]] for f in w.fields}
    bfields = [H.B.Field(f.scalar_bytes, f.width, f.pad_scalar, back[f.name], out["dev"][f.name])
               for f in w.fields]
    H.B.dispatch_inverse(plan, bfields, workspace=out["workspace"])
    torch.cuda.synchronize()
    for f in w.fields:
        want = [np.full_like(b, 0x5A) for b in shards[f.name]]
        O.inverse_field(oplan, out["fields"][f.name], want)
        for s in range(w.n_shards):
            got = back[f.name][s].cpu().numpy().view(f.np_dtype).reshape(-1, f.width)
            assert np.array_equal(got, want[s]), (f.name, s)
    H.B.plan_destroy(plan)


@pytest.mark.parametrize("n,dp,sp,zigzag,groups,rep", [(2500, 8, 2, 1, 8, 1), (4096, 16, 1, 0, 4, 2)])
def test_both_directions_beyond_2048_sequences(H, n, dp, sp, zigzag, groups, rep):
    """Dispatch and reverse dispatch behind the plan kernel that keeps up to 4096 sequences in LDS
    (its segment table reads the per-sequence outputs back from the workspace)."""
    w = synth.custom_workload([(i * 7919) % 211 + 1 for i in range(n)], n_groups=groups, replication=rep,
                              dp=dp, sp=sp, zigzag=zigzag, pad_multiple=2, mb_token_budget=4096,
                              fields=(synth.F_ID, synth.F_MASK, synth.bytes_field("w40", 8, 5, 0x0102030405060708)),
                              seed=n)
    _dispatch_and_inverse_equal_oracle(H, w)


@pytest.mark.parametrize("n,dp,sp,zigzag,groups,rep", [(300, 3, 2, 1, 4, 1), (2500, 8, 2, 1, 8, 1),
                                                      (700, 5, 4, 0, 2, 3)])
def test_both_directions_behind_the_general_plan_kernel(H, monkeypatch, n, dp, sp, zigzag, groups, rep):
    """The reverse direction takes the prefix of real rows from the plan kernel's scan of the
    lengths when the kernel that keeps the batch in LDS built the plan, and from a scan over the
    segment table otherwise: this is the second case (forced for the small batches, natural for the
    one beyond 2048 sequences), compared with the oracle like the first."""
    monkeypatch.setenv("EARL_PLAN_KERNEL", "general")
    w = synth.custom_workload([(i * 7919) % 211 + 1 for i in range(n)], n_groups=groups, replication=rep,
                              dp=dp, sp=sp, zigzag=zigzag, pad_multiple=2, mb_token_budget=4096,
                              fields=(synth.F_ID, synth.F_MASK, synth.bytes_field("w40", 8, 5, 0x0102030405060708)),
                              seed=n)
    _dispatch_and_inverse_equal_oracle(H, w)


DIRECT_KERNEL_CASES = [
    # more segments in a 4 KiB job than the 64 a wavefront keeps: single-row sequences cut into
    # many chunks, one-byte and two-byte rows (the per-lane path beyond the window)
    ("segments_of_one_byte", dict(L=[1 + (i % 3) for i in range(1500)], dp=2, sp=2, zigzag=1,
                                  B=64), (synth.F_MASK, synth.bytes_field("h", 2, 1, 0x0101))),
    ("segments_of_a_few_bytes", dict(L=[(i * 7) % 5 + 1 for i in range(900)], G=3, R=2, dp=3, sp=4,
                                     zigzag=1, pad=2, B=512),
     (synth.F_MASK, synth.F_ID, synth.bytes_field("b6", 2, 3, 0x7777))),
    # more than 64 source shards and more than 64 destination shards: pointers looked up per
    # segment instead of held one per lane (both directions)
    ("source_shards_96", dict(L=[(i * 37) % 200 + 1 for i in range(700)], G=48, R=2, dp=4, sp=2,
                              zigzag=1, B=4096), (synth.F_ID, synth.F_MASK, synth.F_OLD)),
    ("destination_shards_130", dict(L=[(i * 53) % 300 + 1 for i in range(800)], G=4, dp=65, sp=2,
                                    B=8192), (synth.F_ID, synth.F_MASK)),
    # wide rows in a small launch (decoded in the copy kernel as well), odd widths, rows that are
    # not a multiple of 16 bytes, padding that is not zero
    ("wide_rows_small_launch", dict(L=[(i * 101) % 700 + 1 for i in range(300)], G=4, dp=4, sp=2,
                                    zigzag=1, pad=8, B=8192),
     (synth.bytes_field("bf16x1024", 2, 1024, 0x3F80), synth.bytes_field("w24", 8, 3, 0x1122334455667788),
      synth.bytes_field("w50", 2, 25, 0xBEEF), synth.F_MASK)),
    # many records (a field table of more than 64 entries), shards of a few rows, empty ranks
    ("many_small_shards", dict(L=[(i * 11) % 9 + 1 for i in range(90)], G=2, dp=40, sp=3, zigzag=1,
                               B=64), (synth.F_ID, synth.F_MASK, synth.F_OLD, synth.F_ADV)),
]


@pytest.mark.parametrize("desc,kw,fields", DIRECT_KERNEL_CASES, ids=[c[0] for c in DIRECT_KERNEL_CASES])
def test_rare_paths_of_the_direct_kernels(H, desc, kw, fields):
    """Dispatch and reverse dispatch against the oracle on batches built to leave the common path
    of the kernels that decode inside the copy."""
    w = synth.custom_workload(kw["L"], n_groups=kw.get("G", 1), replication=kw.get("R", 1),
                              dp=kw["dp"], sp=kw["sp"], zigzag=kw.get("zigzag", 0),
                              pad_multiple=kw.get("pad", 1), mb_token_budget=kw["B"], fields=fields,
                              seed=len(kw["L"]))
    _dispatch_and_inverse_equal_oracle(H, w)


def test_field_shape_limits(H):
    """The widest row the library accepts (1 MiB), a row one scalar short of it (so rows are not
    a multiple of 16 bytes and every vector load is unaligned), and the largest number of
    fields in one call, each forward and back."""
    max_row = 1 << 20
    lengths = [3, 1, 5, 2, 4, 1, 2]
    for fields in ((synth.bytes_field("row_1MiB", 8, max_row // 8, 0x0123456789ABCDEF),),
                   (synth.bytes_field("row_1MiB_minus_2", 2, max_row // 2 - 1, 0xA5C3),
                    synth.bytes_field("row_1MiB_minus_1", 1, max_row - 1, 0x5A))):
        w = synth.custom_workload(lengths, n_groups=2, dp=2, sp=2, zigzag=1, pad_multiple=2,
                                  mb_token_budget=1 << 20, fields=fields, seed=41)
        _dispatch_and_inverse_equal_oracle(H, w)
    many = tuple(synth.bytes_field(f"f{k}", (1, 2, 4, 8)[k % 4], 1 + (k * 5) % 7, 0x1F2E3D4C5B6A7988 >> k)
                 for k in range(32))
    rng = np.random.default_rng(43)
    w = synth.custom_workload(rng.integers(1, 400, size=150), n_groups=3, replication=2, dp=3, sp=2,
                              zigzag=1, pad_multiple=4, mb_token_budget=4000, fields=many, seed=43)
    _dispatch_and_inverse_equal_oracle(H, w)
    # one field more is refused before anything is enqueued
    plan = H.build_plan(w)
    sm = H.B.plan_get_summary(plan)
    import torch
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    f33 = [H.B.Field(1, 1, 0, [buf] * w.n_shards, [buf] * sm["n_dst_shards"]) for _ in range(33)]
    with pytest.raises(H.B.EarlError) as e:
        H.B.dispatch(plan, f33, workspace=torch.empty(1 << 22, dtype=torch.uint8, device="cuda"))
    assert e.value.status == H.B.EARL_INVALID_ARG
    H.B.plan_destroy(plan)


def test_dispatch_at_the_largest_sequence_parallel_degree(H):
    """sp = 64 with zigzag: 128 chunks per sequence, most of them a few rows, many all padding."""
    rng = np.random.default_rng(64)
    fields = (synth.F_ID, synth.F_MASK, synth.bytes_field("v", 2, 24, 0x7E57))
    w = synth.custom_workload(rng.integers(1, 700, size=90), n_groups=3, replication=2, dp=2, sp=64,
                              zigzag=1, pad_multiple=1, mb_token_budget=20000, fields=fields, seed=64)
    _dispatch_and_inverse_equal_oracle(H, w)


def test_explicit_source_rows_with_gaps(H):
    rng = np.random.default_rng(21)
    L = rng.integers(1, 300, size=37)
    w = synth.custom_workload(L, n_groups=3, dp=3, sp=2, zigzag=1, pad_multiple=4,
                              mb_token_budget=4096, fields=(synth.F_ID, synth.F_MASK,
                                                            synth.bytes_field("h", 2, 40, 0)))
    # every sequence starts 5 rows after the previous one ends, inside its group's buffer
    packed = checkers.packed_source_rows(w.lengths, w.seq_group, w.n_groups)
    k_in_group = np.zeros(len(L), np.int64)
    for g in range(3):
        idx = np.nonzero(w.seq_group == g)[0]
        k_in_group[idx] = np.arange(len(idx))
    seq_row = packed + 5 * (k_in_group + 1)
    oplan = oracle_plan(w, seq_row=seq_row)
    plan = H.build_plan(w, seq_row=seq_row)
    assert_plan_equal(H.plan_result(plan), oplan)
    shards = {}
    for f in w.fields:
        bufs = []
        for g in range(3):
            packed_buf = w.group_buffer(f, g)
            idx = np.nonzero(w.seq_group == g)[0]
            rows = int(seq_row[idx[-1]] + L[idx[-1]]) if len(idx) else 0
            buf = np.full((rows, f.width), 0xEE, f.np_dtype)
            for i in idx:
                buf[seq_row[i]:seq_row[i] + L[i]] = packed_buf[packed[i]:packed[i] + L[i]]
            bufs.append(buf)
        shards[f.name] = bufs
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.plan_destroy(plan)


# ---------------------------------------------------------------------------------------
# plan-only edge cases (no field data needed)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("desc,kw", [
    ("one_sequence", dict(L=[1], dp=1, sp=1)),
    ("one_sequence_many_ranks", dict(L=[77], dp=7, sp=4, zigzag=1, pad=8, B=1024)),
    ("all_length_one", dict(L=[1] * 300, dp=3, sp=2, zigzag=1, B=8)),
    ("fewer_sequences_than_ranks", dict(L=[5, 9, 2], dp=5, sp=2, zigzag=1, B=100)),
    ("dp_40", dict(L=[(i * 7919) % 601 + 1 for i in range(777)], dp=40, sp=2, zigzag=1, B=100000)),
    ("many_shard_pairs", dict(L=[(i * 13) % 70 + 1 for i in range(900)], G=64, dp=48, sp=1, B=100000)),
    ("dp_100", dict(L=list(range(1, 1301)), dp=100, sp=1, B=100000)),
    ("dp_1024", dict(L=[(i * 7919) % 997 + 1 for i in range(3000)], dp=1024, sp=1, B=100000)),
    ("groups_300", dict(L=[(i * 31) % 50 + 1 for i in range(2500)], G=300, dp=4, sp=2, B=1 << 20)),
    ("replicated_5x3", dict(L=[(i * 17) % 90 + 1 for i in range(157)], G=5, R=3, dp=2, sp=3, B=4096)),
    ("n_9000_global_sort", dict(L=[(i * 2654435761) % 4000 + 1 for i in range(9000)], dp=16, sp=2,
                                zigzag=1, pad=16, B=20000)),
    ("loads_beyond_32_bits", dict(L=[1 << 30] * 5 + [(1 << 30) - 12345] * 6, dp=3, sp=1, B=(1 << 31) - 1)),
    ("equal_lengths_round_robin", dict(L=[64] * 96, dp=8, sp=2, B=1 << 20)),
    # sort keys: one padded length of 2^21 or more switches the whole batch to the 64-bit packing
    ("wide_keys_1500_sequences", dict(L=[(i * 7919) % 5000 + 1 for i in range(1500)] +
                                      [3 << 20, 1 << 21, (1 << 21) - 1], dp=24, sp=2, zigzag=1, B=1 << 30)),
    ("narrow_keys_at_their_limit", dict(L=[(1 << 21) - 1 - (i % 3) for i in range(2048)], dp=1, sp=1,
                                        B=1 << 30)),
    ("narrow_keys_at_their_limit_dp_9", dict(L=[(1 << 21) - 1 - i for i in range(70)] +
                                             [(i * 13) % 999 + 1 for i in range(500)], dp=9, sp=1)),
    # beyond 2048 sequences the batch still stays in LDS, with 12 index bits in the narrow keys
    ("sequences_4096_ranks_64", dict(L=[(i * 7919) % 3001 + 1 for i in range(4096)], G=16, dp=64, sp=1,
                                     B=1 << 17, packed=True)),
    ("sequences_2049", dict(L=[(i * 104729) % 777 + 1 for i in range(2049)], G=4, R=2, dp=5, sp=2, zigzag=1,
                            pad=4, B=1 << 15, packed=True)),
    ("sequences_3000_wide_keys", dict(L=[(i * 31) % 4000 + 1 for i in range(2999)] + [1 << 20], dp=12, sp=2,
                                      B=1 << 30)),
    ("sequences_3000_narrow_keys_at_their_limit", dict(L=[(i * 31) % 4000 + 1 for i in range(2998)] +
                                                       [(1 << 20) - 1, (1 << 20) - 2], dp=12, sp=1, B=1 << 30)),
    ("budget_exactly_one_sequence", dict(L=[16] * 40, dp=2, sp=2, zigzag=1, B=16)),
    ("sp_64_zigzag_128_chunks", dict(L=[(i * 37) % 900 + 1 for i in range(120)], G=3, dp=3, sp=64,
                                     zigzag=1, pad=2, B=40000)),
    ("src_shards_4096", dict(L=[(i * 11) % 40 + 1 for i in range(6000)], G=2048, R=2, dp=2, sp=2,
                             B=100000)),
    ("dp_1024_sp_4_groups_64", dict(L=[(i * 29) % 300 + 1 for i in range(5000)], G=64, dp=1024, sp=4,
                                    zigzag=1, B=100000)),
])
def test_plan_edge_cases(H, desc, kw):
    w = synth.custom_workload(kw["L"], n_groups=kw.get("G", 1), replication=kw.get("R", 1),
                              dp=kw["dp"], sp=kw["sp"], zigzag=kw.get("zigzag", 0),
                              pad_multiple=kw.get("pad", 1), mb_token_budget=kw.get("B", 1 << 40))
    if kw.get("G", 1) > 1 and not kw.get("packed"):
        rng = np.random.default_rng(len(kw["L"]))
        w.seq_group = rng.integers(0, kw["G"], size=len(kw["L"])).astype(np.int32)
    plan = H.build_plan(w)
    assert_plan_equal(H.plan_result(plan), oracle_plan(w))
    H.B.plan_destroy(plan)


def test_more_plans_alive_than_summary_mailboxes(H):
    """The library hands a plan's totals to the host through one of 64 pinned mailboxes; plans
    beyond that read their totals with a copy.  All 80 plans built here are alive at once, every
    one is compared with the oracle, in an order that differs from the order they were built in."""
    works = [synth.custom_workload([(i * (7 + k)) % 97 + 1 for i in range(40 + 3 * k)], n_groups=2,
                                   dp=1 + k % 5, sp=1 + k % 3, zigzag=k % 2, pad_multiple=1 + k % 4,
                                   mb_token_budget=4096) for k in range(80)]
    plans = [H.build_plan(w) for w in works]
    for k in list(range(79, -1, -2)) + list(range(0, 80, 2)):
        assert_plan_equal(H.plan_result(plans[k]), oracle_plan(works[k]))
    for plan in plans:
        H.B.plan_destroy(plan)


def test_one_workspace_reused_by_batches_of_different_shape(H):
    """Plans built one after the other in the SAME workspace (the earlier plan destroyed first):
    nothing of an earlier batch may show in a later one, whichever kernel serves it."""
    import torch
    shapes = [dict(n=1500, dp=24, sp=2, zz=1), dict(n=40, dp=3, sp=1, zz=0), dict(n=700, dp=16, sp=4, zz=1),
              dict(n=2048, dp=64, sp=1, zz=0), dict(n=2300, dp=8, sp=2, zz=1), dict(n=64, dp=16, sp=2, zz=1)]
    works = [synth.custom_workload([(i * 7919 + 13 * k) % (3000 // (k + 1)) + 1 for i in range(sh["n"])],
                                   n_groups=4, dp=sh["dp"], sp=sh["sp"], zigzag=sh["zz"],
                                   mb_token_budget=1 << 16) for k, sh in enumerate(shapes)]
    layouts = [H.layouts_of(w, False, None, 0, 0) for w in works]
    size = max(H.B.plan_workspace_bytes(w.n_seqs, src, dst) for w, (src, dst, _) in zip(works, layouts))
    ws = torch.empty(size, dtype=torch.uint8, device="cuda")
    for rounds in range(2):
        for w, (src, dst, keep) in zip(works, layouts):
            lengths = H.to_dev(w.lengths.astype(np.int32))
            plan = H.B.plan_build(lengths, w.n_seqs, src, dst, ws)
            assert_plan_equal(H.plan_result(plan), oracle_plan(w))
            H.B.plan_destroy(plan)


@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("mid", 1.0), ("agentic", 1.0), ("heavy", 1.0),
                                        ("longctx", 1.0), ("mid", 0.02)])
def test_snake_deal_policy(H, name, scale):
    w = synth.make_workload(name, seed=5, scale=scale)
    plan = H.build_plan(w, balance_policy=1)
    oplan = oracle_plan(w, balance_policy=1)
    assert_plan_equal(H.plan_result(plan), oplan)
    if name in ("tiny", "mid") and scale == 1.0:
        _, shards = H.host_sources(w, w.fields)
        out = H.run_dispatch(w, plan, w.fields, src_host=shards)
        assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.plan_destroy(plan)


@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("mid", 1.0), ("agentic", 1.0), ("heavy", 1.0),
                                        ("longctx", 1.0), ("mid", 0.02)])
def test_quadratic_cost_policy_and_equal_micro_batch_counts(H, name, scale):
    """balance_policy 2 (list scheduling on squared padded lengths) with equal_mb: plan parity on
    every workload, dispatch parity (fields, position ids, cu_seqlens with the empty
    micro-batches) on the two small ones."""
    w = synth.make_workload(name, seed=6, scale=scale)
    plan = H.build_plan(w, balance_policy=2, equal_mb=1)
    oplan = oracle_plan(w, balance_policy=2, equal_mb=1)
    res = H.plan_result(plan)
    assert_plan_equal(res, oplan)
    assert res["n_mb"].tolist() == [res["n_mb_max"]] * w.dp
    if name in ("tiny", "mid") and scale == 1.0:
        _, shards = H.host_sources(w, w.fields)
        out = H.run_dispatch(w, plan, w.fields, src_host=shards)
        assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.plan_destroy(plan)


def test_equal_micro_batch_counts_with_tight_budget_and_empty_ranks(H):
    """Many micro-batches on some ranks, none on others (fewer sequences than ranks)."""
    rng = np.random.default_rng(31)
    for D, N, hi, budget in ((4, 200, 900, 1000), (7, 3, 50, 50), (64, 40, 300, 300),
                             (130, 500, 64, 64), (2, 1, 5, 5)):
        L = rng.integers(1, hi + 1, size=N)
        w = synth.custom_workload(L, dp=D, sp=2, zigzag=1, mb_token_budget=budget + 3,
                                  fields=(synth.F_ID,), seed=D)
        for policy in (0, 1, 2):
            plan = H.build_plan(w, balance_policy=policy, equal_mb=1)
            oplan = oracle_plan(w, balance_policy=policy, equal_mb=1)
            assert_plan_equal(H.plan_result(plan), oplan)
            if policy == 0:
                _, shards = H.host_sources(w, w.fields)
                out = H.run_dispatch(w, plan, w.fields, src_host=shards)
                assert_dispatch_equal(w, oplan, out, shards, w.fields)
            H.B.plan_destroy(plan)


def test_quadratic_policy_rejects_padded_lengths_beyond_its_limit(H):
    w = synth.custom_workload([10, (1 << 21) + 1, 7], dp=2, sp=1, mb_token_budget=1 << 40)
    plan = H.build_plan(w, balance_policy=2)
    with pytest.raises(H.B.EarlError) as e:
        H.B.plan_get_summary(plan)
    assert e.value.status == H.B.EARL_INVALID_ARG
    H.B.plan_destroy(plan)
    # the limit itself is fine, and the squares are added exactly
    w = synth.custom_workload([1 << 21, (1 << 21) - 1, (1 << 21) - 2, 5, 1 << 20], dp=2, sp=1,
                              mb_token_budget=1 << 40)
    plan = H.build_plan(w, balance_policy=2)
    assert_plan_equal(H.plan_result(plan), oracle_plan(w, balance_policy=2))
    H.B.plan_destroy(plan)


COUNT_FIELDS = (synth.F_MASK, synth.sparse_field("s_u8x3", 1, 3, 0xAB), synth.sparse_field("s_u16", 2, 1, 0xFFFF),
                synth.sparse_field("s_u16x5", 2, 5, 1), synth.sparse_field("s_u32", 4, 1, 7),
                synth.sparse_field("s_u32x3", 4, 3, 0), synth.sparse_field("s_u64", 8, 1, 9), synth.F_ID)


@pytest.mark.parametrize("case", small_cases()[1::3] + [
    dict(L=np.random.default_rng(19).integers(1, 3000, size=400), G=4, R=2, D=4, C=2, z=1, P=8,
         B=9000, grp=None, seed=98),
    dict(L=np.random.default_rng(20).integers(1, 40, size=900), G=1, R=1, D=3, C=1, z=0, P=1,
         B=64, grp=None, seed=97)], ids=lambda c: f"case{c['seed']}")
def test_nonzero_counts_per_micro_batch(H, case):
    """The counting consumer: every scalar size, widths that do not divide 16, non-zero padding
    scalars (which must not count), many small micro-batches, equal_mb on and off."""
    w = synth.custom_workload(case["L"], n_groups=case["G"], replication=case["R"],
                              seq_group=case["grp"], dp=case["D"], sp=case["C"], zigzag=case["z"],
                              pad_multiple=case["P"], mb_token_budget=case["B"], fields=COUNT_FIELDS,
                              seed=case["seed"])
    for equal_mb in (0, 1):
        oplan = oracle_plan(w, equal_mb=equal_mb)
        plan = H.build_plan(w, equal_mb=equal_mb)
        _, shards = H.host_sources(w, w.fields)
        names = [f.name for f in COUNT_FIELDS[:-1]]
        out = H.run_dispatch(w, plan, w.fields, src_host=shards, count_nonzero=names)
        assert_dispatch_equal(w, oplan, out, shards, w.fields)
        for f in COUNT_FIELDS[:-1]:
            want = O.nonzero_counts(oplan, shards[f.name], f.width)
            assert np.array_equal(out["nonzero_counts"][f.name], want), f.name
        H.B.plan_destroy(plan)


def test_nonzero_counts_on_the_mid_workload_and_argument_checks(H):
    import torch
    w = synth.make_workload("mid", seed=3)
    plan, oplan = H.build_plan(w), oracle_plan(w)
    _, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards, count_nonzero=["loss_mask"])
    want = O.nonzero_counts(oplan, shards["loss_mask"])
    assert np.array_equal(out["nonzero_counts"]["loss_mask"], want)
    assert int(want.sum()) == sum(int(np.count_nonzero(a)) for a in shards["loss_mask"][::w.replication])
    # a second call into the same array starts from zero again
    sm = H.B.plan_get_summary(plan)
    n_dst = sm["n_dst_shards"]
    mask = [f for f in w.fields if f.name == "loss_mask"][0]
    cnt = torch.full((n_dst * sm["n_mb_max"],), 123, dtype=torch.int64, device="cuda")
    dsts = [torch.empty((int(r),), dtype=torch.uint8, device="cuda") for r in sm["shard_rows"]]
    fld = H.B.Field(1, 1, 0, out["src_dev"]["loss_mask"], dsts, nonzero_counts=cnt)
    ws = torch.empty(H.B.dispatch_workspace_bytes(plan, [fld], False, False), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        H.B.dispatch(plan, [fld], workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(cnt.cpu().numpy().reshape(n_dst, -1), want)
    # too small an array, a wide field, a per-sequence field, the inverse
    small = H.B.Field(1, 1, 0, out["src_dev"]["loss_mask"], dsts, nonzero_counts=cnt[:-1])
    with pytest.raises(H.B.EarlError) as e:
        H.B.dispatch(plan, [small], workspace=ws)
    assert e.value.status == H.B.EARL_CAPACITY
    wide_dst = [torch.empty((int(r) * 16,), dtype=torch.uint8, device="cuda") for r in sm["shard_rows"]]
    wide_src = [torch.zeros((int(r) * 16,), dtype=torch.uint8, device="cuda") for r in sm["src_rows_needed"]]
    wide = H.B.Field(4, 4, 0, wide_src, wide_dst, nonzero_counts=cnt)
    with pytest.raises(H.B.EarlError) as e:
        H.B.dispatch(plan, [wide], workspace=torch.empty(1 << 24, dtype=torch.uint8, device="cuda"))
    assert e.value.status == H.B.EARL_INVALID_ARG
    with pytest.raises(H.B.EarlError) as e:
        H.B.dispatch_inverse(plan, [fld], workspace=ws)
    assert e.value.status == H.B.EARL_INVALID_ARG
    H.B.plan_destroy(plan)


SEQ_FIELDS = (synth.per_sequence_field("adv_f32", 4, 1, 0x7FC00000), synth.per_sequence_field("flag_u8", 1),
              synth.per_sequence_field("pair_u16", 2, 2, 0xBEEF), synth.per_sequence_field("ret_f64", 8, 1, 5),
              synth.per_sequence_field("half", 2, 1, 0x3C00), synth.F_ID)


@pytest.mark.parametrize("case", small_cases()[::3] + [dict(L=np.random.default_rng(9).integers(1, 3000, size=300),
                                                           G=4, R=2, D=4, C=2, z=1, P=8, B=1 << 20, grp=None,
                                                           seed=99)],
                         ids=lambda c: f"case{c['seed']}")
def test_per_sequence_fields_are_broadcast(H, case):
    w = synth.custom_workload(case["L"], n_groups=case["G"], replication=case["R"],
                              seq_group=case["grp"], dp=case["D"], sp=case["C"], zigzag=case["z"],
                              pad_multiple=case["P"], mb_token_budget=case["B"], fields=SEQ_FIELDS,
                              seed=case["seed"])
    oplan = oracle_plan(w)
    plan = H.build_plan(w)
    res = H.plan_result(plan)
    assert_plan_equal(res, oplan)
    need = np.zeros(oplan.S, np.int64)
    for i in range(oplan.N):
        need[oplan.seq_shard[i]] = max(need[oplan.seq_shard[i]], int(oplan.seq_k[i]) + 1)
    assert np.array_equal(res["src_seqs_needed"], need)
    _, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    # not invertible, and only scalar-sized rows
    B = H.B
    f = SEQ_FIELDS[0]
    bf = B.Field(4, 1, 0, out["src_dev"][f.name], out["dev"][f.name], per_sequence=True)
    with pytest.raises(B.EarlError) as e:
        B.dispatch_inverse(plan, [bf], workspace=out["workspace"])
    assert e.value.status == B.EARL_INVALID_ARG
    with pytest.raises(B.EarlError) as e:
        B.dispatch(plan, [B.Field(4, 4, 0, out["src_dev"][f.name], out["dev"][f.name], per_sequence=True)],
                   workspace=out["workspace"])
    assert e.value.status == B.EARL_INVALID_ARG
    B.plan_destroy(plan)


def test_two_pass_gather_then_scatter_equals_direct_dispatch(H):
    """Gathering everything into one canonical buffer and scattering it from there (the
    single-controller pattern) gives the same training layout as the direct dispatch."""
    import torch
    B = H.B
    w = synth.make_workload("mid", seed=6, scale=0.25)
    _, shards = H.host_sources(w, w.fields)
    direct_plan = H.build_plan(w)
    direct = H.run_dispatch(w, direct_plan, w.fields, src_host=shards)
    gather_w = synth.custom_workload(w.lengths, n_groups=w.n_groups, replication=w.replication,
                                     seq_group=w.seq_group, dp=1, sp=1, fields=w.fields)
    gather_plan = H.build_plan(gather_w)
    one = H.run_dispatch(gather_w, gather_plan, w.fields, src_host=shards, want_position_ids=False,
                         want_cu=False)
    scatter_w = synth.custom_workload(w.lengths, n_groups=1, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                                      pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget,
                                      fields=w.fields)
    scatter_plan = H.build_plan(scatter_w)
    canon = {f.name: [one["fields"][f.name][0]] for f in w.fields}
    two = H.run_dispatch(scatter_w, scatter_plan, w.fields, src_host=canon)
    for f in w.fields:
        for a, b in zip(two["fields"][f.name], direct["fields"][f.name]):
            assert np.array_equal(a, b), f.name
    for a, b in zip(two["position_ids"], direct["position_ids"]):
        assert np.array_equal(a, b)
    for p in (direct_plan, gather_plan, scatter_plan):
        B.plan_destroy(p)


@pytest.mark.parametrize("kernel", ["default", "general"])
def test_random_plans_sweep(H, kernel, monkeypatch):
    """Plan-only parity on many random layouts: every size class of the rank-assignment code
    (1, 2, 4, 8, 16, 64 and more ranks), tight budgets with many micro-batches, replicated and
    scattered source groups, all balancing policies, equal micro-batch counts on and off.
    The library has two plan kernels (one that keeps a batch of up to 4096 sequences in registers
    and LDS, one for everything else); "general" sends every case through the second."""
    if kernel == "general":
        monkeypatch.setenv("EARL_PLAN_KERNEL", "general")
    rng = np.random.default_rng(2024)
    for t in range(160):
        D = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 33, 64, 65, 130]))
        C = int(rng.choice([1, 1, 2, 3, 4, 8]))
        z = int(rng.integers(0, 2))
        P = int(rng.choice([1, 1, 4, 64]))
        G = int(rng.choice([1, 2, 5, 8]))
        R = int(rng.choice([1, 1, 2, 4]))
        N = int(rng.integers(1, 700)) if t % 8 else int(rng.integers(1000, 4097))
        hi = int(rng.choice([8, 300, 5000]))
        L = rng.integers(1, hi + 1, size=N)
        K = 2 * C if (z and C > 1) else C
        worst = K * P * (-(-(-(-int(L.max()) // K)) // P))
        B = int(worst * rng.choice([1, 1, 2, 7, 1000]))
        policy = int(rng.integers(0, 2))
        if t % 4 == 1:
            policy = 2
        equal_mb = int(t % 5 < 2)
        w = synth.custom_workload(L, n_groups=G, replication=R, dp=D, sp=C, zigzag=z,
                                  pad_multiple=P, mb_token_budget=B, seed=t)
        if t % 3 == 0:
            w.seq_group = rng.integers(0, G, size=N).astype(np.int32)
        plan = H.build_plan(w, balance_policy=policy, equal_mb=equal_mb)
        try:
            assert_plan_equal(H.plan_result(plan),
                              oracle_plan(w, balance_policy=policy, equal_mb=equal_mb))
        except AssertionError as err:
            raise AssertionError(f"case {t}: N={N} D={D} C={C} z={z} P={P} G={G} R={R} B={B} "
                                 f"policy={policy} equal_mb={equal_mb}: {err}")
        H.B.plan_destroy(plan)


def test_dispatch_with_empty_ranks_and_no_fields(H):
    w = synth.custom_workload([5, 9, 2], dp=5, sp=2, zigzag=1, mb_token_budget=100,
                              fields=(synth.F_ID, synth.F_MASK))
    oplan = oracle_plan(w)
    plan = H.build_plan(w)
    _, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.dispatch(plan, [], position_ids=None, cu_seqlens=None)     # nothing to do is not an error
    assert H.B.dispatch_workspace_bytes(plan, [], False, False) < 4096
    H.B.plan_destroy(plan)


# ---------------------------------------------------------------------------------------
# error paths: detected on the device or on the host, nothing is written
# ---------------------------------------------------------------------------------------
def test_errors(H):
    import torch
    B = H.B
    # a zero length
    w = synth.custom_workload([4, 0, 7], dp=2)
    plan = H.build_plan(w)
    with pytest.raises(B.EarlError) as e:
        B.plan_get_summary(plan)
    assert e.value.status == B.EARL_INVALID_ARG
    B.plan_destroy(plan)
    # a group id out of range
    w = synth.custom_workload([4, 5, 7], n_groups=2, dp=2)
    w.seq_group = np.array([0, 2, 1], np.int32)
    plan = H.build_plan(w)
    with pytest.raises(B.EarlError) as e:
        B.plan_get_summary(plan)
    assert e.value.status == B.EARL_INVALID_ARG
    B.plan_destroy(plan)
    # a sequence over the budget
    w = synth.custom_workload([10, 200], dp=1, sp=2, zigzag=1, mb_token_budget=199)
    plan = H.build_plan(w)
    with pytest.raises(B.EarlError) as e:
        B.plan_get_summary(plan)
    assert e.value.status == B.EARL_SEQ_EXCEEDS_BUDGET
    with pytest.raises(B.EarlError) as e:
        B.dispatch(plan, [])
    assert e.value.status == B.EARL_SEQ_EXCEEDS_BUDGET
    B.plan_destroy(plan)
    # capacity, alignment and field-shape errors leave the destination untouched
    w = synth.custom_workload([33, 18, 90, 7], dp=2, sp=2, zigzag=1, mb_token_budget=4096,
                              fields=(synth.F_ID,))
    plan = H.build_plan(w)
    sm = B.plan_get_summary(plan)
    f = synth.F_ID
    _, shards = H.host_sources(w, w.fields)
    srcs = [H.to_dev(a) for a in shards[f.name]]
    rows = [int(x) for x in sm["shard_rows"]]
    good = [torch.full((r * 4 + 64,), 0xCD, dtype=torch.uint8, device="cuda") for r in rows]

    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")

    def attempt(dsts, sb=4, width=1, srcs_=None, ws=scratch):
        with pytest.raises(B.EarlError) as e:
            B.dispatch(plan, [B.Field(sb, width, 0, srcs_ or srcs, dsts)], workspace=ws)
        torch.cuda.synchronize()
        for t in good:
            assert bool((t == 0xCD).all().item())
        return e.value.status

    small = [t[:max(0, r * 4 - 4)] for t, r in zip(good, rows)]
    assert attempt(small) == B.EARL_CAPACITY
    assert attempt([t[4:] for t in good]) == B.EARL_INVALID_ARG          # not 16-byte aligned
    assert attempt([t[:r * 4] for t, r in zip(good, rows)], sb=3) == B.EARL_INVALID_ARG
    assert attempt([t[:r * 4] for t, r in zip(good, rows)], width=0) == B.EARL_INVALID_ARG
    assert attempt([t[:r * 4] for t, r in zip(good, rows)],
                   srcs_=[s[:-1] for s in srcs]) == B.EARL_CAPACITY       # source too short
    assert attempt([None] + [t[:r * 4] for t, r in zip(good[1:], rows[1:])]) == B.EARL_INVALID_ARG
    fit = [t[:r * 4] for t, r in zip(good, rows)]
    assert attempt(fit, ws=None) == B.EARL_INVALID_ARG                   # no scratch
    assert attempt(fit, ws=scratch[:64]) == B.EARL_CAPACITY              # scratch too small
    assert attempt(fit, ws=scratch[8:]) == B.EARL_INVALID_ARG            # scratch misaligned
    # and the same plan still works afterwards
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    assert_dispatch_equal(w, oracle_plan(w), out, shards, w.fields)
    B.plan_destroy(plan)

"""earl_dispatch_async through the C ABI: the same bytes as the oracle with launches sized by buffer
capacities, nothing written when the device-side checks fail, rows beyond a shard's size untouched."""
import numpy as np
import pytest

from oracle import earl_oracle as O
from paper_2510_05943_amd import synth

pytestmark = pytest.mark.gpu

POISON = 0xCD


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import gpu_harness
    return gpu_harness


def oracle_plan(w):
    return O.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                        seq_group=w.seq_group, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                        pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget)


def enqueue(H, w, fields, dst_rows, src_bufs, cu_entries, lengths=None):
    """earl_plan_build and earl_dispatch_async back to back, no host wait in between.
    dst_rows[q] = capacity of every destination buffer of shard q."""
    import torch
    B = H.B
    src, dst, keep = H.layouts_of(w, False)
    lens = H.to_dev(np.asarray(w.lengths if lengths is None else lengths).astype(np.int32))
    ws = torch.empty(B.plan_workspace_bytes(w.n_seqs, src, dst), dtype=torch.uint8, device="cuda")
    bufs, bfields = {}, []
    for f in fields:
        bufs[f.name] = [torch.full((int(r) * f.row_bytes,), POISON, dtype=torch.uint8, device="cuda")
                        for r in dst_rows]
        bfields.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src_bufs[f.name], bufs[f.name],
                               per_sequence=f.per_sequence))
    pos = [torch.full((int(r),), -2, dtype=torch.int32, device="cuda") for r in dst_rows]
    cu = torch.full((cu_entries,), -2, dtype=torch.int32, device="cuda")
    scratch = None
    plan = B.plan_build(lens, w.n_seqs, src, dst, ws)
    plan.keepalive = plan.keepalive + tuple(keep) + (lens,)
    scratch = torch.empty(B.dispatch_async_workspace_bytes(plan, bfields, pos, cu), dtype=torch.uint8,
                          device="cuda")
    B.dispatch_async(plan, bfields, position_ids=pos, cu_seqlens=cu, workspace=scratch)
    return plan, bufs, pos, cu, scratch


def untouched(bufs, pos, cu):
    return (all(bool((t == POISON).all().item()) for ts in bufs.values() for t in ts)
            and all(bool((t == -2).all().item()) for t in pos) and bool((cu == -2).all().item()))


def check_against_oracle(H, w, fields, slack_rows, seed):
    oplan = oracle_plan(w)
    rng = np.random.default_rng(seed)
    rows = oplan.shard_rows
    cap = [int(r) + int(rng.integers(0, slack_rows + 1)) for r in rows]
    _, shards = H.host_sources(w, fields)
    src_dev = {f.name: [H.to_dev(a) for a in shards[f.name]] for f in fields}
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, cap, src_dev, len(oplan.cu_seqlens) + 5)
    assert H.B.dispatch_async_status(plan) == H.B.EARL_OK
    for f in fields:
        for q in range(oplan.D * oplan.C):
            want = O.dispatch_field_shard(oplan, q, shards[f.name], f.np_dtype, f.width, f.pad_scalar,
                                          per_sequence=f.per_sequence)
            got = bufs[f.name][q].cpu().numpy()
            n = int(rows[q]) * f.row_bytes
            assert np.array_equal(got[:n].view(f.np_dtype).reshape(-1, f.width), want), (f.name, q)
            assert np.all(got[n:] == POISON), (f.name, q, "rows beyond the shard were written")
    for q in range(oplan.D * oplan.C):
        got = pos[q].cpu().numpy()
        assert np.array_equal(got[:int(rows[q])], O.position_ids_shard(oplan, q))
        assert np.all(got[int(rows[q]):] == -2)
    got = cu.cpu().numpy()
    assert np.array_equal(got[:len(oplan.cu_seqlens)], oplan.cu_seqlens)
    assert np.all(got[len(oplan.cu_seqlens):] == -2)
    # the summary is still available afterwards, and a synchronous dispatch agrees
    sm = H.B.plan_get_summary(plan)
    assert sm["shard_rows"].tolist() == rows.tolist()
    H.B.plan_destroy(plan)


FIELDS = (synth.F_ID, synth.F_MASK, synth.bytes_field("wide", 2, 24, 0xBEEF),
          synth.bytes_field("odd", 4, 3, 0x01020304), synth.bytes_field("bf16x64", 2, 64, 0x3F80),
          synth.per_sequence_field("adv", 4, 1, 0x7FC00000))


@pytest.mark.parametrize("slack", [0, 7, 5000])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_async_dispatch_matches_the_oracle(H, seed, slack):
    rng = np.random.default_rng(500 + seed)
    n = int(rng.integers(1, 120))
    w = synth.custom_workload(rng.integers(1, int(rng.choice([20, 900])) + 1, size=n),
                              n_groups=int(rng.choice([1, 3])), replication=int(rng.choice([1, 2])),
                              dp=int(rng.choice([1, 2, 5])), sp=int(rng.choice([1, 2, 4])),
                              zigzag=int(rng.integers(0, 2)), pad_multiple=int(rng.choice([1, 8])),
                              mb_token_budget=4000, fields=FIELDS, seed=seed)
    check_against_oracle(H, w, FIELDS, slack, seed)


@pytest.mark.parametrize("name", ["tiny", "mid", "agentic"])
def test_async_dispatch_on_the_named_workloads(H, name):
    w = synth.make_workload(name, seed=4)
    check_against_oracle(H, w, w.fields, 300, 4)


def test_async_dispatch_with_ranks_that_hold_nothing(H):
    w = synth.custom_workload([5, 9, 2], dp=5, sp=2, zigzag=1, mb_token_budget=100,
                              fields=(synth.F_ID, synth.F_MASK), seed=9)
    check_against_oracle(H, w, w.fields, 40, 9)


def small_setup(H):
    rng = np.random.default_rng(77)
    fields = (synth.F_ID, synth.bytes_field("wide", 2, 24, 0xBEEF))
    w = synth.custom_workload(rng.integers(1, 300, size=60), n_groups=2, dp=2, sp=2, zigzag=1,
                              mb_token_budget=5000, fields=fields, seed=77)
    oplan = oracle_plan(w)
    _, shards = H.host_sources(w, fields)
    src_dev = {f.name: [H.to_dev(a) for a in shards[f.name]] for f in fields}
    return w, fields, oplan, src_dev


def test_async_dispatch_writes_nothing_when_a_buffer_is_too_small(H):
    w, fields, oplan, src_dev = small_setup(H)
    rows = [int(r) for r in oplan.shard_rows]
    # one destination shard one row short
    cap = list(rows)
    cap[2] -= 1
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, cap, src_dev, len(oplan.cu_seqlens))
    assert H.B.dispatch_async_status(plan) == H.B.EARL_CAPACITY
    assert untouched(bufs, pos, cu)
    H.B.plan_destroy(plan)
    # cu_seqlens one entry short
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, rows, src_dev, len(oplan.cu_seqlens) - 1)
    assert H.B.dispatch_async_status(plan) == H.B.EARL_CAPACITY
    assert untouched(bufs, pos, cu)
    H.B.plan_destroy(plan)
    # a source buffer one row short
    short = {k: list(v) for k, v in src_dev.items()}
    short["wide"][1] = short["wide"][1][:-48]
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, rows, short, len(oplan.cu_seqlens))
    assert H.B.dispatch_async_status(plan) == H.B.EARL_CAPACITY
    assert untouched(bufs, pos, cu)
    H.B.plan_destroy(plan)
    # and with everything large enough the same call goes through
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, rows, src_dev, len(oplan.cu_seqlens))
    assert H.B.dispatch_async_status(plan) == H.B.EARL_OK
    assert not untouched(bufs, pos, cu)
    H.B.plan_destroy(plan)


def test_async_dispatch_writes_nothing_when_the_plan_fails(H):
    w, fields, oplan, src_dev = small_setup(H)
    rows = [int(r) + 10 for r in oplan.shard_rows]
    bad = np.array(w.lengths).copy()
    bad[7] = 0
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, rows, src_dev, len(oplan.cu_seqlens) + 4, lengths=bad)
    assert H.B.dispatch_async_status(plan) == H.B.EARL_INVALID_ARG
    assert untouched(bufs, pos, cu)
    with pytest.raises(H.B.EarlError):
        H.B.plan_get_summary(plan)
    H.B.plan_destroy(plan)
    long_ = np.array(w.lengths).copy()
    long_[3] = 6000    # beyond the budget of 5000
    plan, bufs, pos, cu, _ = enqueue(H, w, fields, rows, src_dev, len(oplan.cu_seqlens) + 4, lengths=long_)
    assert H.B.dispatch_async_status(plan) == H.B.EARL_SEQ_EXCEEDS_BUDGET
    assert untouched(bufs, pos, cu)
    H.B.plan_destroy(plan)


def test_async_argument_checks(H):
    import torch
    B = H.B
    w, fields, oplan, src_dev = small_setup(H)
    plan = H.build_plan(w)
    rows = [int(r) for r in oplan.shard_rows]
    dsts = [torch.empty((r * 4,), dtype=torch.uint8, device="cuda") for r in rows]
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.EarlError) as e:   # status before any asynchronous call
        B.dispatch_async_status(plan)
    assert e.value.status == B.EARL_INVALID_ARG
    cnt = torch.zeros(64, dtype=torch.int64, device="cuda")
    cases = [
        B.Field(4, 1, 0, src_dev["token_id"], dsts, nonzero_counts=cnt),
        B.Field(4, 1, 0, src_dev["token_id"], dsts, check_src_capacity=False),
        B.Field(3, 1, 0, src_dev["token_id"], dsts),
        B.Field(4, 1, 0, src_dev["token_id"], [t[1:] for t in dsts]),
    ]
    for fld in cases:
        with pytest.raises(B.EarlError) as e:
            B.dispatch_async(plan, [fld], workspace=ws)
        assert e.value.status == B.EARL_INVALID_ARG
    good = B.Field(4, 1, 0, src_dev["token_id"], dsts)
    with pytest.raises(B.EarlError) as e:
        B.dispatch_async(plan, [good], workspace=ws[:64])
    assert e.value.status == B.EARL_CAPACITY
    B.dispatch_async(plan, [good], workspace=ws)
    assert B.dispatch_async_status(plan) == B.EARL_OK
    want = O.dispatch_field_shard(oplan, 1, [np.asarray(a.cpu().numpy()).view(np.uint32).reshape(-1, 1)
                                            for a in src_dev["token_id"]], np.uint32, 1, 0)
    assert np.array_equal(dsts[1].cpu().numpy().view(np.uint32).reshape(-1, 1), want)
    B.plan_destroy(plan)


def test_async_dispatch_does_not_wait_for_the_stream_with_4096_destination_shards(H):
    """dp = 1024, sp = 4 and six fields (eight with position ids and cu_seqlens): a parameter block
    of some 3 MB, more than one staging slot.  The call must come back while work that was
    enqueued before it is still running (the block goes up in pieces, nothing blocks), and the
    result is still the oracle's."""
    import time
    import torch
    B = H.B
    rng = np.random.default_rng(77)
    fields = tuple(synth.bytes_field(f"f{k}", sb, wd, 0x11 * (k + 1))
                   for k, (sb, wd) in enumerate([(4, 1), (1, 1), (2, 1), (8, 1), (4, 3), (2, 16)]))
    w = synth.custom_workload(rng.integers(1, 40, size=3000), n_groups=4, dp=1024, sp=4, zigzag=1,
                              pad_multiple=1, mb_token_budget=4096, fields=fields, seed=5)
    oplan = oracle_plan(w)
    _, shards = H.host_sources(w, fields)
    src_bufs = {f.name: [H.to_dev(a) for a in shards[f.name]] for f in fields}
    dst_rows = [int(r) for r in oplan.shard_rows]
    # several milliseconds of work in front of the calls
    ballast = torch.empty(1 << 30, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    for _ in range(12):
        ballast.fill_(7)
    t0 = time.perf_counter()
    plan, bufs, pos, cu, scratch = enqueue(H, w, fields, dst_rows, src_bufs, len(oplan.cu_seqlens))
    host_s = time.perf_counter() - t0
    behind = torch.cuda.Event()
    behind.record()
    still_running = not behind.query()
    torch.cuda.synchronize()
    assert still_running, f"the calls took {host_s * 1e3:.1f} ms on the host and the stream was idle after them"
    assert B.dispatch_async_status(plan) == B.EARL_OK
    for q in range(w.dp * w.sp):
        assert np.array_equal(pos[q].cpu().numpy(), O.position_ids_shard(oplan, q)), q
    for f in fields:
        for q in range(0, w.dp * w.sp, 97):
            want = O.dispatch_field_shard(oplan, q, shards[f.name], f.np_dtype, f.width, f.pad_scalar)
            got = bufs[f.name][q].cpu().numpy().view(f.np_dtype).reshape(-1, f.width)
            assert np.array_equal(got, want), (f.name, q)
    assert np.array_equal(cu.cpu().numpy(), oplan.cu_seqlens)
    B.plan_destroy(plan)

"""earl_dispatch_noalloc (the entry point for callers that cannot allocate) against earl_dispatch:
same plan, same fields, bit-identical outputs, on two calls in a row, the second on a smaller
batch (the library's fixed scratch array still holds the first call's contents then)."""
import numpy as np
import pytest
import torch

import gpu_harness as H
from paper_2510_05943_amd import binding as B
from paper_2510_05943_amd import synth

pytestmark = pytest.mark.gpu


def _both_ways(w, count_mask: bool):
    """Dispatches workload w through earl_dispatch and through earl_dispatch_noalloc into
    separate poisoned, guarded buffers and compares every output byte."""
    stream = torch.cuda.current_stream()
    plan = H.build_plan(w, stream=stream)
    sm = B.plan_get_summary(plan)
    n_dst, shard_rows = sm["n_dst_shards"], sm["shard_rows"]
    _, shards = H.host_sources(w, w.fields)
    src_dev = {f.name: [H.to_dev(a) for a in shards[f.name]] for f in w.fields}
    ref = H.run_dispatch(w, plan, w.fields, src_dev=src_dev, stream=stream,
                         count_nonzero=("mask",) if count_mask else ())

    wholes, inner, bfields, counters = {}, {}, [], None
    for f in w.fields:
        pairs = [H.guarded(int(shard_rows[q]) * f.row_bytes) for q in range(n_dst)]
        wholes[f.name] = [p[0] for p in pairs]
        inner[f.name] = [p[1] for p in pairs]
        cnt = None
        if count_mask and f.name == "mask":
            counters = H.guarded(8 * n_dst * sm["n_mb_max"])
            cnt = counters[1].view(torch.int64)
        bfields.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src_dev[f.name], inner[f.name],
                               nonzero_counts=cnt))
    pos = [H.guarded(int(shard_rows[q]) * 4) for q in range(n_dst)]
    cu = H.guarded(sm["cu_seqlens_len"] * 4)
    B.dispatch_noalloc(plan, bfields, position_ids=[p[1] for p in pos], cu_seqlens=cu[1],
                       stream=stream)
    torch.cuda.synchronize()
    for f in w.fields:
        for q in range(n_dst):
            assert H.guards_intact(wholes[f.name][q]), (f.name, q)
            got = inner[f.name][q].cpu().numpy().view(f.np_dtype).reshape(-1, f.width)
            assert np.array_equal(got, ref["fields"][f.name][q]), (f.name, q)
    for q in range(n_dst):
        assert H.guards_intact(pos[q][0])
        assert np.array_equal(pos[q][1].cpu().numpy().view(np.int32), ref["position_ids"][q]), q
    assert H.guards_intact(cu[0])
    assert np.array_equal(cu[1].cpu().numpy().view(np.int32), ref["cu_seqlens"])
    if counters is not None:
        assert H.guards_intact(counters[0])
        got = counters[1].view(torch.int64).cpu().numpy().reshape(n_dst, sm["n_mb_max"])
        assert np.array_equal(got, ref["nonzero_counts"]["mask"])
    B.plan_destroy(plan)


def test_noalloc_matches_dispatch_on_two_calls_in_a_row():
    print("earl_dispatch_noalloc: mid workload (1024 sequences), then 40 sequences of it", flush=True)
    _both_ways(synth.make_workload("mid", seed=1), count_mask=True)
    _both_ways(synth.make_workload("mid", seed=2, scale=40 / 1024), count_mask=False)


def test_noalloc_refuses_what_it_cannot_hold_and_unfetched_plans():
    print("earl_dispatch_noalloc: argument checks", flush=True)
    stream = torch.cuda.current_stream()
    w = synth.make_workload("tiny", seed=0)
    plan = H.build_plan(w, stream=stream)
    f = w.fields[0]
    dummy = torch.zeros(16, dtype=torch.uint8, device="cuda")
    bf = B.Field(f.scalar_bytes, f.width, 0, [dummy] * w.n_shards, [dummy] * (w.dp * w.sp))
    with pytest.raises(B.EarlError) as e:          # summary not fetched yet: nothing may wait here
        B.dispatch_noalloc(plan, [bf], stream=stream)
    assert e.value.status == B.EARL_INVALID_ARG
    sm = B.plan_get_summary(plan)
    with pytest.raises(B.EarlError) as e:          # destination too small: the usual checks apply
        B.dispatch_noalloc(plan, [bf], stream=stream)
    assert e.value.status == B.EARL_CAPACITY
    B.plan_destroy(plan)
    # a batch whose tile codes exceed the fixed array: refused, nothing enqueued
    big = synth.custom_workload(np.full(64, 4096), n_groups=1, replication=1, seq_group=None, dp=1,
                                sp=1, zigzag=0, pad_multiple=1, mb_token_budget=1 << 30,
                                fields=(synth.bytes_field("wide", 2, 32768, 0),), seed=0)
    plan = H.build_plan(big, stream=stream)
    sm = B.plan_get_summary(plan)
    rows = int(sm["shard_rows"][0])
    # 64 * 4096 rows of 64 KiB = 16 GiB of destination: 4 M tile codes = 64 MiB of scratch
    fake = B.Field(2, 32768, 0, [dummy], [dummy])
    fake._rows = lambda t: rows                    # capacities as if the buffers were large enough
    with pytest.raises(B.EarlError) as e:
        B.dispatch_noalloc(plan, [fake], stream=stream)
    assert e.value.status == B.EARL_CAPACITY and "scratch" in str(e.value)
    torch.cuda.synchronize()
    B.plan_destroy(plan)

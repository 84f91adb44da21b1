"""GPU parity at the full size of the two largest workloads, in the launch configuration the
benchmark times (same entry points, same buffers, one earl_dispatch for all fields).

Narrow fields, position ids and cu_seqlens are compared with the oracle element by element.
The wide bf16 field (tens of GB) is checked on every destination shard against the oracle's
per-row source map, with the expected shard assembled on the device by torch indexing, and on
sampled shards against the oracle's own numpy output computed from lazily drawn host rows.
"""
import numpy as np
import pytest

import checkers
from oracle import earl_oracle as O
from paper_2510_05943_amd import synth

pytestmark = pytest.mark.gpu


class LazyRows:
    """Rows of one source shard buffer of the wide field, drawn on the host only when sliced."""

    def __init__(self, w, field, g):
        self.pool = w.hidden_pool(field.width)
        self.index = w.hidden_rows_index(g)

    def __getitem__(self, sl):
        return self.pool[self.index[sl]]


@pytest.mark.parametrize("name", ["heavy", "longctx"])
def test_full_size_parity(name):
    import torch
    import gpu_harness as H
    B = H.B
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    w = synth.make_workload(name, seed=0)
    oplan = O.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                         seq_group=w.seq_group, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                         pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget)
    print(f"[{name}] staging {w.total_tokens} tokens", flush=True)
    src = {f.name: w.device_shard_buffers(f, torch) for f in w.fields}
    plan = H.build_plan(w)
    sm = B.plan_get_summary(plan)
    rows = [int(r) for r in sm["shard_rows"]]
    assert rows == oplan.shard_rows.tolist()
    fields, dsts = [], {}
    for f in w.fields:
        dsts[f.name] = [torch.full((r * f.row_bytes,), 0xCD, dtype=torch.uint8, device="cuda") for r in rows]
        fields.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src[f.name], dsts[f.name]))
    pos = [torch.full((r,), -7, dtype=torch.int32, device="cuda") for r in rows]
    cu = torch.full((sm["cu_seqlens_len"],), -7, dtype=torch.int32, device="cuda")
    scratch = torch.empty(B.dispatch_workspace_bytes(plan, fields), dtype=torch.uint8, device="cuda")
    B.dispatch(plan, fields, position_ids=pos, cu_seqlens=cu, workspace=scratch)
    torch.cuda.synchronize()
    print(f"[{name}] dispatched; checking", flush=True)

    # metadata and narrow fields: everything, element by element
    assert np.array_equal(cu.cpu().numpy(), oplan.cu_seqlens)
    pos_host = [p.cpu().numpy() for p in pos]
    for q in range(len(rows)):
        assert np.array_equal(pos_host[q], O.position_ids_shard(oplan, q)), ("pos", q)
    narrow = [f for f in w.fields if f.kind != "hidden"]
    wide = [f for f in w.fields if f.kind == "hidden"][0]
    host = {f.name: [w.group_buffer(f, s // w.replication) for s in range(w.n_shards)] for f in narrow}
    for f in narrow:
        for q in range(len(rows)):
            want = O.dispatch_field_shard(oplan, q, host[f.name], f.np_dtype, f.width, f.pad_scalar)
            got = dsts[f.name][q].cpu().numpy().view(f.np_dtype).reshape(-1, f.width)
            assert np.array_equal(got, want), (f.name, q)

    # the result explains itself (size-independent properties)
    res = dict(sm)
    res.update(B.plan_export(plan))
    res["position_ids"] = pos_host
    res["cu_seqlens"] = cu.cpu().numpy()
    checkers.check_structure(res, w.lengths, w.dp, w.sp, oplan.K, w.pad_multiple, w.mb_token_budget)

    # wide field, every shard: expected rows gathered on the device from the oracle's row map
    for q in range(len(rows)):
        shard, row = O.source_row_map_shard(oplan, q)
        got = dsts[wide.name][q].view(torch.int16).reshape(-1, wide.width)
        want = torch.full_like(got, wide.pad_scalar)
        shard_t = torch.from_numpy(shard).cuda()
        row_t = torch.from_numpy(row).cuda()
        for s in range(w.n_shards):
            sel = torch.nonzero(shard_t == s).squeeze(1)
            if sel.numel():
                want[sel] = src[wide.name][s].index_select(0, row_t[sel])
        assert torch.equal(got, want), (wide.name, q)
        del want, got, shard_t, row_t
    print(f"[{name}] wide field: all {len(rows)} shards match the row map", flush=True)

    # wide field, sampled shards: the oracle's own output from host-drawn rows
    lazy = [LazyRows(w, wide, s // w.replication) for s in range(w.n_shards)]
    for q in sorted({0, len(rows) // 2 + 1, len(rows) - 1}):
        want = O.dispatch_field_shard(oplan, q, lazy, wide.np_dtype, wide.width, wide.pad_scalar)
        got = dsts[wide.name][q].cpu().numpy().view(wide.np_dtype).reshape(-1, wide.width)
        assert np.array_equal(got, want), (wide.name, q)

    # reverse direction at full size: every source row is read by the plan here (no replicas),
    # so the round trip must give back the source buffers bit for bit
    back = {f.name: [torch.full_like(t, 0x5A) for t in src[f.name]] for f in w.fields}
    inv_fields = [B.Field(f.scalar_bytes, f.width, f.pad_scalar, back[f.name], dsts[f.name])
                  for f in w.fields]
    B.dispatch_inverse(plan, inv_fields, workspace=scratch)
    torch.cuda.synchronize()
    for f in w.fields:
        for s in range(w.n_shards):
            assert torch.equal(back[f.name][s], src[f.name][s]), (f.name, s)
    print(f"[{name}] inverse: round trip restores all source shards", flush=True)
    B.plan_destroy(plan)


def test_buffers_beyond_4_gib():
    """One source buffer and one destination shard of more than 4 GiB each: every byte offset
    inside a buffer has to be computed in 64 bits."""
    import torch
    import gpu_harness as H
    B = H.B
    wide = synth.FieldSpec("hidden_bf16", 2, 1024, 0, "hidden")
    lengths = [36000 + 997 * (i % 7) for i in range(64)]            # 2.49 M rows of 2 KiB = 5.1 GB
    w = synth.custom_workload(lengths, n_groups=1, dp=1, sp=1, zigzag=0, pad_multiple=8,
                              mb_token_budget=1 << 30, fields=(synth.F_ID, wide), seed=3)
    oplan = O.build_plan(w.lengths, n_groups=1, dp=1, sp=1, zigzag=0, pad_multiple=8,
                         mb_token_budget=1 << 30)
    src = {f.name: w.device_shard_buffers(f, torch) for f in w.fields}
    assert src[wide.name][0].numel() * 2 > (4 << 30)
    plan = H.build_plan(w)
    sm = B.plan_get_summary(plan)
    rows = [int(r) for r in sm["shard_rows"]]
    assert rows == oplan.shard_rows.tolist() and rows[0] * wide.row_bytes > (4 << 30)
    dsts = {f.name: [torch.full((r * f.row_bytes,), 0xCD, dtype=torch.uint8, device="cuda") for r in rows]
            for f in w.fields}
    fields = [B.Field(f.scalar_bytes, f.width, f.pad_scalar, src[f.name], dsts[f.name]) for f in w.fields]
    scratch = torch.empty(B.dispatch_workspace_bytes(plan, fields, False, False), dtype=torch.uint8,
                          device="cuda")
    B.dispatch(plan, fields, workspace=scratch)
    torch.cuda.synchronize()
    for q in range(len(rows)):
        shard, row = O.source_row_map_shard(oplan, q)
        got = dsts[wide.name][q].view(torch.int16).reshape(-1, wide.width)
        want = torch.full_like(got, 0)
        sel = torch.from_numpy(np.nonzero(shard == 0)[0]).cuda()
        want[sel] = src[wide.name][0].index_select(0, torch.from_numpy(row[shard == 0]).cuda())
        assert torch.equal(got, want), q
        del want
    # and back: the 5 GB source buffer is restored bit for bit
    back = {f.name: [torch.full_like(t, 0x5A) for t in src[f.name]] for f in w.fields}
    inv = [B.Field(f.scalar_bytes, f.width, f.pad_scalar, back[f.name], dsts[f.name]) for f in w.fields]
    B.dispatch_inverse(plan, inv, workspace=scratch)
    torch.cuda.synchronize()
    for f in w.fields:
        assert torch.equal(back[f.name][0], src[f.name][0]), f.name
    B.plan_destroy(plan)


def test_plan_and_dispatch_at_the_maximum_sequence_count():
    """N = 2^20 sequences (the library's limit), short lengths, many micro-batches per rank: the
    plan against the oracle array by array, then one 4-byte field, position ids and cu_seqlens
    against the oracle's dispatch."""
    import torch
    import gpu_harness as H
    import test_gpu_parity as T
    n = 1 << 20
    lengths = np.random.default_rng(77).integers(1, 17, size=n)
    w = synth.custom_workload(lengths, n_groups=8, dp=8, sp=1, zigzag=0, pad_multiple=1,
                              mb_token_budget=4096, fields=(synth.F_ID,), seed=77)
    print("[max N] oracle plan", flush=True)
    oplan = T.oracle_plan(w)
    print("[max N] GPU plan", flush=True)
    plan = H.build_plan(w)
    T.assert_plan_equal(H.plan_result(plan), oplan)
    print("[max N] dispatch", flush=True)
    _, shards = H.host_sources(w, w.fields)
    out = H.run_dispatch(w, plan, w.fields, src_host=shards)
    T.assert_dispatch_equal(w, oplan, out, shards, w.fields)
    H.B.plan_destroy(plan)
    torch.cuda.synchronize()

"""Stages a synthetic workload into GPU memory, runs the library through the binding and
returns everything it produced as numpy arrays.  Used by the GPU parity tests only."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from paper_2510_05943_amd import binding as B
from paper_2510_05943_amd import synth

CANARY = 256          # guard bytes on both sides of every destination buffer
POISON = 0xCD

_TORCH_INT = {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Host array -> device tensor with the same bytes."""
    a = np.ascontiguousarray(a)
    signed = {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[a.dtype.itemsize]
    return torch.from_numpy(a.view(signed)).cuda()


def guarded(nbytes: int):
    """A destination buffer of nbytes with poisoned guard zones; returns (whole, interior)."""
    whole = torch.full((nbytes + 2 * CANARY,), POISON, dtype=torch.uint8, device="cuda")
    return whole, whole[CANARY:CANARY + nbytes]


def guards_intact(whole: torch.Tensor) -> bool:
    return bool((whole[:CANARY] == POISON).all().item() and (whole[-CANARY:] == POISON).all().item())


def layouts_of(w: synth.Workload, explicit_groups: bool, seq_row=None, balance_policy: int = 0,
               equal_mb: int = 0):
    contiguous = (np.arange(w.n_seqs, dtype=np.int64) * w.n_groups) // max(w.n_seqs, 1)
    keep = []
    grp = None
    if explicit_groups or not np.array_equal(contiguous, w.seq_group):
        grp = to_dev(w.seq_group.astype(np.int32))
        keep.append(grp)
    row = None
    if seq_row is not None:
        row = to_dev(np.asarray(seq_row, np.int64))
        keep.append(row)
    src = B.SrcLayout(w.n_groups, w.replication, grp, row)
    dst = B.DstLayout(w.dp, w.sp, w.zigzag, w.pad_multiple, w.mb_token_budget, balance_policy,
                      equal_mb)
    return src, dst, keep


def build_plan(w: synth.Workload, explicit_groups: bool = False, seq_row=None, stream=None,
               balance_policy: int = 0, equal_mb: int = 0):
    src, dst, keep = layouts_of(w, explicit_groups, seq_row, balance_policy, equal_mb)
    lengths = to_dev(w.lengths.astype(np.int32))
    ws = torch.empty(B.plan_workspace_bytes(w.n_seqs, src, dst), dtype=torch.uint8, device="cuda")
    plan = B.plan_build(lengths, w.n_seqs, src, dst, ws, stream=stream)
    plan.keepalive = plan.keepalive + tuple(keep)
    return plan


def plan_result(plan) -> Dict:
    res = B.plan_get_summary(plan)
    res.update(B.plan_export(plan))
    res["segments"] = B.plan_export_segments(plan)
    return res


def run_dispatch(w: synth.Workload, plan, fields: Sequence[synth.FieldSpec],
                 src_host: Optional[Dict[str, List[np.ndarray]]] = None,
                 src_dev: Optional[Dict[str, List[torch.Tensor]]] = None,
                 want_position_ids: bool = True, want_cu: bool = True, stream=None,
                 count_nonzero: Sequence[str] = ()) -> Dict:
    """Runs earl_dispatch for `fields`.  src_host[name][s] / src_dev[name][s] = shard buffer s.
    Fields named in count_nonzero also get a (poisoned, guarded) non-zero counter array."""
    sm = B.plan_get_summary(plan)
    n_dst = sm["n_dst_shards"]
    shard_rows = sm["shard_rows"]
    bfields, wholes, inner, keep = [], {}, {}, []
    counters = {}
    for f in fields:
        if src_dev is not None and f.name in src_dev:
            srcs = src_dev[f.name]
        else:
            srcs = [to_dev(a) if a is not None else None for a in src_host[f.name]]
        keep.append(srcs)
        pairs = [guarded(int(shard_rows[q]) * f.row_bytes) for q in range(n_dst)]
        wholes[f.name] = [p[0] for p in pairs]
        inner[f.name] = [p[1] for p in pairs]
        cnt = None
        if f.name in count_nonzero:
            counters[f.name] = guarded(8 * n_dst * sm["n_mb_max"])
            cnt = counters[f.name][1].view(torch.int64)
        bfields.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, srcs, inner[f.name],
                               per_sequence=f.per_sequence, nonzero_counts=cnt))
    pos_pairs = [guarded(int(shard_rows[q]) * 4) for q in range(n_dst)] if want_position_ids else None
    cu_pair = guarded(sm["cu_seqlens_len"] * 4) if want_cu else None
    ws_whole, ws = guarded(B.dispatch_workspace_bytes(plan, bfields, want_position_ids, want_cu))
    B.dispatch(plan, bfields,
               position_ids=[p[1] for p in pos_pairs] if pos_pairs else None,
               cu_seqlens=cu_pair[1] if cu_pair else None, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    assert guards_intact(ws_whole), "write outside the dispatch scratch"
    out = {"fields": {}, "dev": inner, "src_dev": {f.name: s for f, s in zip(fields, keep)},
           "workspace": ws}
    for f in fields:
        assert all(guards_intact(x) for x in wholes[f.name]), f"{f.name}: write outside its shard"
        out["fields"][f.name] = [
            t.cpu().numpy().view(f.np_dtype).reshape(-1, f.width) for t in inner[f.name]]
    if counters:
        out["nonzero_counts"] = {}
        for name, (whole, inside) in counters.items():
            assert guards_intact(whole), f"{name}: write outside its counters"
            out["nonzero_counts"][name] = inside.view(torch.int64).cpu().numpy().reshape(
                n_dst, sm["n_mb_max"])
    if pos_pairs:
        assert all(guards_intact(p[0]) for p in pos_pairs)
        out["position_ids"] = [p[1].cpu().numpy().view(np.int32) for p in pos_pairs]
    if cu_pair:
        assert guards_intact(cu_pair[0])
        out["cu_seqlens"] = cu_pair[1].cpu().numpy().view(np.int32)
    return out


def host_sources(w: synth.Workload, fields: Sequence[synth.FieldSpec]):
    """Per field: (group buffers, shard buffers) on the host; replicas share the group's array."""
    groups = {f.name: [w.group_buffer(f, g) for g in range(w.n_groups)] for f in fields}
    shards = {n: [g[s // w.replication] for s in range(w.n_shards)] for n, g in groups.items()}
    return groups, shards

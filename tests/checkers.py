"""Checks that read a dispatch result through its own metadata only.

Nothing here calls the oracle or the GPU library: given the exported flat arrays
(`seq_ids`, `mb_seq_start`, `mb_row_start`, `cu_seqlens`), the per-shard `position_ids` and the
destination shards of a field, every destination row is traced back to its (sequence,
position) and compared with the source bytes.  The same functions check the oracle (as a pin)
and the GPU path (as a size-independent property).
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np


def packed_source_rows(L, seq_group, n_groups):
    """Row offset of every sequence inside its group's packed buffer (plain cumsum per group)."""
    L = np.asarray(L, np.int64)
    seq_group = np.asarray(seq_group)
    row = np.zeros(len(L), np.int64)
    for g in range(n_groups):
        idx = np.nonzero(seq_group == g)[0]
        row[idx] = np.cumsum(L[idx]) - L[idx]
    return row


def trace_rows(res: Dict, D: int, C: int):
    """Recover (sequence, position) of every destination row from the metadata alone.

    res holds n_seq[D], n_mb[D], seq_ids, mb_seq_start, mb_row_start, cu_seqlens (flat forms)
    and position_ids (list of D*C int32 arrays).  Returns per shard q: (seq_of_row, pos_of_row).
    """
    n_seq = np.asarray(res["n_seq"], np.int64)
    n_mb = np.asarray(res["n_mb"], np.int64)
    seq_ids = np.asarray(res["seq_ids"])
    mb_seq_start = np.asarray(res["mb_seq_start"])
    mb_row_start = np.asarray(res["mb_row_start"])
    cu = np.asarray(res["cu_seqlens"])
    out = []
    for r in range(D):
        ids_base = int(n_seq[:r].sum())
        mbs_base = int((n_mb[:r] + 1).sum())
        cu_base = int((n_seq[:r] + n_mb[:r]).sum())
        for c in range(C):
            q = r * C + c
            pos = np.asarray(res["position_ids"][q])
            seq_of_row = np.full(pos.shape, -1, np.int64)
            for b in range(int(n_mb[r])):
                s0 = int(mb_seq_start[mbs_base + b])
                s1 = int(mb_seq_start[mbs_base + b + 1])
                row0 = int(mb_row_start[mbs_base + b])
                cu_b = cu[cu_base + s0 + b: cu_base + s1 + b + 1]
                assert cu_b[0] == 0
                assert np.all(np.diff(cu_b) > 0), "cu_seqlens must be strictly increasing"
                assert row0 + int(cu_b[-1]) == int(mb_row_start[mbs_base + b + 1])
                for k, s in enumerate(range(s0, s1)):
                    seq_of_row[row0 + int(cu_b[k]): row0 + int(cu_b[k + 1])] = seq_ids[ids_base + s]
            assert np.all(seq_of_row >= 0), "a destination row belongs to no sequence"
            out.append((seq_of_row, pos.astype(np.int64)))
    return out


def padding_rows_of_shard(res: Dict, L, D: int, C: int, q: int) -> np.ndarray:
    """Boolean mask over the rows of destination shard q: True where the row is padding (its
    traced-back position lies at or beyond the real length of its sequence)."""
    seq_of_row, pos = trace_rows(res, D, C)[q]
    return pos >= np.asarray(L, np.int64)[seq_of_row]


def check_self_describing(res: Dict, L, D: int, C: int, src_group_bufs: Sequence[np.ndarray],
                          seq_group, src_row, dst_shards: Sequence[np.ndarray], pad_row) -> None:
    """Every destination row equals source(i, p) when p < L[i] and the pad row otherwise; every
    real (i, p) occurs exactly once over all shards (token conservation)."""
    L = np.asarray(L, np.int64)
    seen = [np.zeros(int(x), np.int32) for x in L]
    traced = trace_rows(res, D, C)
    for q, (seq_of_row, pos) in enumerate(traced):
        dst = np.asarray(dst_shards[q])
        assert dst.shape[0] == seq_of_row.shape[0]
        for row in range(dst.shape[0]):
            i, p = int(seq_of_row[row]), int(pos[row])
            assert p >= 0
            if p < L[i]:
                want = src_group_bufs[int(seq_group[i])][int(src_row[i]) + p]
                seen[i][p] += 1
            else:
                want = pad_row
            assert np.array_equal(dst[row], want), (q, row, i, p)
    for i, s in enumerate(seen):
        assert np.all(s == 1), f"sequence {i}: some token not delivered exactly once"


def check_self_describing_fast(res: Dict, L, D: int, C: int, src_group_bufs, seq_group, src_row,
                               dst_shards, pad_row) -> None:
    """Vectorised form of check_self_describing for large batches (same assertions)."""
    L = np.asarray(L, np.int64)
    seq_group = np.asarray(seq_group)
    src_row = np.asarray(src_row, np.int64)
    starts = np.cumsum(L) - L
    seen = np.zeros(int(L.sum()), np.int32)
    n_groups = len(src_group_bufs)
    for q, (seq_of_row, pos) in enumerate(trace_rows(res, D, C)):
        dst = np.asarray(dst_shards[q])
        assert dst.shape[0] == seq_of_row.shape[0]
        real = pos < L[seq_of_row]
        assert np.all(pos >= 0)
        assert np.all(dst[~real] == pad_row), f"shard {q}: padding row is not the pad value"
        ri, rp = seq_of_row[real], pos[real]
        np.add.at(seen, starts[ri] + rp, 1)
        got = dst[real]
        grp = seq_group[ri]
        for g in range(n_groups):
            sel = grp == g
            if sel.any():
                want = np.asarray(src_group_bufs[g])[src_row[ri[sel]] + rp[sel]]
                assert np.array_equal(got[sel], want), f"shard {q}: wrong row from group {g}"
    assert np.all(seen == 1), "some token not delivered exactly once"


def check_structure(res: Dict, L, D: int, C: int, K: int, P: int, B: int) -> None:
    """Invariants that hold for any batch: next-fit micro-batches, equal shards over SP ranks,
    P-aligned offsets, zigzag causal balance, a2a row/column sums, list-scheduling bounds."""
    L = np.asarray(L, np.int64)
    N = len(L)
    n_seq = np.asarray(res["n_seq"], np.int64)
    n_mb = np.asarray(res["n_mb"], np.int64)
    rank = np.asarray(res["rank"])
    seq_ids = np.asarray(res["seq_ids"])
    shard_rows = np.asarray(res["shard_rows"], np.int64)
    dst_row = np.asarray(res["dst_row"], np.int64)
    assert n_seq.sum() == N and sorted(seq_ids.tolist()) == list(range(N))
    assert np.array_equal(np.bincount(rank, minlength=D), n_seq)
    traced = trace_rows(res, D, C)
    # per-sequence rows on each SP rank
    loc = np.zeros(N, np.int64)
    for r in range(D):
        for c in range(C):
            q = r * C + c
            seq_of_row, pos = traced[q]
            assert shard_rows[q] == shard_rows[r * C], "SP ranks of one DP rank differ in rows"
            cnt = np.bincount(seq_of_row, minlength=N)
            if c == 0:
                loc += cnt
            else:
                assert np.array_equal(cnt[rank == r], loc[rank == r])
            if K == 2 * C and C > 1:
                # causal balance: the sum of positions held is the same on every SP rank
                sums = np.bincount(seq_of_row, weights=pos.astype(np.float64), minlength=N)
                m = loc // 2
                want = (m * m * (2 * C - 1) + m * (m - 1)).astype(np.float64)
                sel = rank == r
                assert np.array_equal(sums[sel], want[sel]), "zigzag halves are not balanced"
    Lp = loc * C
    m_all = Lp // K
    assert np.all(Lp % K == 0) and np.all(m_all % P == 0), "chunk length is not a multiple of P"
    assert np.all(Lp >= L) and np.all(K * (m_all - P) < L), "chunk length is not the smallest that fits"
    assert np.all(dst_row % P == 0)
    assert np.all(Lp <= B)
    # next-fit along ascending index inside a rank
    ids_base = 0
    mbs_base = 0
    mb_seq_start = np.asarray(res["mb_seq_start"])
    for r in range(D):
        ids = seq_ids[ids_base: ids_base + n_seq[r]]
        assert np.all(np.diff(ids) > 0), "rank order is not ascending index"
        for b in range(int(n_mb[r])):
            s0, s1 = int(mb_seq_start[mbs_base + b]), int(mb_seq_start[mbs_base + b + 1])
            tot = int(Lp[ids[s0:s1]].sum())
            assert s1 > s0 and tot <= B
            if s1 < n_seq[r]:
                assert tot + int(Lp[ids[s1]]) > B, "micro-batch closed although the next fits"
        assert int(mb_seq_start[mbs_base + n_mb[r]]) == n_seq[r]
        ids_base += int(n_seq[r])
        mbs_base += int(n_mb[r]) + 1
    # list-scheduling bounds
    load = np.bincount(rank, weights=Lp.astype(np.float64), minlength=D)
    if N >= D:
        assert load.max() - load.min() <= Lp.max()
    assert load.max() <= Lp.sum() / D + (1 - 1 / D) * Lp.max() + 1e-9
    # a2a counts
    a2a = np.asarray(res["a2a_counts"], np.int64)
    assert a2a.sum() == L.sum()
    if "seq_shard" in res:
        S = a2a.shape[0]
        assert np.array_equal(a2a.sum(axis=1),
                              np.bincount(res["seq_shard"], weights=L.astype(np.float64),
                                          minlength=S).astype(np.int64))
    for q, (seq_of_row, pos) in enumerate(traced):
        assert a2a[:, q].sum() == int((pos < L[seq_of_row]).sum())

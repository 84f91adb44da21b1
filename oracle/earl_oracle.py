"""CPU oracle for the layout-aware re-layout of intermediate rollout batches.

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the GPU library is
compared against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does, and this file imports nothing from the product.

What it follows.  The paper (Section 2, "Data Dispatcher") states the operation only in words:
intermediate batches (tokens, log-probabilities, rewards, returns, other tensors; Section 1)
are sent from the workers that computed them straight to the training workers that need
them, according to the current data layout and the target parallelism configuration, as an
all-to-all instead of a gather on one node followed by a scatter.  It gives no algorithm,
equation or worked example.  The concrete rules below (how sequences are balanced over
data-parallel ranks, how a sequence is cut over sequence-parallel ranks, padding, micro-batch
limits, metadata) are therefore this project's stated reading of that passage; each function
says which part of the reading it implements, and every rule is integer-only, so exactly one
result is correct.

Because the paper prints no example, parity against the paper itself is unpinned.  The
functions here are pinned instead by closed forms, hand-worked cases, brute force on tiny
inputs, invariants and library special cases (tests/test_oracle_pins.py).

Notation: N sequences, L[i] >= 1 real tokens ("rows"); G source groups, each stored as R
identical replica buffers (S = G*R shard buffers per field); D data-parallel ranks, C
sequence-parallel ranks, zigzag flag z, pad multiple P, micro-batch token budget B;
destination shard q = r*C + c.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence

import numpy as np

OK = 0
INVALID_ARG = 1
SEQ_EXCEEDS_BUDGET = 2
CAPACITY = 3


class OracleError(Exception):
    def __init__(self, status: int, msg: str = ""):
        super().__init__(f"status {status}: {msg}")
        self.status = status


# ----------------------------------------------------------------------------------------
# Source layout (where each sequence is read from)
# ----------------------------------------------------------------------------------------
def source_layout(L, n_groups: int, replication: int, seq_group=None, seq_row=None):
    """Origin of every sequence ("from their computation origins", Section 2).

    Group g's buffers hold the sequences with seq_group[i] == g.  With seq_group None, groups
    own equal contiguous index ranges: g = floor(i*G/N).  With seq_row None the sequences of
    a group are packed in index order, so seq_row[i] is the exclusive prefix sum of L over
    the group's earlier members.  Each group exists as R identical replicas (the outputs of
    a tensor-parallel rollout group); to read every row exactly once and spread the reads,
    the k-th of the n_g members of a group is read from replica t = floor(k*R/n_g), i.e.
    shard buffer g*R + t.

    Returns (seq_group, seq_shard, seq_row, group_rows, seq_k) where group_rows[g] is the number
    of rows the packed buffers of group g hold (sum of its members' L) and seq_k[i] says that
    sequence i is the k-th member of its group (the row of a per-sequence field).
    """
    L = [int(x) for x in L]
    N = len(L)
    G, R = int(n_groups), int(replication)
    if N < 1 or G < 1 or R < 1:
        raise OracleError(INVALID_ARG, "N, G, R must be >= 1")
    if seq_group is None:
        seq_group = [(i * G) // N for i in range(N)]
    seq_group = [int(g) for g in seq_group]
    if any(g < 0 or g >= G for g in seq_group):
        raise OracleError(INVALID_ARG, "seq_group out of range")
    members = [[i for i in range(N) if seq_group[i] == g] for g in range(G)]
    seq_shard = [0] * N
    seq_k = [0] * N
    packed_row = [0] * N
    group_rows = [0] * G
    for g in range(G):
        n_g = len(members[g])
        acc = 0
        for k, i in enumerate(members[g]):
            seq_shard[i] = g * R + (k * R) // n_g
            seq_k[i] = k
            packed_row[i] = acc
            acc += L[i]
        group_rows[g] = acc
    if seq_row is None:
        seq_row = packed_row
    else:
        seq_row = [int(x) for x in seq_row]
        if any(x < 0 for x in seq_row):
            raise OracleError(INVALID_ARG, "negative seq_row")
    return (np.array(seq_group, np.int32), np.array(seq_shard, np.int32),
            np.array(seq_row, np.int64), np.array(group_rows, np.int64), np.array(seq_k, np.int32))


# ----------------------------------------------------------------------------------------
# Padded geometry
# ----------------------------------------------------------------------------------------
def padded_geometry(L, C: int, zigzag: int, P: int):
    """Chunk count K, chunk length m[i], padded length Lp[i] and rows per SP rank loc[i].

    A sequence is cut into K equal chunks, K = 2C for zigzag with C > 1, else C.  Each chunk
    is as long as the smallest multiple of P that lets K chunks cover the sequence:
    m = P*ceil(ceil(L/K)/P).  Lp = K*m; positions L..Lp-1 are padding at the logical end.
    Every SP rank holds loc = Lp/C rows of the sequence.
    """
    C, P = int(C), int(P)
    K = 2 * C if (zigzag and C > 1) else C
    m, Lp, loc = [], [], []
    for x in L:
        x = int(x)
        per_chunk = -(-x // K)
        mi = P * (-(-per_chunk // P))
        m.append(mi)
        Lp.append(K * mi)
        loc.append(K * mi // C)
    return K, np.array(m, np.int64), np.array(Lp, np.int64), np.array(loc, np.int64)


# ----------------------------------------------------------------------------------------
# Rank assignment
# ----------------------------------------------------------------------------------------
def lpt_ranks(Lp, D: int, quadratic: bool = False):
    """Length-balanced assignment of sequences to the D data-parallel ranks.

    Longest-processing-time list scheduling (Graham 1969): visit sequences by padded length,
    longest first (equal lengths: lower index first); give each to the rank whose load is
    smallest so far (equal loads: lower rank); its load grows by the sequence's cost.  The cost
    is the padded length (balance_policy 0: equal token counts) or its square (balance_policy
    2: equal causal-attention work, which grows with the square of the length).  Returns the
    ranks and the per-rank sums of the cost.
    """
    N = len(Lp)
    order = sorted(range(N), key=lambda i: (-int(Lp[i]), i))
    load = [0] * D
    rank = [0] * N
    for i in order:
        r = min(range(D), key=lambda d: (load[d], d))
        rank[i] = r
        load[r] += int(Lp[i]) ** 2 if quadratic else int(Lp[i])
    return np.array(rank, np.int32), np.array(load, dtype=object if quadratic else np.int64)


def snake_ranks(Lp, D: int):
    """Alternative balancing without a serial chain (balance_policy 1): visit sequences longest
    first (equal lengths: lower index first) and deal them to the ranks in rounds of D, left to
    right in even rounds and right to left in odd rounds, so that the rank that got the longest
    sequence of one round gets the shortest of the next."""
    N = len(Lp)
    order = sorted(range(N), key=lambda i: (-int(Lp[i]), i))
    load = [0] * D
    rank = [0] * N
    for j, i in enumerate(order):
        t, k = divmod(j, D)
        r = k if t % 2 == 0 else D - 1 - k
        rank[i] = r
        load[r] += int(Lp[i])
    return np.array(rank, np.int32), np.array(load, np.int64)


# ----------------------------------------------------------------------------------------
# Packing order, micro-batches, destination offsets
# ----------------------------------------------------------------------------------------
def pack_ranks(rank, Lp, loc, D: int, B: int, equal_mb: bool = False):
    """Order inside a rank, micro-batch of every sequence, destination row offsets.

    Inside a rank sequences keep ascending original index.  Micro-batches are cut next-fit
    along that order: a sequence opens a new micro-batch when the current one is non-empty
    and adding the sequence's padded length would exceed the budget B (B counts padded tokens
    of whole sequences on the DP rank, before the split over SP ranks).  Rows of a rank's
    shards are consecutive over all its sequences, so micro-batches are consecutive row
    ranges; dst_row[i] is the sum of loc over the sequences packed before i in its rank.
    With equal_mb every rank reports as many micro-batches as the rank that has most: the
    missing ones are appended empty (no sequence, no row), so that all data-parallel ranks run
    the same number of steps.
    """
    N = len(rank)
    slot = [0] * N
    mb = [0] * N
    dst_row = [0] * N
    n_seq = [0] * D
    n_mb = [0] * D
    rows = [0] * D
    seq_ids: List[List[int]] = [[] for _ in range(D)]
    mb_seq_start: List[List[int]] = [[] for _ in range(D)]
    mb_row_start: List[List[int]] = [[] for _ in range(D)]
    cur = [0] * D
    for i in range(N):
        r = int(rank[i])
        if len(seq_ids[r]) == 0 or (cur[r] > 0 and cur[r] + int(Lp[i]) > B):
            mb_seq_start[r].append(len(seq_ids[r]))
            mb_row_start[r].append(rows[r])
            cur[r] = 0
        mb[i] = len(mb_seq_start[r]) - 1
        slot[i] = len(seq_ids[r])
        dst_row[i] = rows[r]
        seq_ids[r].append(i)
        cur[r] += int(Lp[i])
        rows[r] += int(loc[i])
    most = max(len(mb_seq_start[r]) for r in range(D))
    for r in range(D):
        n_seq[r] = len(seq_ids[r])
        n_mb[r] = len(mb_seq_start[r])
        mb_seq_start[r].append(n_seq[r])
        mb_row_start[r].append(rows[r])
        while equal_mb and n_mb[r] < most:
            n_mb[r] += 1
            mb_seq_start[r].append(n_seq[r])
            mb_row_start[r].append(rows[r])
    return dict(slot=np.array(slot, np.int32), mb=np.array(mb, np.int32),
                dst_row=np.array(dst_row, np.int64), n_seq=np.array(n_seq, np.int32),
                n_mb=np.array(n_mb, np.int32), rank_rows=np.array(rows, np.int64),
                seq_ids=seq_ids, mb_seq_start=mb_seq_start, mb_row_start=mb_row_start)


# ----------------------------------------------------------------------------------------
# Chunk -> sequence-parallel rank
# ----------------------------------------------------------------------------------------
def chunk_to_sp(kappa: int, C: int, K: int):
    """SP rank c and local half h of chunk kappa.

    Contiguous split (K == C): chunk kappa goes to SP rank kappa.  Zigzag (K == 2C): SP rank c
    holds chunk c followed by chunk 2C-1-c, pairing an early with a late chunk so that causal
    attention work is equal over SP ranks; h = 1 marks the second (mirrored) chunk.
    """
    if K == C:
        return kappa, 0
    if kappa < C:
        return kappa, 0
    return 2 * C - 1 - kappa, 1


# ----------------------------------------------------------------------------------------
# The plan
# ----------------------------------------------------------------------------------------
@dataclasses.dataclass
class Plan:
    N: int
    S: int
    D: int
    C: int
    K: int
    P: int
    B: int
    L: np.ndarray
    m: np.ndarray
    Lp: np.ndarray
    loc: np.ndarray
    seq_group: np.ndarray
    seq_shard: np.ndarray
    seq_row: np.ndarray
    seq_k: np.ndarray
    group_rows: np.ndarray
    rank: np.ndarray
    rank_load: np.ndarray
    slot: np.ndarray
    mb: np.ndarray
    dst_row: np.ndarray
    n_seq: np.ndarray
    n_mb: np.ndarray
    shard_rows: np.ndarray          # int64[D*C]
    seq_ids: np.ndarray             # int32[N], rank-major
    mb_seq_start: np.ndarray        # int32[sum(n_mb)+D]
    mb_row_start: np.ndarray        # int64[sum(n_mb)+D]
    cu_seqlens: np.ndarray          # int32[N + sum(n_mb)]
    a2a_counts: np.ndarray          # int64[S, D*C]
    # segment table, ordered by (destination shard, destination row)
    seg_src_shard: np.ndarray
    seg_src_row: np.ndarray
    seg_dst_shard: np.ndarray
    seg_dst_row: np.ndarray
    seg_n_real: np.ndarray
    seg_n_rows: np.ndarray
    seg_pos0: np.ndarray
    seg_seq: np.ndarray
    shard_seg_start: np.ndarray     # int32[D*C+1]

    @property
    def total_real_rows(self) -> int:
        return int(self.L.astype(np.int64).sum())

    @property
    def total_dst_rows(self) -> int:
        return int(self.shard_rows.sum())


def build_plan(L, *, n_groups: int, replication: int = 1, seq_group=None, seq_row=None,
               dp: int, sp: int, zigzag: int, pad_multiple: int, mb_token_budget: int,
               balance_policy: int = 0, equal_mb: int = 0) -> Plan:
    """The dispatch plan: for every sequence, where it is read and where each part is written.

    This is the "parallelism- and layout-aware" decision of Section 2 made explicit.  The
    steps, in order: source layout; padded geometry (a sequence whose padded length exceeds
    the budget is an error and nothing is planned); rank assignment; packing; then one
    segment per (sequence, chunk), a run of m rows that is contiguous in both layouts, of
    which the first n_real are copied and the rest are padding.  a2a_counts[s][q] counts the
    real rows read from shard buffer s and written to destination shard q: the split sizes
    the all-to-all of Section 2 would use.
    """
    L = np.asarray(L)
    N = int(L.shape[0])
    D, C, P, B = int(dp), int(sp), int(pad_multiple), int(mb_token_budget)
    if N < 1 or D < 1 or C < 1 or P < 1 or B < 1:
        raise OracleError(INVALID_ARG, "N, dp, sp, pad_multiple, budget must be >= 1")
    if any(int(x) < 1 for x in L):
        raise OracleError(INVALID_ARG, "every length must be >= 1")
    grp, seq_shard, srow, group_rows, seq_k = source_layout(L, n_groups, replication, seq_group,
                                                            seq_row)
    S = int(n_groups) * int(replication)
    K, m, Lp, loc = padded_geometry(L, C, zigzag, P)
    if any(int(x) > B for x in Lp):
        raise OracleError(SEQ_EXCEEDS_BUDGET, "a padded sequence is longer than the budget")
    if balance_policy not in (0, 1, 2) or equal_mb not in (0, 1):
        raise OracleError(INVALID_ARG, "unknown balance_policy or equal_mb")
    if balance_policy == 1:
        rank, _ = snake_ranks(Lp, D)
    else:
        rank, _ = lpt_ranks(Lp, D, quadratic=(balance_policy == 2))
    # reported load of a rank: its padded tokens, whatever cost the policy balanced
    load = np.zeros((D,), np.int64)
    np.add.at(load, rank, np.asarray(Lp, np.int64))
    pk = pack_ranks(rank, Lp, loc, D, B, equal_mb=bool(equal_mb))

    shard_rows = np.repeat(pk["rank_rows"], C).astype(np.int64)

    # flat exported forms
    seq_ids = np.array([i for r in range(D) for i in pk["seq_ids"][r]], np.int32)
    mb_seq_start = np.array([x for r in range(D) for x in pk["mb_seq_start"][r]], np.int32)
    mb_row_start = np.array([x for r in range(D) for x in pk["mb_row_start"][r]], np.int64)

    # cu_seqlens: local rows, restarting at 0 in every micro-batch; one array of n+1 entries
    # per micro-batch, micro-batches of a rank one after the other, ranks one after the other.
    cu: List[int] = []
    for r in range(D):
        ids = pk["seq_ids"][r]
        starts = pk["mb_seq_start"][r]
        for b in range(int(pk["n_mb"][r])):
            acc = 0
            cu.append(0)
            for s in range(starts[b], starts[b + 1]):
                acc += int(loc[ids[s]])
                cu.append(acc)
    cu_seqlens = np.array(cu, np.int32)

    # segments in (q, destination row) order
    a2a = np.zeros((S, D * C), np.int64)
    seg = {k: [] for k in ("src_shard", "src_row", "dst_shard", "dst_row", "n_real", "n_rows",
                           "pos0", "seq")}
    shard_seg_start = [0]
    halves = K // C
    for r in range(D):
        for c in range(C):
            q = r * C + c
            for i in pk["seq_ids"][r]:
                mi = int(m[i])
                for h in range(halves):
                    kappa = c if h == 0 else 2 * C - 1 - c
                    assert chunk_to_sp(kappa, C, K) == (c, h)
                    p0 = kappa * mi
                    n_real = min(max(int(L[i]) - p0, 0), mi)
                    seg["src_shard"].append(int(seq_shard[i]))
                    seg["src_row"].append(int(srow[i]) + p0)
                    seg["dst_shard"].append(q)
                    seg["dst_row"].append(int(pk["dst_row"][i]) + h * mi)
                    seg["n_real"].append(n_real)
                    seg["n_rows"].append(mi)
                    seg["pos0"].append(p0)
                    seg["seq"].append(i)
                    a2a[int(seq_shard[i]), q] += n_real
            shard_seg_start.append(len(seg["seq"]))

    return Plan(N=N, S=S, D=D, C=C, K=K, P=P, B=B, L=np.asarray(L, np.int64), m=m, Lp=Lp, loc=loc,
                seq_group=grp, seq_shard=seq_shard, seq_row=srow, seq_k=seq_k, group_rows=group_rows,
                rank=rank, rank_load=load, slot=pk["slot"], mb=pk["mb"], dst_row=pk["dst_row"],
                n_seq=pk["n_seq"], n_mb=pk["n_mb"], shard_rows=shard_rows, seq_ids=seq_ids,
                mb_seq_start=mb_seq_start, mb_row_start=mb_row_start, cu_seqlens=cu_seqlens,
                a2a_counts=a2a,
                seg_src_shard=np.array(seg["src_shard"], np.int32),
                seg_src_row=np.array(seg["src_row"], np.int64),
                seg_dst_shard=np.array(seg["dst_shard"], np.int32),
                seg_dst_row=np.array(seg["dst_row"], np.int64),
                seg_n_real=np.array(seg["n_real"], np.int32),
                seg_n_rows=np.array(seg["n_rows"], np.int32),
                seg_pos0=np.array(seg["pos0"], np.int32),
                seg_seq=np.array(seg["seq"], np.int32),
                shard_seg_start=np.array(shard_seg_start, np.int32))


# ----------------------------------------------------------------------------------------
# Field materialisation
# ----------------------------------------------------------------------------------------
def pad_row(scalar_dtype, width: int, pad_scalar: int) -> np.ndarray:
    """One padding row: `width` copies of the low bytes of pad_scalar (little-endian)."""
    nbytes = np.dtype(scalar_dtype).itemsize
    raw = int(pad_scalar) & ((1 << (8 * nbytes)) - 1)
    return np.full((width,), raw, dtype=scalar_dtype)


def dispatch_field_shard(plan: Plan, q: int, src_bufs: Sequence, scalar_dtype, width: int,
                         pad_scalar: int, per_sequence: bool = False) -> np.ndarray:
    """Destination shard q of one field, in the training layout.

    src_bufs[s] is shard buffer s as an array of shape (rows, width) (anything that supports
    row slicing).  For sequence i on DP rank r = q // C and each chunk kappa held by SP rank
    c = q % C, logical position p = kappa*m + j lands on row dst_row[i] + h*m + j; it receives
    source row seq_row[i] + p of buffer seq_shard[i] when p < L[i], else the padding row.

    per_sequence: the source buffers hold ONE row per sequence (row seq_k[i] of buffer
    seq_shard[i]), e.g. a sequence-level advantage or reward (Section 5 names them as the next
    tensors to dispatch); every real position of the sequence receives that row.
    """
    C, K = plan.C, plan.K
    r, c = divmod(q, C)
    out = np.empty((int(plan.shard_rows[q]), width), dtype=scalar_dtype)
    pad = pad_row(scalar_dtype, width, pad_scalar)
    first = int(np.sum(plan.n_seq[:r]))
    for i in plan.seq_ids[first:first + int(plan.n_seq[r])]:
        i = int(i)
        mi, Li = int(plan.m[i]), int(plan.L[i])
        src = src_bufs[int(plan.seq_shard[i])]
        for kappa in range(K):
            cc, h = chunk_to_sp(kappa, C, K)
            if cc != c:
                continue
            p0 = kappa * mi
            n_real = min(max(Li - p0, 0), mi)
            d0 = int(plan.dst_row[i]) + h * mi
            s0 = int(plan.seq_row[i]) + p0
            if per_sequence:
                out[d0:d0 + n_real] = src[int(plan.seq_k[i])]
            else:
                out[d0:d0 + n_real] = src[s0:s0 + n_real]
            out[d0 + n_real:d0 + mi] = pad
    return out


def dispatch_field(plan: Plan, src_bufs: Sequence, scalar_dtype, width: int,
                   pad_scalar: int, per_sequence: bool = False) -> List[np.ndarray]:
    """All D*C destination shards of one field."""
    return [dispatch_field_shard(plan, q, src_bufs, scalar_dtype, width, pad_scalar, per_sequence)
            for q in range(plan.D * plan.C)]


def nonzero_counts(plan: Plan, src_bufs: Sequence, width: int = 1) -> np.ndarray:
    """A consumer of the dispatched field computed on the way: counts[q][b] = how many scalars
    of the REAL rows of destination shard q that lie in micro-batch b of its data-parallel rank
    are non-zero, as int64[D*C][max n_mb] (zero where a rank has fewer micro-batches).  For a
    0/1 response mask this is the number of loss tokens every (shard, micro-batch) holds, the
    denominator of a token-mean loss.  Padding rows never count, whatever the padding scalar.
    """
    C, K, D = plan.C, plan.K, plan.D
    most = int(plan.n_mb.max()) if D else 0
    out = np.zeros((D * C, most), np.int64)
    for i in range(plan.N):
        r = int(plan.rank[i])
        mi, Li = int(plan.m[i]), int(plan.L[i])
        src = src_bufs[int(plan.seq_shard[i])]
        for kappa in range(K):
            c, _ = chunk_to_sp(kappa, C, K)
            p0 = kappa * mi
            n_real = min(max(Li - p0, 0), mi)
            s0 = int(plan.seq_row[i]) + p0
            rows = np.asarray(src[s0:s0 + n_real]).reshape(n_real, width)
            out[r * C + c, int(plan.mb[i])] += int(np.count_nonzero(rows))
    return out


def position_ids_shard(plan: Plan, q: int) -> np.ndarray:
    """Position ids of destination shard q: the logical position p of every row, padding rows
    included (they keep counting past L)."""
    C, K = plan.C, plan.K
    r, c = divmod(q, C)
    out = np.empty((int(plan.shard_rows[q]),), np.int32)
    first = int(np.sum(plan.n_seq[:r]))
    for i in plan.seq_ids[first:first + int(plan.n_seq[r])]:
        i = int(i)
        mi = int(plan.m[i])
        for kappa in range(K):
            cc, h = chunk_to_sp(kappa, C, K)
            if cc != c:
                continue
            d0 = int(plan.dst_row[i]) + h * mi
            out[d0:d0 + mi] = np.arange(kappa * mi, (kappa + 1) * mi, dtype=np.int64)
    return out


def source_row_map_shard(plan: Plan, q: int):
    """For every row of destination shard q: (source shard buffer, source row), or (-1, -1)
    for a padding row.  Lets a test build the expected shard of a very large field with any
    gather routine, without holding all source buffers on the host."""
    C, K = plan.C, plan.K
    r, c = divmod(q, C)
    rows = int(plan.shard_rows[q])
    shard = np.full((rows,), -1, np.int32)
    row = np.full((rows,), -1, np.int64)
    first = int(np.sum(plan.n_seq[:r]))
    for i in plan.seq_ids[first:first + int(plan.n_seq[r])]:
        i = int(i)
        mi, Li = int(plan.m[i]), int(plan.L[i])
        for kappa in range(K):
            cc, h = chunk_to_sp(kappa, C, K)
            if cc != c:
                continue
            p0 = kappa * mi
            n_real = min(max(Li - p0, 0), mi)
            d0 = int(plan.dst_row[i]) + h * mi
            shard[d0:d0 + n_real] = int(plan.seq_shard[i])
            row[d0:d0 + n_real] = np.arange(int(plan.seq_row[i]) + p0,
                                            int(plan.seq_row[i]) + p0 + n_real, dtype=np.int64)
    return shard, row


# ----------------------------------------------------------------------------------------
# Inverse
# ----------------------------------------------------------------------------------------
def inverse_field(plan: Plan, dst_shards: Sequence[np.ndarray], src_bufs_out: Sequence[np.ndarray]):
    """Training layout -> rollout layout: every real (i, p) row is copied back to the source
    row it was read from.  Rows of src_bufs_out that no sequence was read from (padding has no
    source; other replicas of a replicated group) are left untouched."""
    C, K = plan.C, plan.K
    for i in range(plan.N):
        mi, Li = int(plan.m[i]), int(plan.L[i])
        r = int(plan.rank[i])
        out = src_bufs_out[int(plan.seq_shard[i])]
        for kappa in range(K):
            c, h = chunk_to_sp(kappa, C, K)
            p0 = kappa * mi
            n_real = min(max(Li - p0, 0), mi)
            d0 = int(plan.dst_row[i]) + h * mi
            s0 = int(plan.seq_row[i]) + p0
            out[s0:s0 + n_real] = dst_shards[r * C + c][d0:d0 + n_real]


# ----------------------------------------------------------------------------------------
# Byte accounting
# ----------------------------------------------------------------------------------------
def algorithmic_bytes(plan: Plan, row_bytes: Sequence[int], with_position_ids: bool = True) -> int:
    """Bytes one dispatch must move: each real source row read once, each destination row
    (padding included) written once, plus 4 bytes of position id per destination row.  Linear
    in the token count for a fixed field set, like Table 1 of the paper."""
    w = int(sum(int(x) for x in row_bytes))
    total = w * plan.total_real_rows + w * plan.total_dst_rows
    if with_position_ids:
        total += 4 * plan.total_dst_rows
    return total

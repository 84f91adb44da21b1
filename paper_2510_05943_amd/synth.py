"""Seeded synthetic rollout batches for the re-layout path.

This module only *draws inputs*: sequence lengths, layout descriptors and per-token field
values shaped like the intermediate batches of the paper's Section 1 (tokens, log
probabilities, advantages, auxiliary tensors) and like agentic multi-turn episodes
(footnote of Section 1: episode-level length is the cumulative token count over the turns).
It holds none of the dispatch arithmetic: no padding, balancing, chunking or offsets are
computed here.  Both the CPU oracle's tests and the GPU path's tests and benchmark take their
inputs from here, so the two sides always see identical bytes.

The paper's own rollouts (Connect Four / Tic-Tac-Toe episodes of a trained model) are not
available; these batches stand in for them.

All draws use numpy's counter-based Philox generator, keyed by (seed, stream id), so every
buffer can be generated on its own, in any order, with the same result.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

__all__ = ["FieldSpec", "Workload", "CONFIG_NAMES", "make_workload", "custom_workload"]


@dataclasses.dataclass(frozen=True)
class FieldSpec:
    """One per-token tensor of the batch: `width` scalars of `scalar_bytes` bytes per token."""
    name: str
    scalar_bytes: int
    width: int
    pad_scalar: int          # low `scalar_bytes` bytes are the fill pattern for padding rows
    kind: str                # which generator draws it (see Workload.group_buffer)
    per_sequence: bool = False   # the source holds one row per sequence instead of one per token

    @property
    def row_bytes(self) -> int:
        return self.scalar_bytes * self.width

    @property
    def np_dtype(self):
        return {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[self.scalar_bytes]


F_ID = FieldSpec("token_id", 4, 1, 0, "token_id")
F_MASK = FieldSpec("loss_mask", 1, 1, 0, "mask")
F_OLD = FieldSpec("old_logprob", 4, 1, 0, "logprob")
F_REF = FieldSpec("ref_logprob", 4, 1, 0, "logprob")
F_ADV = FieldSpec("advantage", 4, 1, 0, "advantage")


def _hidden(width: int) -> FieldSpec:
    return FieldSpec("hidden_bf16", 2, width, 0, "hidden")


def _stream(seed: int, *tags) -> np.random.Generator:
    """Independent generator for (seed, tags): Philox keyed by a CRC of the tag string."""
    tag = zlib.crc32("/".join(str(t) for t in tags).encode())
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(tag)]))


def _f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 values to bfloat16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


_POOL_ROWS = 1 << 16


@dataclasses.dataclass
class Workload:
    """Lengths, layout descriptors and field generators of one synthetic batch."""
    name: str
    seed: int
    lengths: np.ndarray                 # int32[N], real tokens per sequence
    n_groups: int                       # G source replica groups
    replication: int                    # R identical replicas per group (S = G*R shard buffers)
    seq_group: np.ndarray               # int32[N], group that holds sequence i
    dp: int
    sp: int
    zigzag: int
    pad_multiple: int
    mb_token_budget: int
    fields: Tuple[FieldSpec, ...]
    turn_spans: Optional[List[np.ndarray]] = None   # agentic: per episode, [agent, env, agent, env, ...]
    _pool: Dict[int, np.ndarray] = dataclasses.field(default_factory=dict, repr=False)

    @property
    def n_seqs(self) -> int:
        return int(self.lengths.shape[0])

    @property
    def n_shards(self) -> int:
        return self.n_groups * self.replication

    @property
    def total_tokens(self) -> int:
        return int(self.lengths.astype(np.int64).sum())

    def group_members(self, g: int) -> np.ndarray:
        """Sequence indices stored in group g's buffers, in index order."""
        return np.nonzero(self.seq_group == g)[0]

    def group_rows(self, g: int) -> int:
        return int(self.lengths[self.seq_group == g].astype(np.int64).sum())

    # ---- field values -------------------------------------------------------------------
    def hidden_pool(self, width: int) -> np.ndarray:
        """The pool of distinct N(0,1) bf16 rows the wide field is drawn from."""
        return self._hidden_pool(width)

    def hidden_rows_index(self, g: int) -> np.ndarray:
        """Pool row of every row of group g's buffer of the wide field, in buffer order, so
        that the buffer can be materialised by any gather (pool[index]), e.g. on the device."""
        members = self.group_members(g)
        lens = self.lengths[members].astype(np.int64)
        seq = np.repeat(members.astype(np.int64), lens)
        starts = np.cumsum(lens) - lens
        pos = np.arange(int(lens.sum()), dtype=np.int64) - np.repeat(starts, lens)
        return self.hidden_pool_index(seq, pos)

    def _hidden_pool(self, width: int) -> np.ndarray:
        if width not in self._pool:
            rng = _stream(self.seed, self.name, "hidden_pool", width)
            self._pool[width] = _f32_to_bf16_bits(
                rng.standard_normal((_POOL_ROWS, width), dtype=np.float32))
        return self._pool[width]

    def hidden_pool_index(self, seq: np.ndarray, pos: np.ndarray) -> np.ndarray:
        """Pool row used for token `pos` of sequence `seq` (a fixed integer mix, not a draw)."""
        x = (seq.astype(np.uint64) * np.uint64(0x9E3779B97F4A7C15)
             + pos.astype(np.uint64) * np.uint64(0xC2B2AE3D27D4EB4F)
             + np.uint64(self.seed) * np.uint64(0x165667B19E3779F9))
        x ^= x >> np.uint64(29)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(32)
        return (x & np.uint64(_POOL_ROWS - 1)).astype(np.int64)

    def group_buffer(self, field: FieldSpec, g: int) -> np.ndarray:
        """Contents of group g's buffer for `field`: its sequences packed in index order.

        Returns an array of shape (rows, width) of the field's unsigned scalar type (the raw
        bits of the values).  Every replica of the group holds these same bytes.
        """
        members = self.group_members(g)
        lens = self.lengths[members].astype(np.int64)
        rows = int(lens.sum())
        rng = _stream(self.seed, self.name, field.name, g)
        if field.kind == "token_id":
            out = rng.integers(0, 32000, size=rows, dtype=np.int64).astype(np.uint32)
        elif field.kind == "mask":
            if self.turn_spans is not None:
                parts = []
                for i in members:
                    spans = self.turn_spans[int(i)]
                    vals = np.tile(np.array([1, 0], dtype=np.uint8), len(spans) // 2)
                    parts.append(np.repeat(vals, spans))
                out = np.concatenate(parts) if parts else np.zeros(0, np.uint8)
            else:
                out = (rng.random(rows) < 0.7).astype(np.uint8)
        elif field.kind == "logprob":
            out = (-np.abs(rng.normal(0.0, 2.0, size=rows))).astype(np.float32).view(np.uint32)
        elif field.kind == "advantage":
            per_seq = rng.standard_normal(len(members)).astype(np.float32)
            out = np.repeat(per_seq, lens).view(np.uint32)
        elif field.kind == "hidden":
            out = self._hidden_pool(field.width)[self.hidden_rows_index(g)]
        elif field.kind == "seq_value":
            rows = len(members)
            out = rng.integers(0, 256, size=(rows, field.row_bytes), dtype=np.uint8).view(field.np_dtype)
        elif field.kind == "bytes":
            out = rng.integers(0, 256, size=(rows, field.row_bytes),
                               dtype=np.uint8).view(field.np_dtype)
        elif field.kind == "sparse":
            # random scalars, about half of them zero, some with a single non-zero byte
            out = rng.integers(0, 256, size=(rows, field.row_bytes), dtype=np.uint8)
            keep_byte = rng.random((rows, field.row_bytes)) < 0.5
            out = np.where(keep_byte, out, 0).astype(np.uint8).view(field.np_dtype)
            out = np.where(rng.random((rows, field.width)) < 0.5, out.reshape(rows, field.width), 0)
            out = out.astype(field.np_dtype)
        else:
            raise ValueError(field.kind)
        out = np.ascontiguousarray(out.reshape(rows, field.width))
        assert out.dtype == field.np_dtype, (out.dtype, field)
        return out


    def device_shard_buffers(self, field: FieldSpec, torch) -> list:
        """The S shard buffers of `field` as device tensors (input staging only).

        Narrow fields are drawn on the host and uploaded.  The wide bf16 field is materialised on
        the device as pool[index] (torch.index_select), which yields exactly the bytes
        group_buffer() returns, without drawing tens of gigabytes on the host.  Replicas of a
        group are separate buffers holding the same bytes.
        """
        signed = {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}

        def dev(a):
            a = np.ascontiguousarray(a)
            return torch.from_numpy(a.view(signed[a.dtype.itemsize])).cuda()

        groups = []
        for g in range(self.n_groups):
            if field.kind == "hidden":
                pool = dev(self.hidden_pool(field.width))
                idx = torch.from_numpy(self.hidden_rows_index(g)).cuda()
                groups.append(pool.index_select(0, idx))
                del idx, pool
            else:
                groups.append(dev(self.group_buffer(field, g)))
        return [groups[s // self.replication] if s % self.replication == 0
                else groups[s // self.replication].clone() for s in range(self.n_shards)]


CONFIG_NAMES = ("tiny", "mid", "agentic", "heavy", "longctx")


def _contiguous_groups(n: int, g: int) -> np.ndarray:
    """Group of sequence i when G groups own equal contiguous index ranges."""
    return ((np.arange(n, dtype=np.int64) * g) // n).astype(np.int32)


def make_workload(name: str, seed: int = 0, scale: float = 1.0) -> Workload:
    """One of the five named workloads.  `scale` < 1 shrinks only the sequence COUNT (for
    quick checks); lengths, fields and layouts keep their real shape."""
    rng = _stream(seed, name, "lengths")
    turn_spans = None

    def count(n: int, multiple: int) -> int:
        k = max(multiple, int(round(n * scale / multiple)) * multiple)
        return k

    if name == "tiny":
        n = count(64, 4)
        lengths = rng.integers(16, 513, size=n)
        cfg = dict(n_groups=4, replication=1, dp=2, sp=1, zigzag=0, pad_multiple=1,
                   mb_token_budget=4096, fields=(F_ID, F_MASK, F_OLD, F_ADV))
    elif name == "mid":
        n = count(1024, 8)
        lengths = np.clip(np.rint(rng.lognormal(np.log(2048.0), 0.8, size=n)), 64, 8192)
        cfg = dict(n_groups=8, replication=1, dp=8, sp=2, zigzag=1, pad_multiple=64,
                   mb_token_budget=16384, fields=(F_ID, F_MASK, F_OLD, F_ADV, F_REF))
    elif name == "agentic":
        n = count(512, 8)
        turns = rng.integers(2, 13, size=n)
        turn_spans, lengths = [], np.zeros(n, dtype=np.int64)
        for i in range(n):
            agent = rng.integers(128, 1025, size=int(turns[i]))
            env = rng.integers(32, 513, size=int(turns[i]))
            spans = np.stack([agent, env], axis=1).reshape(-1).astype(np.int64)
            over = int(spans.sum()) - 32768          # growing context is cut at the cap
            while over > 0:
                cut = min(over, int(spans[-1]))
                spans[-1] -= cut
                over -= cut
                if spans[-1] == 0:
                    spans = spans[:-1]
            if len(spans) % 2:
                spans = np.append(spans, 0)
            turn_spans.append(spans)
            lengths[i] = spans.sum()
        cfg = dict(n_groups=2, replication=4, dp=4, sp=4, zigzag=0, pad_multiple=1,
                   mb_token_budget=65536, fields=(F_ID, F_MASK, F_OLD, F_ADV, F_REF))
    elif name == "heavy":
        n = count(2048, 8)
        lengths = np.clip(np.rint(rng.lognormal(np.log(4096.0), 0.9, size=n)), 128, 32768)
        cfg = dict(n_groups=8, replication=1, dp=8, sp=4, zigzag=1, pad_multiple=1,
                   mb_token_budget=131072,
                   fields=(F_ID, F_MASK, F_OLD, F_ADV, F_REF, _hidden(1024)))
    elif name == "longctx":
        n = count(256, 8)
        lengths = rng.integers(32768, 131073, size=n)
        cfg = dict(n_groups=8, replication=1, dp=2, sp=8, zigzag=1, pad_multiple=128,
                   mb_token_budget=262144,
                   fields=(F_ID, F_MASK, F_OLD, F_REF, F_ADV, _hidden(512)))
    else:
        raise ValueError(f"unknown workload {name!r}; choose from {CONFIG_NAMES}")
    lengths = np.asarray(lengths).astype(np.int32)
    return Workload(name=name, seed=seed, lengths=lengths,
                    seq_group=_contiguous_groups(n, cfg["n_groups"]),
                    turn_spans=turn_spans, **cfg)


def custom_workload(lengths: Sequence[int], *, n_groups: int = 1, replication: int = 1,
                    seq_group: Optional[Sequence[int]] = None, dp: int = 1, sp: int = 1,
                    zigzag: int = 0, pad_multiple: int = 1, mb_token_budget: int = 1 << 40,
                    fields: Optional[Sequence[FieldSpec]] = None, seed: int = 0,
                    name: str = "custom") -> Workload:
    """A batch with caller-chosen lengths and layouts (edge-case tests)."""
    lengths = np.asarray(lengths, dtype=np.int32)
    n = int(lengths.shape[0])
    if seq_group is None:
        seq_group = _contiguous_groups(n, n_groups) if n else np.zeros(0, np.int32)
    if fields is None:
        fields = (F_ID, F_MASK, F_OLD, F_ADV)
    return Workload(name=name, seed=seed, lengths=lengths, n_groups=n_groups,
                    replication=replication, seq_group=np.asarray(seq_group, dtype=np.int32),
                    dp=dp, sp=sp, zigzag=zigzag, pad_multiple=pad_multiple,
                    mb_token_budget=mb_token_budget, fields=tuple(fields))


def per_sequence_field(name: str, scalar_bytes: int, width: int = 1, pad_scalar: int = 0) -> FieldSpec:
    """One random row per SEQUENCE (a sequence-level reward or advantage), to be broadcast."""
    return FieldSpec(name, scalar_bytes, width, pad_scalar, "seq_value", per_sequence=True)


def sparse_field(name: str, scalar_bytes: int, width: int = 1, pad_scalar: int = 0) -> FieldSpec:
    """Random scalars of which about half are zero (what a non-zero count can be tested on)."""
    return FieldSpec(name, scalar_bytes, width, pad_scalar, "sparse")


def bytes_field(name: str, scalar_bytes: int, width: int, pad_scalar: int = 0) -> FieldSpec:
    """A field of uniformly random bytes with an arbitrary scalar size and width."""
    return FieldSpec(name, scalar_bytes, width, pad_scalar, "bytes")

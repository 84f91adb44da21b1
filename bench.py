#!/usr/bin/env python3
"""Benchmark of the re-layout hot path on one MI355X.

A step is one pass of the whole path over one synthetic rollout batch that is already resident
in HBM: earl_plan_build (source offsets, padded geometry, rank assignment, packing,
micro-batches, segment table), earl_plan_get_summary (the shard sizes reach the host) and
earl_dispatch (every field, every destination shard, position ids, cu_seqlens).  The headline
workload is "heavy" (2048 sequences, about 12.4 M tokens, 2065 bytes per token, DP8 x SP4 zigzag:
the largest of the five workloads by bytes moved).

Prints ONE JSON line:
  value         real tokens re-laid-out per second over the timed steps (plan + dispatch);
  roofline      the kernels of earl_dispatch (decode pass and copy; HIP events recorded by the
                library around them) priced against the 8 TB/s HBM peak with algorithmic bytes:
                each real source row read once, each destination row written once, 4 bytes of
                position id per destination row;
  secondary     the same measurements for the other four workloads (longctx, mid, agentic, tiny)
                and for the reverse direction on the headline workload; the small workloads also
                with the step that never waits between plan and dispatch (earl_dispatch_async);
  cpu_baseline  the CPU oracle timed on the host cores, on the headline workload's own inputs.
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")

WORKLOAD_NOTES = {
    "tiny": "c1 tiny: 64 seqs U[16,512], 4 src shards, 4 fields (13 B/token), DP2 SP1, budget 4096",
    "mid": "c2 mid: 1024 seqs lognormal(2048,0.8) in [64,8192], 8 src shards, 5 fields (17 B/token), "
           "DP8 SP2 zigzag, pad 64, budget 16384",
    "agentic": "c3 agentic multi-turn: 512 episodes x 2-12 turns, TP4xDP2 replicated source "
               "(8 shards), 5 fields (17 B/token), DP4 SP4, budget 65536",
    "heavy": "c4 heavy intermediates: 2048 seqs lognormal(4096,0.9) in [128,32768] (~12.4M tokens), "
             "8 src shards, 5 scalar fields + bf16[1024] (2065 B/token), DP8 SP4 zigzag, budget 131072",
    "longctx": "c5 long-context: 256 seqs U[32768,131072] (~21.9M tokens), 8 src shards, 5 scalar "
               "fields + bf16[512] (1041 B/token), DP2 SP8 zigzag, pad 128, budget 262144",
}
SMALL = ("tiny", "mid", "agentic")     # cache-resident: latency-bound, not an HBM figure


def kernel_source_hash() -> str:
    """sha256 over the sources the re-layout kernels are built from (kernel file + constants)."""
    h = hashlib.sha256()
    for name in ("earl_copy.hip", "earl_internal.h"):
        with open(os.path.join(ROOT, "paper_2510_05943_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload: str, direction: str):
    """HBM bytes of one dispatch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/), or None
    when the kernels have changed since the counters were taken."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if t.get("kernel_source_sha256") != kernel_source_hash():
        return None
    return t.get(direction, {}).get(workload)


class HipEvents:
    """hipEvent_t handles through ctypes (the HIP runtime is already loaded by torch)."""

    def __init__(self):
        import ctypes
        self.c = ctypes
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]

    def create(self) -> int:
        ev = self.c.c_void_p()
        if self.lib.hipEventCreate(self.c.byref(ev)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = self.c.c_float()
        if self.lib.hipEventElapsedTime(self.c.byref(ms), a, b) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.lib.hipEventDestroy(ev)


class Staged:
    """One workload resident in HBM: sources, destination buffers, plan workspace, scratch."""

    def __init__(self, name, seed, balance_policy, torch, B, synth):
        self.name, self.torch, self.B = name, torch, B
        w = self.w = synth.make_workload(name, seed=seed)
        t0 = time.time()
        src = self.src = {f.name: w.device_shard_buffers(f, torch) for f in w.fields}
        torch.cuda.synchronize()
        self.stage_s = time.time() - t0
        self.stream = torch.cuda.current_stream()
        self.src_l = B.SrcLayout(w.n_groups, w.replication)
        self.dst_l = B.DstLayout(w.dp, w.sp, w.zigzag, w.pad_multiple, w.mb_token_budget, balance_policy)
        self.lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
        self.ws = torch.empty(B.plan_workspace_bytes(w.n_seqs, self.src_l, self.dst_l),
                              dtype=torch.uint8, device="cuda")
        # sizes of the destination shards come from a first plan
        plan0 = self.build()
        sm = self.sm = B.plan_get_summary(plan0)
        rows = [int(r) for r in sm["shard_rows"]]
        self.fields = []
        for f in w.fields:
            dsts = [torch.empty((r * f.row_bytes,), dtype=torch.uint8, device="cuda") for r in rows]
            self.fields.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src[f.name], dsts))
        self.pos = [torch.empty((r,), dtype=torch.int32, device="cuda") for r in rows]
        self.cu = torch.empty((sm["cu_seqlens_len"],), dtype=torch.int32, device="cuda")
        need = max(B.dispatch_workspace_bytes(plan0, self.fields),
                   B.dispatch_async_workspace_bytes(plan0, self.fields, self.pos, self.cu))
        self.scratch = torch.empty(need, dtype=torch.uint8, device="cuda")
        B.plan_destroy(plan0)
        self.row_bytes = sum(f.row_bytes for f in w.fields)
        self.algo_forward = (self.row_bytes * (sm["total_real_rows"] + sm["total_dst_rows"])
                             + 4 * sm["total_dst_rows"])
        # training layout -> rollout layout: every real row read once and written once
        self.algo_inverse = 2 * self.row_bytes * sm["total_real_rows"]

    def build(self):
        return self.B.plan_build(self.lengths, self.w.n_seqs, self.src_l, self.dst_l, self.ws,
                                 stream=self.stream)

    def dispatch(self, p):
        self.B.dispatch(p, self.fields, position_ids=self.pos, cu_seqlens=self.cu,
                        workspace=self.scratch, stream=self.stream)

    def step(self, mode, ev=None):
        """mode "sync": plan, wait for its totals, dispatch.  "async": plan, dispatch enqueued
        right behind it (buffers are pre-allocated), totals and the device's verdict afterwards.
        "inverse": plan, wait, reverse direction."""
        B = self.B
        p = self.build()
        if ev is not None:
            B.plan_set_dispatch_events(p, ev[0], ev[1])
        if mode == "async":
            B.dispatch_async(p, self.fields, position_ids=self.pos, cu_seqlens=self.cu,
                             workspace=self.scratch, stream=self.stream)
            B.plan_wait(p)
            return p
        B.plan_wait(p)                  # earl_plan_get_summary: the shard sizes are on the host
        if mode == "inverse":
            B.dispatch_inverse(p, self.fields, workspace=self.scratch, stream=self.stream)
        else:
            self.dispatch(p)
        return p

    def finish(self, plans, mode):
        for p in plans:
            if mode == "async" and self.B.dispatch_async_status(p) != self.B.EARL_OK:
                raise RuntimeError("asynchronous dispatch was refused on the device")
            self.B.plan_destroy(p)

    def timed(self, mode, steps, warmup, hip):
        """W untimed steps, then K steps between device synchronisations; the dispatch kernels of
        every timed step are bracketed by HIP events that the library records on the stream."""
        torch = self.torch
        if mode == "inverse":
            p = self.build()
            self.dispatch(p)            # the destination shards hold a real training layout
            torch.cuda.synchronize()
            self.B.plan_destroy(p)
        plans = [self.step(mode) for _ in range(warmup)]
        torch.cuda.synchronize()
        self.finish(plans, mode)
        events = [(hip.create(), hip.create()) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plans = [self.step(mode, events[k]) for k in range(steps)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        self.finish(plans, mode)
        kern = [hip.elapsed_ms(a, b) for a, b in events]
        for a, b in events:
            hip.destroy(a)
            hip.destroy(b)
        return (t1 - t0) * 1e3 / steps, kern

    def halves(self, mode):
        """The two calls on their own, each ending with a wait (medians of 10): plan = build +
        summary, dispatch = enqueue + stream synchronisation."""
        plan_ms, dispatch_ms = [], []
        for _ in range(10):
            ta = time.perf_counter()
            p = self.build()
            self.B.plan_wait(p)
            tb = time.perf_counter()
            if mode == "inverse":
                self.B.dispatch_inverse(p, self.fields, workspace=self.scratch, stream=self.stream)
            else:
                self.dispatch(p)
            self.torch.cuda.synchronize()
            tc = time.perf_counter()
            self.B.plan_destroy(p)
            plan_ms.append((tb - ta) * 1e3)
            dispatch_ms.append((tc - tb) * 1e3)
        return float(np.median(plan_ms)), float(np.median(dispatch_ms))

    def measure(self, mode, steps, warmup, hip):
        ms, kern = self.timed(mode, steps, warmup, hip)
        algo = self.algo_inverse if mode == "inverse" else self.algo_forward
        k_avg = float(np.mean(kern))
        out = {"ms_per_step": ms, "steps": steps,
               "tokens_per_s": self.sm["total_real_rows"] / (ms * 1e-3),
               "whole_path_GBps": algo / (ms * 1e-3) / 1e9,
               "kernels_ms_avg": k_avg, "kernels_ms_min": float(np.min(kern)),
               "kernels_ms_median": float(np.median(kern)),
               "algorithmic_bytes": algo, "achieved_GBps": algo / (k_avg * 1e-3) / 1e9,
               "frac": algo / (k_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        if mode != "async":
            out["plan_ms"], out["dispatch_ms"] = self.halves(mode)
        return out


def run_two_pass(args, torch, B, synth, hip):
    """The single-controller pattern the paper argues against (Section 1: all intermediate data is
    aggregated in one place before it is redistributed), done with the same library on one GPU:
    pass 1 gathers every field into one canonical buffer (plan with dp = sp = 1), pass 2 scatters
    it from there into the training layout.  Same result as the direct dispatch, twice the bytes."""
    w = synth.make_workload(args.workload, seed=args.seed)
    t0 = time.time()
    src = {f.name: w.device_shard_buffers(f, torch) for f in w.fields}
    torch.cuda.synchronize()
    stage_s = time.time() - t0
    stream = torch.cuda.current_stream()
    lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
    lay_a = (B.SrcLayout(w.n_groups, w.replication), B.DstLayout(1, 1, 0, 1, 1 << 40))
    lay_b = (B.SrcLayout(1, 1), B.DstLayout(w.dp, w.sp, w.zigzag, w.pad_multiple, w.mb_token_budget,
                                            args.balance_policy))
    ws_a = torch.empty(B.plan_workspace_bytes(w.n_seqs, *lay_a), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(B.plan_workspace_bytes(w.n_seqs, *lay_b), dtype=torch.uint8, device="cuda")
    pa = B.plan_build(lengths, w.n_seqs, *lay_a, ws_a, stream=stream)
    pb = B.plan_build(lengths, w.n_seqs, *lay_b, ws_b, stream=stream)
    sm_a, sm = B.plan_get_summary(pa), B.plan_get_summary(pb)
    total = int(sm_a["shard_rows"][0])
    shard_rows = [int(r) for r in sm["shard_rows"]]
    fields_a, fields_b = [], []
    for f in w.fields:
        canon = torch.empty((total * f.row_bytes,), dtype=torch.uint8, device="cuda")
        dsts = [torch.empty((r * f.row_bytes,), dtype=torch.uint8, device="cuda") for r in shard_rows]
        fields_a.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src[f.name], [canon]))
        fields_b.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, [canon], dsts))
    pos = [torch.empty((r,), dtype=torch.int32, device="cuda") for r in shard_rows]
    cu = torch.empty((sm["cu_seqlens_len"],), dtype=torch.int32, device="cuda")
    scr_a = torch.empty(B.dispatch_workspace_bytes(pa, fields_a, False, False), dtype=torch.uint8, device="cuda")
    scr_b = torch.empty(B.dispatch_workspace_bytes(pb, fields_b), dtype=torch.uint8, device="cuda")
    B.plan_destroy(pa)
    B.plan_destroy(pb)
    row_bytes = sum(f.row_bytes for f in w.fields)
    algo = (2 * row_bytes * total
            + row_bytes * (sm["total_real_rows"] + sm["total_dst_rows"]) + 4 * sm["total_dst_rows"])

    def step(ev=None):
        a = B.plan_build(lengths, w.n_seqs, *lay_a, ws_a, stream=stream)
        B.plan_wait(a)
        if ev is not None:
            B.plan_set_dispatch_events(a, ev[0], ev[1])
        B.dispatch(a, fields_a, workspace=scr_a, stream=stream)
        b = B.plan_build(lengths, w.n_seqs, *lay_b, ws_b, stream=stream)
        B.plan_wait(b)
        if ev is not None:
            B.plan_set_dispatch_events(b, ev[2], ev[3])
        B.dispatch(b, fields_b, position_ids=pos, cu_seqlens=cu, workspace=scr_b, stream=stream)
        return [a, b]

    plans = [p for _ in range(args.warmup) for p in step()]
    torch.cuda.synchronize()
    for p in plans:
        B.plan_destroy(p)
    events = [tuple(hip.create() for _ in range(4)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plans = [p for k in range(args.steps) for p in step(events[k])]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for p in plans:
        B.plan_destroy(p)
    ms = (t1 - t0) * 1e3 / args.steps
    kern = [hip.elapsed_ms(e[0], e[1]) + hip.elapsed_ms(e[2], e[3]) for e in events]
    for e in events:
        for x in e:
            hip.destroy(x)
    k_avg = float(np.mean(kern))
    res = {"ms_per_step": ms, "steps": args.steps, "tokens_per_s": sm["total_real_rows"] / (ms * 1e-3),
           "whole_path_GBps": algo / (ms * 1e-3) / 1e9, "kernels_ms_avg": k_avg,
           "kernels_ms_min": float(np.min(kern)), "kernels_ms_median": float(np.median(kern)),
           "algorithmic_bytes": algo, "achieved_GBps": algo / (k_avg * 1e-3) / 1e9,
           "frac": algo / (k_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    return w, sm, res, stage_s, row_bytes


def run_copy_ceiling(torch, gib: int = 8, iters: int = 10):
    """What the chip does on plain copies of the shape the re-layout kernels use (one 16-byte load
    and one 16-byte store per lane, one-wavefront workgroups), on reads alone and on writes alone:
    the yardstick kernels of tests/yardstick/copy_ceiling.hip, timed with HIP events."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "tests", "yardstick", "libcopy_ceiling.so"))
    vp, u64 = ctypes.c_void_p, ctypes.c_uint64
    lib.yardstick_copy.argtypes = [vp, vp, u64, vp]
    lib.yardstick_read.argtypes = [vp, vp, u64, vp]
    lib.yardstick_write.argtypes = [vp, u64, vp]
    n = gib << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    src.view(torch.int32).fill_(1)
    dst.view(torch.int32).fill_(2)
    stream = torch.cuda.current_stream().cuda_stream
    runs = {"copy": (lambda: lib.yardstick_copy(src.data_ptr(), dst.data_ptr(), n, stream), 2 * n),
            "read": (lambda: lib.yardstick_read(src.data_ptr(), sink.data_ptr(), n, stream), n),
            "write": (lambda: lib.yardstick_write(dst.data_ptr(), n, stream), n),
            "torch_copy_": (lambda: (dst.view(torch.int32).copy_(src.view(torch.int32)), 0)[1], 2 * n)}
    out = {"bytes": n}
    for name, (fn, moved) in runs.items():
        for _ in range(3):
            if fn():
                raise RuntimeError(f"yardstick {name} failed")
        ms = []
        for _ in range(iters):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ms.append(a.elapsed_time(b))
        t = float(np.median(ms))
        out[name] = {"ms_median": t, "ms_min": float(np.min(ms)), "GBps": moved / t / 1e6,
                     "frac_of_peak": moved / t / 1e6 / HBM_PEAK_GBPS}
    return out


def run_path_histogram(args, torch, B, synth):
    """Which path the destination bytes of every field take, computed on the host from the plan's
    exported segment table with the kernels' own rules.  Direct records (rows under 16 bytes,
    position ids, every field of a small launch) are classified per 16-byte vector: plain copy
    (inside the real rows of one segment), padding fill, position ids (inside one segment),
    straddling (crosses a segment edge or the real/padding edge: moved byte by byte), shard end
    (holds the shard's last bytes: per-lane path).  Coded records (rows of 16 bytes and more in a
    launch above 64 MiB of them) are classified per 4 KiB tile: copy, fill, generic."""
    w = synth.make_workload(args.workload, seed=args.seed)
    stream = torch.cuda.current_stream()
    src_l = B.SrcLayout(w.n_groups, w.replication)
    dst_l = B.DstLayout(w.dp, w.sp, w.zigzag, w.pad_multiple, w.mb_token_budget, args.balance_policy)
    lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
    ws = torch.empty(B.plan_workspace_bytes(w.n_seqs, src_l, dst_l), dtype=torch.uint8, device="cuda")
    plan = B.plan_build(lengths, w.n_seqs, src_l, dst_l, ws, stream=stream)
    sm = B.plan_get_summary(plan)
    seg = B.plan_export_segments(plan)
    B.plan_destroy(plan)
    rows = sm["shard_rows"].astype(np.int64)
    coarse_bytes = sum(int(rows.sum()) * f.row_bytes for f in w.fields if f.row_bytes >= 16)
    names = [(f.name, f.row_bytes, False) for f in w.fields] + [("position_ids", 4, True)]
    table = []
    for name, wb, is_pos in names:
        coded = wb >= 16 and coarse_bytes > (64 << 20)
        unit = 4096 if coded else 16
        counts = {}
        for q in range(len(rows)):
            e0, e1 = int(seg["shard_seg_start"][q]), int(seg["shard_seg_start"][q + 1])
            end = int(rows[q]) * wb
            if end == 0:
                continue
            lo = seg["dst_row"][e0:e1].astype(np.int64) * wb
            real_hi = lo + seg["n_real"][e0:e1].astype(np.int64) * wb
            hi = lo + seg["n_rows"][e0:e1].astype(np.int64) * wb
            first = np.arange(0, end, unit, dtype=np.int64)
            last = first + unit
            e = np.searchsorted(lo, first, side="right") - 1
            in_seg = last <= hi[e]
            beyond = last > end
            if is_pos and not coded:
                kinds = {"position ids": in_seg & ~beyond}
            else:
                kinds = {"copy": in_seg & (last <= real_hi[e]) & ~beyond,
                         ("fill" if coded else "padding"): in_seg & (first >= real_hi[e]) & ~beyond}
            taken = np.zeros(first.shape, bool)
            for k, m in kinds.items():
                counts[k] = counts.get(k, 0) + int(m.sum())
                taken |= m
            rest = ~taken
            if coded:
                counts["generic"] = counts.get("generic", 0) + int(rest.sum())
            else:
                counts["shard end"] = counts.get("shard end", 0) + int((rest & beyond).sum())
                counts["straddling"] = counts.get("straddling", 0) + int((rest & ~beyond).sum())
        total = sum(counts.values())
        table.append({"field": name, "row_bytes": wb, "path": "tile codes (4 KiB tiles)" if coded else
                      "direct (16-byte vectors)", "units": total,
                      "share": {k: v / total for k, v in counts.items()}, "counts": counts})
    return {"workload": args.workload, "seed": args.seed, "fields": table}


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def run_cpu_baseline(args, synth, staged_src=None):
    """The oracle as it stands (one thread: Python loops + numpy slice copies) on the inputs of
    the benchmarked workload itself (same generator, same seed): plan, every field, every
    destination shard, position ids, one pass.  The oracle emits one destination shard at a
    time, so only the source buffers (25.6 GB for the heavy workload) stay in host memory;
    they are the staged input buffers copied back from the GPU (the generator draws the wide
    field much faster there, with the same bytes).  If they do not fit the host's memory, a
    1/8-sequence-count sample of the same distribution is timed instead."""
    from oracle import earl_oracle as O
    sample = None
    try:
        w = synth.make_workload(args.workload, seed=args.seed)
        host = {f.name: [None] * w.n_shards for f in w.fields}
        for f in w.fields:
            for g in range(w.n_groups):
                if staged_src is not None:
                    buf = staged_src[f.name][g * w.replication].cpu().numpy().view(f.np_dtype).reshape(
                        -1, f.width)
                else:
                    buf = w.group_buffer(f, g)
                for t in range(w.replication):
                    host[f.name][g * w.replication + t] = buf
    except MemoryError:
        host = None
        gc.collect()
        w = synth.make_workload(args.workload, seed=args.seed, scale=1.0 / 8)
        host = {f.name: [w.group_buffer(f, s // w.replication) for s in range(w.n_shards)]
                for f in w.fields}
        sample = "the source buffers of the whole workload did not fit the host's memory: "
    row_bytes = sum(f.row_bytes for f in w.fields)
    passes = 0
    t0 = time.perf_counter()
    while True:
        plan = O.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                            seq_group=w.seq_group, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                            pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget)
        for q in range(w.dp * w.sp):
            O.position_ids_shard(plan, q)
            for f in w.fields:
                O.dispatch_field_shard(plan, q, host[f.name], f.np_dtype, f.width, f.pad_scalar)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or passes >= 200:
            break
    algo = row_bytes * (plan.total_real_rows + plan.total_dst_rows) + 4 * plan.total_dst_rows
    what = (f"{w.n_seqs} sequences drawn like the workload" if sample else
            f"the benchmarked inputs themselves (workload {args.workload}, seed {args.seed}, "
            f"{w.n_seqs} sequences)")
    return {"value": passes * w.total_tokens / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "GBps": passes * algo / dt / 1e9, "ms_per_pass": dt * 1e3 / passes,
            "cpu_model": cpu_model(), "host_logical_cpus": os.cpu_count(),
            "sample": (sample or "") + f"{what}: {w.total_tokens} tokens, {algo / 1e9:.2f} GB moved per "
                      f"pass, plan + all fields + all {w.dp * w.sp} destination shards + position ids, "
                      f"{passes} pass(es) in {dt:.1f} s on one core"}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="heavy", choices=list(WORKLOAD_NOTES))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="only the headline workload (profiling runs)")
    ap.add_argument("--two-pass", action="store_true",
                    help="gather into one canonical buffer, then scatter (single-controller pattern)")
    ap.add_argument("--balance-policy", type=int, default=0, choices=[0, 1, 2],
                    help="0 longest-first list scheduling (default), 1 sorted snake deal, "
                         "2 list scheduling on squared padded lengths")
    ap.add_argument("--async-dispatch", action="store_true",
                    help="step = earl_plan_build + earl_dispatch_async + earl_plan_get_summary "
                         "(no host wait between plan and dispatch)")
    ap.add_argument("--inverse", action="store_true",
                    help="time the reverse direction (earl_dispatch_inverse) instead of earl_dispatch")
    ap.add_argument("--path-histogram", action="store_true",
                    help="only print which path (plain copy, padding, straddling, ...) the bytes of "
                         "every field of --workload take")
    ap.add_argument("--copy-ceiling", action="store_true",
                    help="only time the plain-copy yardstick kernels (8 GiB) and print their rates")
    ap.add_argument("--reference-copy", action="store_true",
                    help="also run three plain 4 GiB device copies (for scaling profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the re-layout (all destination shards in one "
              "HBM); this library has no multi-GPU path: run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2510_05943_amd import binding as B
    from paper_2510_05943_amd import synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    B.load_library()
    torch.cuda.set_device(0)
    if args.copy_ceiling:
        print(json.dumps({"copy_ceiling": run_copy_ceiling(torch)}))
        return 0
    if args.path_histogram:
        print(json.dumps({"path_histogram": run_path_histogram(args, torch, B, synth)}))
        return 0
    hip = HipEvents()
    mode = "inverse" if args.inverse else ("async" if args.async_dispatch else "sync")

    if args.reference_copy:
        # a plain copy of known size on the same stream: the yardstick for the HBM counters
        n = 4 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        a.view(torch.int32).fill_(1)
        for _ in range(3):
            b.view(torch.int32).copy_(a.view(torch.int32))
        torch.cuda.synchronize()
        del a, b

    secondary = {}
    cpu = None
    if args.two_pass:
        w, sm, r, stage_s, row_bytes = run_two_pass(args, torch, B, synth, hip)
        kernel_name = "all kernels of both dispatches"
        traffic = None
    else:
        st = Staged(args.workload, args.seed, args.balance_policy, torch, B, synth)
        w, sm, stage_s, row_bytes = st.w, st.sm, st.stage_s, st.row_bytes
        r = st.measure(mode, args.steps, args.warmup, hip)
        kernel_name = ("inverse_code_kernel + inverse_kernel" if args.inverse else
                       "relayout_direct_kernel + tile_code_kernel + relayout_kernel")
        traffic = None if args.balance_policy else measured_traffic(
            args.workload, "inverse" if args.inverse else "forward")
        if not args.no_secondary and mode == "sync" and not args.balance_policy:
            secondary[args.workload + "_inverse"] = st.measure("inverse", args.steps, args.warmup, hip)
        if not args.no_cpu_baseline:
            cpu = run_cpu_baseline(args, synth, st.src)
        del st
        gc.collect()
        torch.cuda.empty_cache()
        if not args.no_secondary and mode == "sync" and not args.balance_policy:
            for name in ("longctx", "heavy", "mid", "agentic", "tiny"):
                if name == args.workload:
                    continue
                s2 = Staged(name, args.seed, 0, torch, B, synth)
                small = name in SMALL
                steps = max(args.steps, 200) if small else args.steps
                entry = s2.measure("sync", steps, max(args.warmup, 3), hip)
                entry["config"] = WORKLOAD_NOTES[name]
                entry["real_tokens"] = s2.sm["total_real_rows"]
                if small:
                    a2 = s2.measure("async", steps, max(args.warmup, 3), hip)
                    entry["ms_per_step_async"] = a2["ms_per_step"]
                    entry["tokens_per_s_async"] = a2["tokens_per_s"]
                    entry["kernels_ms_avg_async"] = a2["kernels_ms_avg"]
                    entry["note"] = ("cache-resident batch: latency-bound, frac is not an HBM figure; "
                                     "async = earl_plan_build + earl_dispatch_async + earl_plan_get_summary")
                secondary[name] = entry
                del s2
                gc.collect()
                torch.cuda.empty_cache()

    line = {
        "metric": "re-layout throughput: tokens/s and achieved HBM GB/s (% of peak) at 1 GPU",
        "value": sm["total_real_rows"] / (r["ms_per_step"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NOTES[args.workload], "name": args.workload,
                   "seed": args.seed, "n_seqs": w.n_seqs, "real_tokens": sm["total_real_rows"],
                   "dst_rows": sm["total_dst_rows"], "bytes_per_token_row": row_bytes,
                   "dst_shards": w.dp * w.sp, "src_shards": w.n_shards,
                   "balance_policy": args.balance_policy,
                   "step": ("two passes (gather to one buffer, scatter from it), each " if args.two_pass
                            else "") + ("earl_plan_build + earl_dispatch_async + earl_plan_get_summary"
                                        if args.async_dispatch else
                                        "earl_plan_build + earl_plan_get_summary + " +
                                        ("earl_dispatch_inverse" if args.inverse else "earl_dispatch"))},
        "whole_path_GBps": r["whole_path_GBps"],
        "roofline": {"bound": "hbm", "achieved": r["achieved_GBps"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": r["frac"], "traffic": traffic,
                     "kernel": kernel_name,
                     "interval": "HIP events around every kernel of the dispatch call (decode pass "
                                 "and copy), parameter upload excluded",
                     "algorithmic_bytes_per_launch": r["algorithmic_bytes"],
                     "kernel_ms_avg": r["kernels_ms_avg"], "kernel_ms_min": r["kernels_ms_min"],
                     "kernel_ms_median": r["kernels_ms_median"]},
        "input_staging_s": stage_s,
    }
    if "plan_ms" in r:
        line["plan_ms"] = r["plan_ms"]
        line["dispatch_ms"] = r["dispatch_ms"]
    if secondary:
        line["secondary"] = secondary
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu if cpu is not None else run_cpu_baseline(args, synth)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())

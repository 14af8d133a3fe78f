#!/usr/bin/env python3
"""Benchmark of the LowDiff hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic gradients:

  sparse leg (GPT-2-XL-shaped, 1.56 B fp32 parameters, 580 segments, rho = 1 %):
      W = 20 chained ld_compress_topk calls (error-feedback residual carried from
      call to call) followed by one ld_merge_sparse of the 20-diff window;
  dense leg (Llama-7B-shaped, 6.74 B parameters, fp32 w/m/v, bf16 gradients):
      W = 4 iterations of layer-wise snapshots - one ld_snapshot_layers call per model
      layer as its gradient becomes available in the backward pass (head + final norm,
      32 transformer layers of 9 tensors each, embedding: 34 calls, 291 tensors) -
      followed by one fused ld_merge_dense_adam of the 4 snapshots.

All inputs are resident in HBM before the timed region.  State (residual, w, m, v)
is carried from step to step, as in training: nothing is restored inside the
timed region.  `value` is gradient bytes turned into (and merged from)
differential checkpoints per second over the whole step.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2509_04084_amd import lowdiff as ld  # noqa: E402
from paper_2509_04084_amd import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Timer:
    """HIP-event pairs on the current stream (the stream the library launches on)."""

    def __init__(self):
        self.pairs = {}

    def start(self, name):
        e0 = torch.cuda.Event(enable_timing=True)
        e0.record()
        return name, e0

    def stop(self, tok):
        name, e0 = tok
        e1 = torch.cuda.Event(enable_timing=True)
        e1.record()
        self.pairs.setdefault(name, []).append((e0, e1))

    def ms(self):
        return {k: [a.elapsed_time(b) for a, b in v] for k, v in self.pairs.items()}


class SparseLeg:
    def __init__(self, wl, dev, pool):
        self.wl, self.dev = wl, dev
        self.off, self.k = wl.seg_off, wl.seg_k
        self.n, self.W = wl.n, wl.window
        self.K = int(self.k.astype(np.int64).sum())
        log(f"[sparse] {wl.name}: n={self.n:,} segs={len(wl.sizes)} K={self.K:,} W={self.W} pool={pool}")
        self.grads = [synth.gradient(wl, t, device=dev) for t in range(pool)]
        self.r = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.w = synth.base_weights(self.n, device=dev, std=wl.w_std)
        self.idx = [torch.empty(self.K, dtype=torch.int32, device=dev) for _ in range(self.W)]
        self.val = [torch.empty(self.K, dtype=torch.float32, device=dev) for _ in range(self.W)]
        self.ws_c = torch.empty(ld.ld_compress_topk_workspace(self.off), dtype=torch.uint8, device=dev)
        self.ws_m = torch.empty(ld.ld_merge_sparse_workspace(self.n, [self.K] * self.W), dtype=torch.uint8,
                                device=dev)
        self.it = 0

    def step(self, tm):
        for t in range(self.W):
            g = self.grads[self.it % len(self.grads)]
            tok = tm.start("compress")
            ld.ld_compress_topk(g, self.r, self.off, self.k, self.idx[t], self.val[t], self.ws_c)
            tm.stop(tok)
            self.it += 1
        tok = tm.start("merge_sparse")
        ld.ld_merge_sparse(self.w, self.idx, self.val, self.wl.lr, self.ws_m)
        tm.stop(tok)

    # algorithmic bytes per call
    def bytes_compress(self):
        return 12 * self.n + 8 * self.K

    def bytes_merge(self):
        return 8 * self.n + 8 * self.K * self.W

    # -- next row: the same window replayed through Adam on (w, m, v); timed on its own, after the
    #    timed steps, and not part of `value`
    def time_sparse_adam(self, reps=3):
        m = torch.zeros(self.n, dtype=torch.float32, device=self.dev)
        v = torch.zeros(self.n, dtype=torch.float32, device=self.dev)
        ws = torch.empty(ld.ld_merge_sparse_adam_workspace(self.n, [self.K] * self.W), dtype=torch.uint8,
                         device=self.dev)
        tm = Timer()
        for i in range(reps + 1):
            tok = tm.start("sparse_adam")
            ld.ld_merge_sparse_adam(self.w, m, v, self.idx, self.val, i * self.W, 1e-4, workspace=ws, **synth.ADAM)
            tm.stop(tok)
        torch.cuda.synchronize()
        return float(np.mean(tm.ms()["sparse_adam"][1:]))

    # -- next row: the first 8 diffs of the window taken as the record lists of 8 workers (a stand-in:
    #    same shapes and density as 8 workers' top-k lists) and combined into one synchronized diff
    def time_combine(self, workers=8, reps=3):
        idx, val = self.idx[:workers], self.val[:workers]
        total = sum(t.numel() for t in idx)
        out_i = torch.empty(total, dtype=torch.int32, device=self.dev)
        out_v = torch.empty(total, dtype=torch.float32, device=self.dev)
        cnt = torch.zeros(1, dtype=torch.int64, device=self.dev)
        ws = torch.empty(ld.ld_combine_sparse_workspace(self.n, workers), dtype=torch.uint8, device=self.dev)
        tm = Timer()
        for i in range(reps + 1):
            tok = tm.start("combine")
            ld.ld_combine_sparse(idx, val, self.n, 1.0 / workers, out_i, out_v, cnt, ws)
            tm.stop(tok)
        torch.cuda.synchronize()
        return float(np.mean(tm.ms()["combine"][1:])), total, int(cnt.item())

    # -- next row: the window's diffs in page-locked host memory, merged as they arrive (pipelined
    #    recovery); wall-clock from the first copy to the end of the last merge
    def time_recovery_from_host(self, group=5, reps=2):
        hi = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t) for t in self.idx]
        hv = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t) for t in self.val]
        K = np.array([t.numel() for t in hi], dtype=np.int64)
        lib = ld.load()
        out = {}
        cs, ms = torch.cuda.Stream(), torch.cuda.Stream()
        for name, g in (("pipelined", group), ("copy_then_merge", min(self.W, 64))):
            staging = torch.empty(int(lib.ld_merge_sparse_from_host_staging(K.ctypes.data, self.W, g)),
                                  dtype=torch.uint8, device=self.dev)
            times = []
            for _ in range(reps + 1):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ld.ld_merge_sparse_from_host(self.w, hi, hv, self.wl.lr, group=g, staging=staging,
                                             copy_stream=cs, merge_stream=ms)
                cs.synchronize()
                ms.synchronize()
                times.append((time.perf_counter() - t0) * 1e3)
            out[name] = float(np.mean(times[1:]))
            del staging
        return out, int(8 * K.sum())

    def bytes_sparse_adam(self):
        return 24 * self.n + 8 * self.K * self.W

    def flops_sparse_adam(self):
        return 14 * self.n * self.W  # per element and step: 3 (m) + 4 (v) + 3 (root, eps) + 3 (update) + 1

    def grad_bytes(self):
        return 4 * self.n * self.W


class DenseLeg:
    def __init__(self, wl, dev, n_src=2):
        self.wl, self.dev = wl, dev
        self.n, self.W = wl.n, wl.window
        self.off = wl.seg_off
        log(f"[dense] {wl.name}: n={self.n:,} layers={len(wl.sizes)} W={self.W}")
        self.src = []
        for t in range(n_src):
            g = torch.empty(self.n, dtype=torch.bfloat16, device=dev)
            for s in range(len(wl.sizes)):  # layer by layer: bounds the fp32 temporary
                lo, hi = int(self.off[s]), int(self.off[s + 1])
                g[lo:hi] = synth.gradient_layer_bf16(wl, t, s, dev)
            self.src.append(g)
        self.snap = [torch.empty(self.n, dtype=torch.bfloat16, device=dev) for _ in range(self.W)]
        self.w = synth.base_weights(self.n, device=dev, std=wl.w_std)
        self.m = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.v = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.layers = [(int(self.off[s]), int(self.off[s + 1])) for s in range(len(wl.sizes))]
        # model layers: embedding | 32 x (q, k, v, o, gate, up, down, 2 norms) | final norm + head;
        # backward order: the last layer's gradient exists first
        nt = len(self.layers)
        groups = [[0]] + [list(range(1 + 9 * b, 10 + 9 * b)) for b in range((nt - 3) // 9)] + [[nt - 2, nt - 1]]
        self.groups = list(reversed(groups))
        self.src_views = [[[g[self.layers[s][0]:self.layers[s][1]] for s in grp] for grp in self.groups]
                          for g in self.src]
        self.snap_views = [[[g[self.layers[s][0]:self.layers[s][1]] for s in grp] for grp in self.groups]
                           for g in self.snap]
        self.step0 = 0
        self.it = 0

    def step(self, tm):
        for t in range(self.W):
            sv = self.src_views[self.it % len(self.src)]
            dv = self.snap_views[t]
            tok = tm.start("snapshot_iter")
            for a, b in zip(sv, dv):
                ld.ld_snapshot_layers(a, b)
            tm.stop(tok)
            self.it += 1
        tok = tm.start("adam")
        ld.ld_merge_dense_adam(self.w, self.m, self.v, self.snap, self.step0, self.wl.lr, **synth.ADAM)
        tm.stop(tok)
        self.step0 += self.W

    # -- next row: the paper's snapshot destination, pinned host memory (bound by the host link, not HBM)
    def time_snapshot_to_host(self, reps=3):
        lo, hi = self.layers[-1]  # the head: 131 M elements, 262 MB
        src = self.src[0][lo:hi]
        dst = torch.empty(hi - lo, dtype=torch.bfloat16).pin_memory()
        tm = Timer()
        for _ in range(reps + 1):
            tok = tm.start("to_host")
            ld.ld_snapshot_layer(src, dst)
            tm.stop(tok)
        torch.cuda.synchronize()
        return float(np.mean(tm.ms()["to_host"][1:])), 2 * (hi - lo)

    def bytes_snapshot_iter(self):
        return 4 * self.n

    def bytes_adam(self):
        return (24 + 2 * self.W) * self.n

    def grad_bytes(self):
        return 2 * self.n * self.W


class CopyCal:
    """A plain copy of known size (1 GiB in, 1 GiB out) through ld_snapshot_layer: the yardstick the
    FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by."""

    def __init__(self, dev):
        self.n = 1 << 29  # bf16 elements
        self.src = torch.randint(-30000, 30000, (self.n,), dtype=torch.int16, device=dev).view(torch.bfloat16)
        self.dst = torch.empty_like(self.src)

    def step(self, tm):
        tok = tm.start("copycal")
        ld.ld_snapshot_layer(self.src, self.dst)
        tm.stop(tok)


def measured_traffic(path):
    """HBM bytes per call from the committed counter summary (lines 'traffic <entry> <bytes>')."""
    out = {}
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic":
                    out[parts[1]] = int(float(parts[2]))
    except OSError:
        pass
    return out


def cpu_baseline():
    """The CPU oracle, as it stands (single thread), on a bounded sample of the same workload:
    about 10-20 s of host work, extrapolated to the full step by gradient bytes."""
    import oracle
    xl, ll = synth.workload("gpt2xl"), synth.workload("llama7b")
    # sparse: the four weight matrices of two transformer blocks (61 M elements), 10 chained diffs
    segs = [4, 6, 10, 12, 16, 18, 22, 24]
    sizes = [xl.sizes[s] for s in segs]
    off, k = synth.seg_offsets(sizes), synth.seg_topk(sizes, *xl.rho)
    n = int(off[-1])
    Wc = 10
    grads = []
    for t in range(Wc):
        g = np.empty(n, np.float32)
        for j, s in enumerate(segs):
            g[off[j]:off[j + 1]] = synth.gradient_segment(xl, t, s, "cpu").numpy()
        grads.append(g)
    w0 = synth.base_weights(n).numpy()
    t0 = time.perf_counter()
    r = np.zeros(n, np.float32)
    idxs, vals = [], []
    for g in grads:
        i, v, r = oracle.topk_ef(g, r, off, k, select=True)
        idxs.append(i)
        vals.append(v)
    oracle.merge_sparse(w0, idxs, vals, xl.lr)
    t_sparse = time.perf_counter() - t0
    sparse_bytes = 4 * n * Wc
    del grads
    # dense: the seven weight matrices of the first block (202 M elements), W = 4
    dsegs = [1, 2, 3, 4, 5, 6, 7]
    Wd = ll.window
    t_dense, nd = 0.0, 0
    for s in dsegs:
        ns = ll.sizes[s]
        gs = [synth.gradient_layer_bf16(ll, t, s, "cpu").view(torch.int16).numpy().view(np.uint16) for t in range(Wd)]
        wd = synth.base_weights(ns).numpy()
        z = np.zeros(ns, np.float32)
        t0 = time.perf_counter()
        snaps = [oracle.snapshot(g) for g in gs]
        oracle.adam_replay(wd, z, z, snaps, 0, ll.lr, **synth.ADAM)
        t_dense += time.perf_counter() - t0
        nd += ns
    dense_bytes = 2 * nd * Wd
    # weight the two legs as the full step does (gradient bytes of each leg)
    full_sparse = 4 * xl.n * xl.window
    full_dense = 2 * ll.n * ll.window
    est_full_s = t_sparse * full_sparse / sparse_bytes + t_dense * full_dense / dense_bytes
    value = (full_sparse + full_dense) / est_full_s / 1e9
    return {
        "value": value, "unit": "GB/s (gradient bytes)", "cores": 1, "kind": "oracle",
        "sample": (f"gpt2xl segments {segs} ({n:,} elements), {Wc} chained top-k (nth_element variant) + "
                   f"window merge: {t_sparse:.2f} s; llama7b layers {dsegs} ({nd:,} elements), snapshot + Adam "
                   f"replay W={Wd}: {t_dense:.2f} s; extrapolated to the full step by gradient bytes"),
        "sparse_GBps": sparse_bytes / t_sparse / 1e9, "dense_GBps": dense_bytes / t_dense / 1e9,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--pool", type=int, default=10, help="distinct gradients cycled by the sparse leg")
    ap.add_argument("--sparse", default="gpt2xl")
    ap.add_argument("--dense", default="llama7b")
    ap.add_argument("--legs", default="sparse,dense",
                    help="comma list of sparse, dense, copycal (copycal: a 1 GiB plain copy, for counter calibration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true", help="skip the calls measured outside the step")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ld.load()
    legs = args.legs.split(",")
    t_setup = time.perf_counter()
    sparse = SparseLeg(synth.workload(args.sparse), dev, args.pool) if "sparse" in legs else None
    dense = DenseLeg(synth.workload(args.dense), dev) if "dense" in legs else None
    copycal = CopyCal(dev) if "copycal" in legs else None
    torch.cuda.synchronize()
    log(f"[setup] {time.perf_counter() - t_setup:.1f} s, {torch.cuda.memory_allocated() / 1e9:.1f} GB resident")

    def one_step(tm):
        if sparse:
            sparse.step(tm)
        if dense:
            dense.step(tm)
        if copycal:
            copycal.step(tm)

    for i in range(args.warmup):
        one_step(Timer())
        torch.cuda.synchronize()
        log(f"[warmup] {i + 1}/{args.warmup}")
    tm = Timer()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(tm)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    per = {k: float(np.mean(v)) for k, v in tm.ms().items()}
    log(f"[timed] {args.steps} steps, {ms_per_step:.2f} ms/step; mean ms per call: {per}")

    grad_bytes = (sparse.grad_bytes() if sparse else 0) + (dense.grad_bytes() if dense else 0)
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    def roof(name, nbytes):
        ach = nbytes / (per[name] * 1e-3) / 1e9
        return {"ms": per[name], "algorithmic_bytes": nbytes, "achieved_GBps": ach, "frac": ach / HBM_PEAK_GBS}

    calls = {}
    if sparse:
        calls["ld_compress_topk"] = roof("compress", sparse.bytes_compress())
        calls["ld_merge_sparse"] = roof("merge_sparse", sparse.bytes_merge())
        calls["ld_compress_topk"]["grad_GBps"] = 4 * sparse.n / (per["compress"] * 1e-3) / 1e9
        calls["ld_merge_sparse"]["grad_GBps"] = 4 * sparse.n * sparse.W / (per["merge_sparse"] * 1e-3) / 1e9
    if dense:
        calls["ld_snapshot_layers(x34)"] = roof("snapshot_iter", dense.bytes_snapshot_iter())
        calls["ld_merge_dense_adam"] = roof("adam", dense.bytes_adam())
    # the call that takes the largest share of the step
    share = {}
    if sparse:
        share["ld_compress_topk"] = per["compress"] * sparse.W
        share["ld_merge_sparse"] = per["merge_sparse"]
    if dense:
        share["ld_snapshot_layers(x34)"] = per["snapshot_iter"] * dense.W
        share["ld_merge_dense_adam"] = per["adam"]
    if copycal:
        calls["copycal(ld_snapshot_layer, 1 GiB)"] = roof("copycal", 4 * copycal.n)
    next_rows = {}
    if sparse and not args.no_next_rows:
        ms = sparse.time_sparse_adam()
        log(f"[next row] ld_merge_sparse_adam: {ms:.2f} ms per call (W={sparse.W})")
        tf = sparse.flops_sparse_adam() / (ms * 1e-3) / 1e12
        next_rows["ld_merge_sparse_adam"] = {
            "ms": ms, "algorithmic_bytes": sparse.bytes_sparse_adam(),
            "hbm_GBps": sparse.bytes_sparse_adam() / (ms * 1e-3) / 1e9,
            "hbm_frac": sparse.bytes_sparse_adam() / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "roofline": {"bound": "alu", "achieved": tf, "peak": 157.3, "unit": "TFLOP/s", "frac": tf / 157.3,
                         "note": "14 flops per element and step; peak = fp32 vector rate with packed FMA"},
            "note": "same gpt2xl window replayed through Adam on (w, m, v); not part of `value`"}
        ms, k_in, k_out = sparse.time_combine()
        log(f"[next row] ld_combine_sparse: {ms:.3f} ms per call (8 lists, {k_in:,} records -> {k_out:,})")
        nb = 8 * k_in + 8 * k_out
        next_rows["ld_combine_sparse"] = {
            "ms": ms, "algorithmic_bytes": nb, "records_in": k_in, "records_out": k_out,
            "roofline": {"bound": "hbm", "achieved": nb / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "note": "8 B per input record + 8 B per output record"},
            "note": "8 of the window's diffs taken as 8 workers' lists; not part of `value`"}
        rec, nb = sparse.time_recovery_from_host()
        log(f"[next row] ld_merge_sparse_from_host: {rec['pipelined']:.1f} ms pipelined, "
            f"{rec['copy_then_merge']:.1f} ms copy-then-merge ({nb / 1e6:.0f} MB of records over the host link)")
        next_rows["ld_merge_sparse_from_host"] = {
            "ms": rec["pipelined"], "ms_copy_then_merge": rec["copy_then_merge"], "record_bytes": nb,
            "host_link_GBps": nb / (rec["pipelined"] * 1e-3) / 1e9,
            "note": "the window's 20 diffs in page-locked host memory, copied in groups of 5 on one stream while "
                    "the previous group is merged on another; wall-clock; bound by the host link; not part of `value`"}
    if dense and not args.no_next_rows:
        ms, nb = dense.time_snapshot_to_host()
        log(f"[next row] ld_snapshot_layer into pinned host memory: {ms:.2f} ms for {nb / 1e6:.0f} MB")
        next_rows["ld_snapshot_layer(to pinned host)"] = {
            "ms": ms, "bytes": nb, "GBps": nb / (ms * 1e-3) / 1e9,
            "note": "one 131 M-element layer copied by the same kernel into page-locked host memory: bound by the "
                    "host link; not part of `value`"}
    if not share:
        print(json.dumps({"calls": calls}), flush=True)
        return
    dom = max(share, key=share.get)
    # the committed counter summary was taken on the default workloads: it says nothing about others
    traffic = {}
    if args.sparse == "gpt2xl" and args.dense == "llama7b":
        traffic = measured_traffic(os.path.join(ROOT, "profiles", "hbm_traffic_gpt2xl_llama7b.txt"))
    for name, c in calls.items():
        c["traffic_bytes"] = traffic.get(name.split("(")[0])
    roofline = {"bound": "hbm", "kernel": dom, "achieved": calls[dom]["achieved_GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": calls[dom]["frac"], "traffic": calls[dom]["traffic_bytes"],
                "note": "per call of the entry point (all its kernels), HIP events on the launch stream; "
                        "traffic = HBM bytes per call from rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by "
                        "what the same counter reads for a 1 GiB plain copy (profiles/)"}
    if dense:
        # the layer snapshots are plain copies: what a copy kernel reaches on this machine in this run
        roofline["plain_copy_GBps"] = calls["ld_snapshot_layers(x34)"]["achieved_GBps"]
    out = {
        "metric": "diff-build GB/s + merge GB/s (grad bytes), % of MI355X HBM roofline",
        "value": value, "unit": "GB/s (gradient bytes)", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "+".join(x for x in (args.sparse if sparse else None,
                                                    args.dense if dense else None) if x),
                   "sparse": (f"{args.sparse}: n={sparse.n} segs={len(sparse.wl.sizes)} "
                              f"rho={100.0 * sparse.wl.rho[0] / sparse.wl.rho[1]:g}% W={sparse.W} "
                              f"chained compress + window merge") if sparse else None,
                   "dense": (f"{args.dense}: n={dense.n} layers={len(dense.wl.sizes)} W={dense.W} "
                             f"snapshots per model layer ({len(dense.groups)} calls) + fused Adam replay") if dense else None},
        "roofline": roofline, "calls": calls,
    }
    if next_rows:
        out["next_rows"] = next_rows
    if not args.no_cpu_baseline:
        log("[cpu_baseline] timing the oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

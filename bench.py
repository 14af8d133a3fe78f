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

After the timed steps, outside the timed region: the outputs are verified (properties on the
last timed step's records and snapshots, then one more step of the same buffers and launch
configuration with the state saved before its last calls, checked against the CPU oracle on
sampled segments, slices and layers: "verified" in the line, non-zero exit on a mismatch); the
next rows, the small configurations and the configuration model are measured; the CPU oracle is
timed on a bounded sample (one thread, then all cores).

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import concurrent.futures
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


def bits(t):
    return t.view(torch.int32)


def np_bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


class VerifyError(AssertionError):
    pass


def require(cond, what):
    if not bool(cond):
        raise VerifyError(what)


def stats(ms_list):
    a = np.asarray(ms_list, dtype=np.float64)
    return {"ms": float(a.mean()), "ms_median": float(np.median(a)), "ms_min": float(a.min()), "calls_timed": int(a.size)}


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
        self.ws_c = torch.empty(ld.ld_compress_topk_workspace(self.off, self.k), dtype=torch.uint8, device=dev)
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


    # -- verification (outside the timed region)
    def _seg_tables(self):
        k64 = torch.from_numpy(self.k.astype(np.int64)).to(self.dev)
        seg_of_rec = torch.repeat_interleave(torch.arange(len(self.k), device=self.dev), k64)
        off_t = torch.from_numpy(np.asarray(self.off, np.int64)).to(self.dev)
        return seg_of_rec, off_t

    def _check_records(self, idx, seg_of_rec, off_t, what):
        i64 = idx.to(torch.int64)
        require(idx.numel() == self.K, f"{what}: record count")
        require((i64[1:] > i64[:-1]).all(), f"{what}: indices not strictly ascending")
        require((i64 >= off_t[seg_of_rec]).all() and (i64 < off_t[seg_of_rec + 1]).all(),
                f"{what}: a record lies outside its segment")
        return i64

    def _check_threshold(self, i64, val, seg_of_rec, what):
        n_seg = len(self.k)
        require((self.r[i64] == 0).all() and not torch.signbit(self.r[i64]).any(), f"{what}: selected residual is not +0")
        min_sel = torch.full((n_seg,), float("inf"), device=self.dev).scatter_reduce(
            0, seg_of_rec, val.abs(), reduce="amin", include_self=True)
        seg_of_elem_max = torch.zeros(n_seg, device=self.dev)
        for s0 in range(n_seg):  # per-segment max of what was left behind
            lo, hi = int(self.off[s0]), int(self.off[s0 + 1])
            if hi > lo:
                seg_of_elem_max[s0] = self.r[lo:hi].abs().max()
        require((seg_of_elem_max <= min_sel).all(), f"{what}: an unselected magnitude exceeds a selected one")

    def verify(self):
        """Checks the last timed step's outputs by properties, then runs one more step (same buffers,
        same launch configuration) with the state saved before its last compress call and before its
        merge, and checks that step against the definition and the CPU oracle. Raises VerifyError."""
        import oracle
        seg_of_rec, off_t = self._seg_tables()
        # (1) the window the last timed step left behind: every diff well-formed; the last call's
        #     threshold property against the residual as it stands
        for t in range(self.W):
            i64 = self._check_records(self.idx[t], seg_of_rec, off_t, f"timed step, diff {t}")
        self._check_threshold(i64, self.val[self.W - 1], seg_of_rec, "timed step, last diff")
        # (2) one more step with saved state
        for t in range(self.W - 1):
            g = self.grads[self.it % len(self.grads)]
            ld.ld_compress_topk(g, self.r, self.off, self.k, self.idx[t], self.val[t], self.ws_c)
            self.it += 1
        r_before = self.r.clone()
        g = self.grads[self.it % len(self.grads)]
        t = self.W - 1
        ld.ld_compress_topk(g, self.r, self.off, self.k, self.idx[t], self.val[t], self.ws_c)
        self.it += 1
        w_before = self.w.clone()
        ld.ld_merge_sparse(self.w, self.idx, self.val, self.wl.lr, self.ws_m)
        torch.cuda.synchronize()
        idx, val = self.idx[t], self.val[t]
        i64 = self._check_records(idx, seg_of_rec, off_t, "verification step, last diff")
        a = r_before + g  # one fp32 add per element: the definition's accumulation
        require(torch.equal(bits(val), bits(a[i64])), "val is not r + g bit for bit")
        self._check_threshold(i64, val, seg_of_rec, "verification step, last diff")
        a[i64] = 0.0
        require(torch.equal(bits(a), bits(self.r)), "residual is not r + g with the selected positions zeroed")
        del a
        # the oracle on sampled segments: two small ones, one of every large shape, the last
        n_seg = len(self.k)
        out0 = np.concatenate([[0], np.cumsum(self.k.astype(np.int64))])
        by_size = {}
        for s0 in range(n_seg):
            by_size.setdefault(int(self.off[s0 + 1] - self.off[s0]), s0)
        sample = sorted(set(list(by_size.values())[:12]) | {n_seg - 1})
        sample = [s0 for s0 in sample if self.off[s0 + 1] - self.off[s0] <= 12_000_000][:8]
        for s0 in sample:
            lo, hi = int(self.off[s0]), int(self.off[s0 + 1])
            oi, ov, orr = oracle.topk_ef(g[lo:hi].cpu().numpy(), r_before[lo:hi].cpu().numpy(),
                                         np.array([0, hi - lo], np.int64), self.k[s0:s0 + 1], select=True)
            o0, o1 = int(out0[s0]), int(out0[s0 + 1])
            require(np.array_equal(idx[o0:o1].cpu().numpy(), oi + lo), f"oracle: idx of segment {s0}")
            require(np.array_equal(np_bits(val[o0:o1].cpu().numpy()), np_bits(ov)), f"oracle: val of segment {s0}")
            require(np.array_equal(np_bits(self.r[lo:hi].cpu().numpy()), np_bits(orr)), f"oracle: residual of segment {s0}")
        del r_before
        # the merge: the per-record definition redone with torch on the whole array, the oracle on slices
        n = self.n
        m_len = min(n, 2_000_000)
        slices = [(0, m_len), (max(0, n // 2 - m_len // 2), max(0, n // 2 - m_len // 2) + m_len), (n - m_len, n)]
        for (a0, b0) in slices:
            sub_i, sub_v = [], []
            for i_t, v_t in zip(self.idx, self.val):
                p0 = int(torch.searchsorted(i_t.to(torch.int64), torch.tensor([a0], dtype=torch.int64, device=self.dev)))
                p1 = int(torch.searchsorted(i_t.to(torch.int64), torch.tensor([b0], dtype=torch.int64, device=self.dev)))
                sub_i.append((i_t[p0:p1].cpu().numpy().astype(np.int64) - a0).astype(np.int32))
                sub_v.append(v_t[p0:p1].cpu().numpy())
            ref = oracle.merge_sparse(w_before[a0:b0].cpu().numpy(), sub_i, sub_v, self.wl.lr)
            require(np.array_equal(np_bits(self.w[a0:b0].cpu().numpy()), np_bits(ref)), f"oracle: merged w[{a0}:{b0}]")
        lr_t = torch.tensor(self.wl.lr, dtype=torch.float32, device=self.dev)
        for i_t, v_t in zip(self.idx, self.val):
            j = i_t.to(torch.int64)
            w_before[j] = w_before[j] - lr_t * v_t   # rounded product, then rounded difference
            del j
        require(torch.equal(bits(self.w), bits(w_before)), "merged w differs from the per-record definition")
        return {"sampled_segments": [int(x) for x in sample], "merge_slices": slices}

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


    # -- verification (outside the timed region)
    def verify(self):
        """The last timed step's snapshots against their sources, bit for bit; then one more step with
        slices of (w, m, v) saved first, checked against the CPU oracle within the Adam tolerance."""
        import oracle
        for t in range(self.W):
            src = self.src[(self.it - self.W + t) % len(self.src)]
            require(torch.equal(src.view(torch.int16), self.snap[t].view(torch.int16)), f"snapshot {t} differs from its source")
        nt = len(self.layers)
        checked = sorted({0, 1, 5, 7, 8, nt - 2, nt - 1})
        saved = []
        for s0 in checked:
            lo, hi = self.layers[s0]
            hi = min(hi, lo + 2_000_000)
            saved.append((lo, hi, self.w[lo:hi].cpu().numpy(), self.m[lo:hi].cpu().numpy(), self.v[lo:hi].cpu().numpy()))
        step0 = self.step0
        self.step(Timer())
        torch.cuda.synchronize()
        for t in range(self.W):
            src = self.src[(self.it - self.W + t) % len(self.src)]
            require(torch.equal(src.view(torch.int16), self.snap[t].view(torch.int16)), f"snapshot {t} differs from its source")
        for lo, hi, w0, m0, v0 in saved:
            gs = [sn[lo:hi].view(torch.int16).cpu().numpy().view(np.uint16) for sn in self.snap]
            wr, mr, vr = oracle.adam_replay(w0, m0, v0, gs, step0, self.wl.lr, **synth.ADAM)
            for name, got, ref in (("w", self.w, wr), ("m", self.m, mr), ("v", self.v, vr)):
                x = got[lo:hi].cpu().numpy().astype(np.float64)
                require(np.all(np.abs(x - ref) <= 1e-7 + 1e-6 * np.abs(ref)), f"oracle: Adam {name}[{lo}:{hi}]")
            xv = self.v[lo:hi].cpu().numpy().astype(np.float64)
            require(np.all(np.abs(xv - vr) <= 2e-6 * np.abs(vr)), f"oracle: Adam v[{lo}:{hi}], relative")
        return {"sampled_layers": [int(x) for x in checked], "adam_step0": int(step0)}

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

    def time_adam_incremental(self):
        """The replay as LowDiff+ runs it (Sec. VI-A): one call per iteration's gradient, (w, m, v)
        read and written every time: 26 n bytes per step where the fused window moves (24 + 2 W) n
        for W steps. Returns ms per single-step call (mean over the window's W calls, after one
        untimed call)."""
        tm = Timer()
        for t in range(self.W + 1):
            tok = tm.start("adam1")
            ld.ld_merge_dense_adam(self.w, self.m, self.v, [self.snap[t % self.W]], self.step0, self.wl.lr, **synth.ADAM)
            tm.stop(tok)
            self.step0 += 1
        torch.cuda.synchronize()
        return float(np.mean(tm.ms()["adam1"][1:]))

    def bytes_snapshot_iter(self):
        return 4 * self.n

    def bytes_adam(self):
        return (24 + 2 * self.W) * self.n

    def grad_bytes(self):
        return 2 * self.n * self.W


class MergeOnlyLeg:
    """The window merge of a sparse workload on its own, for profiling runs: W random ascending index
    lists of (up to) K records each with values of the workload's scale, no compress calls."""

    def __init__(self, wl, dev):
        self.wl, self.dev, self.n, self.W = wl, dev, wl.n, wl.window
        K = int(wl.seg_k.astype(np.int64).sum())
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        self.idx, self.val = [], []
        for _ in range(self.W):
            i = torch.unique_consecutive(torch.sort(torch.randint(0, self.n, (K,), device=dev, generator=gen)).values)
            self.idx.append(i.to(torch.int32))
            self.val.append(torch.randn(i.numel(), device=dev, generator=gen) * wl.scale)
        self.records = sum(t.numel() for t in self.idx)
        self.w = torch.randn(self.n, device=dev, generator=gen) * wl.w_std
        self.ws = torch.empty(ld.ld_merge_sparse_workspace(self.n, [t.numel() for t in self.idx]), dtype=torch.uint8,
                              device=dev)
        log(f"[mergeonly] {wl.name}: n={self.n:,} W={self.W} records={self.records:,}")

    def step(self, tm):
        tok = tm.start("merge_only")
        ld.ld_merge_sparse(self.w, self.idx, self.val, self.wl.lr, self.ws)
        tm.stop(tok)

    def bytes_merge(self):
        return 8 * self.n + 8 * self.records


class CombineOnlyLeg:
    """ld_combine_sparse on its own, for profiling runs: `workers` random ascending lists of (up to) K
    records each, as many workers' top-k lists of the sparse workload's shape and density."""

    def __init__(self, wl, dev, workers=8):
        self.n, self.workers = wl.n, workers
        K = int(wl.seg_k.astype(np.int64).sum())
        gen = torch.Generator(device=dev)
        gen.manual_seed(11)
        self.idx, self.val = [], []
        for _ in range(workers):
            i = torch.unique_consecutive(torch.sort(torch.randint(0, self.n, (K,), device=dev, generator=gen)).values)
            self.idx.append(i.to(torch.int32))
            self.val.append(torch.randn(i.numel(), device=dev, generator=gen) * wl.scale)
        self.records = sum(t.numel() for t in self.idx)
        self.out_i = torch.empty(self.records, dtype=torch.int32, device=dev)
        self.out_v = torch.empty(self.records, dtype=torch.float32, device=dev)
        self.cnt = torch.zeros(1, dtype=torch.int64, device=dev)
        self.ws = torch.empty(ld.ld_combine_sparse_workspace(self.n, workers), dtype=torch.uint8, device=dev)
        log(f"[combineonly] {wl.name}: n={self.n:,} lists={workers} records={self.records:,}")

    def step(self, tm):
        tok = tm.start("combine_only")
        ld.ld_combine_sparse(self.idx, self.val, self.n, 1.0 / self.workers, self.out_i, self.out_v, self.cnt, self.ws)
        tm.stop(tok)

    def bytes_combine(self):
        return 8 * (self.records + int(self.cnt.item()))


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


def host_cores():
    """(threads the all-core leg uses, logical CPUs this process may run on, CPU model string)."""
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return max(1, min(avail, 16)), avail, model  # a one-GPU machine's CPU share is 16 threads whatever nproc says


def cpu_baseline(gen_dev="cpu"):
    """The CPU oracle, as it stands, on a bounded sample of the same workload (about 20 s of host
    work), extrapolated to the full step by gradient bytes: once on one thread, once on all cores
    (threads of this harness over independent segments / parameter ranges; the oracle itself stays
    single-threaded and untouched). The inputs are drawn on `gen_dev` (the GPU when there is one:
    drawing 2.5 G Student-t values is what would take minutes on the host) and handed over as host arrays."""
    import oracle
    threads, avail, model = host_cores()
    xl, ll = synth.workload("gpt2xl"), synth.workload("llama7b")
    Wc, Wd = 10, ll.window

    def sparse_inputs(segs):
        out = []
        for s in segs:
            ns = xl.sizes[s]
            gs = [synth.gradient_segment(xl, t, s, gen_dev).cpu().numpy() for t in range(Wc)]
            out.append((ns, gs, synth.base_weights(ns, gen_dev).cpu().numpy()))
        return out

    def sparse_chain(item):  # one segment: Wc chained top-k calls and the merge of its window
        ns, gs, w0 = item
        off, k = np.array([0, ns], np.int64), synth.seg_topk([ns], *xl.rho)
        r = np.zeros(ns, np.float32)
        idxs, vals = [], []
        for g in gs:
            i, v, r = oracle.topk_ef(g, r, off, k, select=True)
            idxs.append(i)
            vals.append(v)
        oracle.merge_sparse(w0, idxs, vals, xl.lr)

    def dense_inputs(layers, parts):
        out = []
        for s in layers:
            ns = ll.sizes[s]
            gs = [synth.gradient_layer_bf16(ll, t, s, gen_dev).view(torch.int16).cpu().numpy().view(np.uint16)
                  for t in range(Wd)]
            wd = synth.base_weights(ns, gen_dev).cpu().numpy()
            cut = np.linspace(0, ns, parts + 1).astype(np.int64)
            for a0, b0 in zip(cut[:-1], cut[1:]):
                out.append((wd[a0:b0], [g[a0:b0] for g in gs]))
        return out

    def dense_range(item):  # one parameter range: W snapshots and the Adam replay over them
        wd, gs = item
        z = np.zeros(wd.size, np.float32)
        snaps = [oracle.snapshot(g) for g in gs]
        oracle.adam_replay(wd, z, z, snaps, 0, ll.lr, **synth.ADAM)

    def timed(fn, items, nthreads):
        t0 = time.perf_counter()
        if nthreads == 1:
            for it in items:
                fn(it)
        else:  # ctypes releases the interpreter lock while the oracle runs
            with concurrent.futures.ThreadPoolExecutor(nthreads) as ex:
                list(ex.map(fn, items))
        return time.perf_counter() - t0

    full_sparse = 4 * xl.n * xl.window
    full_dense = 2 * ll.n * ll.window

    def extrapolate(t_sparse, n_sparse, t_dense, n_dense):
        sb, db = 4 * n_sparse * Wc, 2 * n_dense * Wd
        est = t_sparse * full_sparse / sb + t_dense * full_dense / db
        return (full_sparse + full_dense) / est / 1e9, sb / t_sparse / 1e9, db / t_dense / 1e9

    # one thread: the four weight matrices of two transformer blocks (61 M elements), the seven
    # weight matrices of the first llama block (202 M elements)
    segs1 = [4, 6, 10, 12, 16, 18, 22, 24]
    lay1 = [1, 2, 3, 4, 5, 6, 7]
    it_s, it_d = sparse_inputs(segs1), dense_inputs(lay1, 1)
    n_s1, n_d1 = sum(x[0] for x in it_s), sum(x[0].size for x in it_d)
    t_s1, t_d1 = timed(sparse_chain, it_s, 1), timed(dense_range, it_d, 1)
    v1, s1, d1 = extrapolate(t_s1, n_s1, t_d1, n_d1)
    log(f"[cpu_baseline] 1 thread: sparse {t_s1:.2f} s, dense {t_d1:.2f} s")
    # all cores: the weight matrices of eight blocks (one chain per matrix), the same llama layers cut
    # into ranges
    segsN = [4 + 12 * b + j for b in range(8) for j in (0, 2, 6, 8)]
    it_sN = sparse_inputs(segsN)
    it_dN = dense_inputs(lay1, max(1, threads // 2))
    n_sN, n_dN = sum(x[0] for x in it_sN), sum(x[0].size for x in it_dN)
    del it_s, it_d
    t_sN, t_dN = timed(sparse_chain, it_sN, threads), timed(dense_range, it_dN, threads)
    vN, sN, dN = extrapolate(t_sN, n_sN, t_dN, n_dN)
    log(f"[cpu_baseline] {threads} threads: sparse {t_sN:.2f} s, dense {t_dN:.2f} s")
    return {
        "value": vN, "unit": "GB/s (gradient bytes)", "cores": threads, "kind": "oracle",
        "sample": (f"all-core leg ({threads} threads of the harness over independent work items): gpt2xl segments "
                   f"{segsN[0]}..{segsN[-1]} (32 weight matrices, {n_sN:,} elements), {Wc} chained top-k (nth_element variant) "
                   f"+ window merge per matrix: {t_sN:.2f} s; llama7b layers {lay1} ({n_dN:,} elements) in "
                   f"{len(it_dN)} ranges, snapshot + Adam replay W={Wd}: {t_dN:.2f} s; extrapolated to the full step by "
                   f"gradient bytes"),
        "sparse_GBps": sN, "dense_GBps": dN,
        "single_thread": {
            "value": v1, "cores": 1, "sparse_GBps": s1, "dense_GBps": d1, "sparse_s": t_s1, "dense_s": t_d1,
            "sample": (f"gpt2xl segments {segs1} ({n_s1:,} elements), {Wc} chained top-k + window merge; llama7b layers "
                       f"{lay1} ({n_d1:,} elements), snapshot + Adam replay W={Wd}")},
        "all_cores": {"sparse_s": t_sN, "dense_s": t_dN},
        "nproc": avail, "cpu_model": model,
    }


def config_model_row(sparse):
    """Sec. V-C closed loop: the costs of Eqs. (8) and (9) measured with this library on the sparse
    leg's window, fed to ld_config_select over the 24 candidates of the paper's Example
    (f in {10, 30, 50, 100}, b in {1..6}).
      C_replay(b)  ld_merge_sparse of b diffs resident in HBM (HIP events)
      R_B(b)       ld_merge_sparse_from_host of b diffs: read over the host link + replay (wall clock);
                   decompression is part of the merge kernels
      C_B(b)       the b diffs copied device -> page-locked host memory, persistence's first hop
                   (storage is out of scope here), wall clock
      C_F, R_F     a full checkpoint (w, m, v: 12 n bytes) over the host link, from one measured copy of w each way
    N, T, M and tau are stated, not measured: nothing here trains."""
    dev = sparse.dev
    fs, bs = (10, 30, 50, 100), (1, 2, 3, 4, 5, 6)
    nb = max(bs)
    hi = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t) for t in sparse.idx[:nb]]
    hv = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t) for t in sparse.val[:nb]]
    oi = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True) for t in sparse.idx[:nb]]
    ov = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True) for t in sparse.val[:nb]]
    K = [t.numel() for t in sparse.idx[:nb]]
    lib = ld.load()
    Kh = np.asarray(K, np.int64)
    staging = torch.empty(int(lib.ld_merge_sparse_from_host_staging(Kh.ctypes.data, nb, nb)), dtype=torch.uint8, device=dev)
    ws = torch.empty(ld.ld_merge_sparse_workspace(sparse.n, K), dtype=torch.uint8, device=dev)
    st = torch.cuda.current_stream()

    def wall(fn, reps=3):
        best = []
        for _ in range(reps + 1):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            best.append(time.perf_counter() - t0)
        return float(np.median(best[1:]))

    c_replay, r_b, c_b = {}, {}, {}
    for b in bs:
        tm = Timer()
        for _ in range(4):
            tok = tm.start("m")
            ld.ld_merge_sparse(sparse.w, sparse.idx[:b], sparse.val[:b], sparse.wl.lr, ws)
            tm.stop(tok)
        torch.cuda.synchronize()
        c_replay[b] = float(np.median(tm.ms()["m"][1:])) * 1e-3
        r_b[b] = wall(lambda: ld.ld_merge_sparse_from_host(sparse.w, hi[:b], hv[:b], sparse.wl.lr, group=b, staging=staging,
                                                           workspace=ws, copy_stream=st, merge_stream=st))

        def persist():
            for t in range(b):
                oi[t].copy_(sparse.idx[t], non_blocking=True)
                ov[t].copy_(sparse.val[t], non_blocking=True)
        c_b[b] = wall(persist)
    hw = torch.empty(sparse.n, dtype=torch.float32, pin_memory=True)
    c_f = 3.0 * wall(lambda: hw.copy_(sparse.w, non_blocking=True), reps=2)
    r_f = 3.0 * wall(lambda: sparse.w.copy_(hw, non_blocking=True), reps=2)  # the same bits back: w is unchanged
    del hw
    P = dict(N=1.0, T=86400.0, M=3600.0, tau=1.0, R_F=r_f, C_F=c_f)
    cf, cb = [f for f in fs for _ in bs], [b for _ in fs for b in bs]
    best, tw = ld.ld_config_select(ld.ConfigParams(**P), cf, cb, [r_b[b] for b in cb], [c_b[b] for b in cb])
    grid = {f"f={f}": [float(tw[i * len(bs) + j] / tw[best]) for j in range(len(bs))] for i, f in enumerate(fs)}
    return {
        "selected": {"f": int(cf[best]), "b": int(cb[best]), "T_w_s": float(tw[best])},
        "T_w_normalised": grid, "b_values": list(bs),
        "f_c": {str(b): ld.ld_config_critical_interval(ld.ConfigParams(**P), b, r_b[b], c_b[b]) for b in bs},
        "measured_s": {"C_replay": {str(b): c_replay[b] for b in bs}, "R_B": {str(b): r_b[b] for b in bs},
                       "C_B": {str(b): c_b[b] for b in bs}, "C_F": c_f, "R_F": r_f},
        "stated": {"N": P["N"], "T_s": P["T"], "M_s": P["M"], "tau_s": P["tau"]},
        "note": "Eqs. (8)-(12) of Sec. V-C through ld_config_select; R_B(b) = read of b diffs from page-locked host memory "
                "+ replay (ld_merge_sparse_from_host), C_B(b) = the b diffs copied to page-locked host memory, C_F / R_F = "
                "12 n bytes over the host link; N, T, M, tau stated (no training runs here); not part of `value`"}


def small_configs(dev, steps=3):
    """Configurations 1-3 (the parity-test cases): compress and window-merge time per call, and the
    same verification as the main legs. Their whole traffic fits the last-level cache or is a few
    launches long: latencies, not roofline fractions, and not part of `value`."""
    out = {}
    for name in ("flat1m", "resnet50", "gpt2s"):
        wl = synth.workload(name)
        leg = SparseLeg(wl, dev, pool=min(10, wl.window))
        leg.step(Timer())
        tm = Timer()
        torch.cuda.synchronize()
        for _ in range(steps):
            leg.step(tm)
        torch.cuda.synchronize()
        ms = tm.ms()
        leg.verify()
        c, m = stats(ms["compress"]), stats(ms["merge_sparse"])
        out[name] = {
            "n": leg.n, "segments": len(wl.sizes), "K": leg.K, "W": leg.W,
            "compress_us": {"mean": 1e3 * c["ms"], "median": 1e3 * c["ms_median"], "min": 1e3 * c["ms_min"]},
            "merge_window_us": {"mean": 1e3 * m["ms"], "median": 1e3 * m["ms_median"], "min": 1e3 * m["ms_min"]},
            "compress_algorithmic_GBps": leg.bytes_compress() / (c["ms_median"] * 1e-3) / 1e9,
            "merge_algorithmic_GBps": leg.bytes_merge() / (m["ms_median"] * 1e-3) / 1e9,
            "verified": True,
            "bound": "launch latency / last-level cache" if name != "gpt2s" else "partly HBM (0.5 GB per array), partly launch latency"}
        log(f"[small] {name}: compress {1e3 * c['ms_median']:.0f} us, window merge {1e3 * m['ms_median']:.0f} us (medians), verified")
        del leg
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--pool", type=int, default=10, help="distinct gradients cycled by the sparse leg")
    ap.add_argument("--sparse", default="gpt2xl")
    ap.add_argument("--dense", default="llama7b")
    ap.add_argument("--legs", default="sparse,dense",
                    help="comma list of sparse, dense, mergeonly, combineonly, copycal (mergeonly: the sparse workload's "
                         "window merge alone, on random diffs; combineonly: ld_combine_sparse alone, on 8 random lists; "
                         "copycal: a 1 GiB plain copy, for counter calibration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true", help="skip the calls measured outside the step")
    ap.add_argument("--no-verify", action="store_true", help="skip the check of the outputs (profiling runs)")
    ap.add_argument("--no-small-configs", action="store_true", help="skip the three small configurations")
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
    mergeonly = MergeOnlyLeg(synth.workload(args.sparse), dev) if "mergeonly" in legs else None
    combineonly = CombineOnlyLeg(synth.workload(args.sparse), dev) if "combineonly" in legs else None
    torch.cuda.synchronize()
    log(f"[setup] {time.perf_counter() - t_setup:.1f} s, {torch.cuda.memory_allocated() / 1e9:.1f} GB resident")

    def one_step(tm):
        if sparse:
            sparse.step(tm)
        if dense:
            dense.step(tm)
        if copycal:
            copycal.step(tm)
        if mergeonly:
            mergeonly.step(tm)
        if combineonly:
            combineonly.step(tm)

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
    all_ms = tm.ms()
    per = {k: float(np.mean(v)) for k, v in all_ms.items()}
    log(f"[timed] {args.steps} steps, {ms_per_step:.2f} ms/step; mean ms per call: {per}")

    # the outputs of what was just timed, checked outside the timed region
    verified = None
    if not args.no_verify:
        verified = {}
        try:
            if sparse:
                t1 = time.perf_counter()
                verified["sparse"] = sparse.verify()
                log(f"[verify] sparse leg ok ({time.perf_counter() - t1:.1f} s)")
            if dense:
                t1 = time.perf_counter()
                verified["dense"] = dense.verify()
                log(f"[verify] dense leg ok ({time.perf_counter() - t1:.1f} s)")
        except VerifyError as e:
            log(f"[verify] FAILED: {e}")
            print(json.dumps({"verified": False, "error": str(e)}), flush=True)
            sys.exit(3)

    grad_bytes = (sparse.grad_bytes() if sparse else 0) + (dense.grad_bytes() if dense else 0)
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    def roof(name, nbytes):
        ach = nbytes / (per[name] * 1e-3) / 1e9
        out = stats(all_ms[name])
        out.update({"algorithmic_bytes": nbytes, "achieved_GBps": ach, "frac": ach / HBM_PEAK_GBS,
                    "frac_at_median": nbytes / (out["ms_median"] * 1e-3) / 1e9 / HBM_PEAK_GBS})
        return out

    calls = {}
    if sparse:
        calls["ld_compress_topk"] = roof("compress", sparse.bytes_compress())
        calls["ld_merge_sparse"] = roof("merge_sparse", sparse.bytes_merge())
        calls["ld_compress_topk"]["grad_GBps"] = 4 * sparse.n / (per["compress"] * 1e-3) / 1e9
        calls["ld_merge_sparse"]["grad_GBps"] = 4 * sparse.n * sparse.W / (per["merge_sparse"] * 1e-3) / 1e9
        calls["ld_merge_sparse"]["record_GBps"] = 8 * sparse.K * sparse.W / (per["merge_sparse"] * 1e-3) / 1e9
    if dense:
        calls["ld_snapshot_layers(x34)"] = roof("snapshot_iter", dense.bytes_snapshot_iter())
        calls["ld_merge_dense_adam"] = roof("adam", dense.bytes_adam())
        calls["ld_snapshot_layers(x34)"]["grad_GBps"] = 2 * dense.n / (per["snapshot_iter"] * 1e-3) / 1e9
        calls["ld_merge_dense_adam"]["grad_GBps"] = 2 * dense.n * dense.W / (per["adam"] * 1e-3) / 1e9
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
    if mergeonly:
        calls["ld_merge_sparse(random window)"] = roof("merge_only", mergeonly.bytes_merge())
    if combineonly:
        calls["ld_combine_sparse(random lists)"] = roof("combine_only", combineonly.bytes_combine())
    next_rows = {}
    if sparse and not args.no_next_rows:
        ms = sparse.time_sparse_adam()
        log(f"[next row] ld_merge_sparse_adam: {ms:.2f} ms per call (W={sparse.W})")
        tf = sparse.flops_sparse_adam() / (ms * 1e-3) / 1e12
        # vector ALU ceilings of the chip: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s.
        # Plain fp32 FMA: 2 flops per lane-operation = 78.6 TFLOP/s (the published 157.3 counts packed
        # two-wide FMA, which this build does not emit). Issue model of one Adam step on one element:
        # 12 vector instructions, 2 of them (sqrt, rcp) quarter-rate: 18 issue slots if those do not overlap
        # with full-rate issue, 12 if they overlap completely.
        lane_ops = 256 * 4 * 16 * 2.4e9
        steps = sparse.n * sparse.W
        next_rows["ld_merge_sparse_adam"] = {
            "ms": ms, "algorithmic_bytes": sparse.bytes_sparse_adam(),
            "hbm_GBps": sparse.bytes_sparse_adam() / (ms * 1e-3) / 1e9,
            "hbm_frac": sparse.bytes_sparse_adam() / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "roofline": {"bound": "alu", "achieved": tf, "peak": 78.6, "unit": "TFLOP/s", "frac": tf / 78.6,
                         "peak_packed_fma": 157.3, "frac_of_packed_peak": tf / 157.3,
                         "issue_model_ms": {"18_slots_no_overlap": 18 * steps / lane_ops * 1e3,
                                            "12_slots_full_overlap": 12 * steps / lane_ops * 1e3},
                         "note": "14 flops per element and step; peak = plain (non-packed) fp32 FMA rate of the vector "
                                 "ALUs, 256 CUs x 4 SIMDs x 16 lanes x 2 x 2.4 GHz; the measured time lies between the "
                                 "two issue models: quarter-rate sqrt / rcp overlap partly with full-rate issue"},
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
    if sparse and not args.no_next_rows:
        next_rows["config_model"] = config_model_row(sparse)
        sel = next_rows["config_model"]["selected"]
        log(f"[next row] configuration model: selected (f, b) = ({sel['f']}, {sel['b']})")
    if dense and not args.no_next_rows:
        ms, nb = dense.time_snapshot_to_host()
        log(f"[next row] ld_snapshot_layer into pinned host memory: {ms:.2f} ms for {nb / 1e6:.0f} MB")
        next_rows["ld_snapshot_layer(to pinned host)"] = {
            "ms": ms, "bytes": nb, "GBps": nb / (ms * 1e-3) / 1e9,
            "note": "one 131 M-element layer copied by the same kernel into page-locked host memory: bound by the "
                    "host link; not part of `value`"}
        ms = dense.time_adam_incremental()
        nb = 26 * dense.n
        log(f"[next row] ld_merge_dense_adam, one step per call: {ms:.2f} ms per step")
        next_rows["ld_merge_dense_adam(one step per call)"] = {
            "ms_per_step": ms, "algorithmic_bytes": nb, "achieved_GBps": nb / (ms * 1e-3) / 1e9,
            "frac": nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "grad_GBps": 2 * dense.n / (ms * 1e-3) / 1e9,
            "note": "the replay as the paper runs it, one call per iteration's gradient (26 n bytes per step; the "
                    "fused window of W = 4 moves 8 n per step); not part of `value`"}
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
                "note": "achieved: per call of the entry point (all its kernels), mean over the timed calls, HIP events on "
                        "the launch stream, measured in this run; traffic: NOT measured in this run - HBM bytes per "
                        "call from the committed counter summary profiles/hbm_traffic_gpt2xl_llama7b.txt (rocprofv3 "
                        "FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a 1 GiB plain copy)"}
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
    if verified is not None:
        out["verified"] = True
        out["verification"] = verified
    if next_rows:
        out["next_rows"] = next_rows
    del sparse, dense, copycal
    torch.cuda.empty_cache()
    if not args.no_small_configs:
        try:
            out["small_configs"] = small_configs(dev)
        except VerifyError as e:
            log(f"[verify] FAILED on a small configuration: {e}")
            print(json.dumps({"verified": False, "error": str(e)}), flush=True)
            sys.exit(3)
    if not args.no_cpu_baseline:
        log("[cpu_baseline] timing the oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(gen_dev=str(dev))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

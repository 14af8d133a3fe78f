"""GPU parity on randomly drawn problems: every entry point of the sparse path against the CPU
oracle on seeded cases whose shapes no hand-written test lists (segment tables with empty, tiny
and multi-tile segments; k from 0 to the whole segment; gradients that are normal, heavy-tailed,
quantised, mostly zero, constant or fp16-valued; residuals that cancel the gradient; chains of
calls on a carried residual; long windows of very sparse, shared or clustered diffs).

Bars as everywhere: bit-exact for records, residuals, merged weights and combined lists;
|x - y| <= 1e-7 + 1e-6 |y| for the Adam replay.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_04084_amd import lowdiff as ld
from paper_2509_04084_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def to_gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def draw_table(rs):
    sizes = []
    for _ in range(int(rs.choice([1, 2, 3, 8, 25]))):
        kind = rs.rand()
        if kind < 0.25:
            sizes.append(int(rs.randint(0, 200)))
        elif kind < 0.6:
            sizes.append(int(rs.randint(200, 70000)))
        elif kind < 0.9:
            sizes.append(int(rs.randint(70000, 600000)))
        else:
            sizes.append(int(rs.randint(600000, 2500000)))
    ks = []
    for size in sizes:
        u = rs.rand()
        if size == 0:
            k = 0
        elif u < 0.5:
            k = max(1, int(np.ceil(size * rs.choice([0.001, 0.01, 0.03, 0.1]))))
        elif u < 0.7:
            k = int(rs.randint(0, size + 1))
        elif u < 0.8:
            k = size
        elif u < 0.9:
            k = 1
        else:
            k = 0
        ks.append(min(size, k))
    return synth.seg_offsets(sizes), np.array(ks, np.int32)


def draw_gradient(rs, n):
    kind = rs.rand()
    if n == 0:
        return np.zeros(0, np.float32)
    if kind < 0.35:
        return rs.standard_normal(n).astype(np.float32)
    if kind < 0.5:
        return (rs.standard_t(3, n) * 1e-3).astype(np.float32)
    if kind < 0.65:  # heavy duplication: ties across the threshold
        return (np.round(rs.standard_normal(n) * rs.choice([2, 8, 64])) / 8).astype(np.float32)
    if kind < 0.8:   # mostly zero
        g = rs.standard_normal(n).astype(np.float32)
        g[rs.rand(n) < rs.choice([0.5, 0.9, 0.995])] = 0
        return g
    if kind < 0.9:   # one value everywhere
        return np.full(n, rs.choice([0.0, 1.5, -2.0]), np.float32)
    return rs.standard_normal(n).astype(np.float32).astype(np.float16).astype(np.float32)


@pytest.mark.parametrize("strategy", [ld.LD_COMPRESS_AUTO, ld.LD_COMPRESS_FULL], ids=["auto", "full"])
@pytest.mark.parametrize("seed", range(7000, 7016))
def test_random_chain_compress_merge_adam_combine(seed, strategy):
    rs = np.random.RandomState(seed)
    seg_off, seg_k = draw_table(rs)
    n = int(seg_off[-1])
    g = draw_gradient(rs, n)
    r = np.zeros(n, np.float32) if rs.rand() < 0.4 else (rs.standard_normal(n) * 0.3).astype(np.float32)
    if rs.rand() < 0.2:
        r = (-g).astype(np.float32)
    W = int(rs.choice([1, 2, 5]))
    print(f"[random chain] seed={seed} strategy={strategy} n={n} n_seg={len(seg_k)} K={int(seg_k.sum())} W={W}", flush=True)
    idxs, vals = [], []
    r_gpu = to_gpu(r)
    for t in range(W):
        gt = g if t == 0 else (rs.standard_normal(n) * 0.5).astype(np.float32)
        oi, ov, r = oracle.topk_ef(gt, r, seg_off, seg_k, select=True)
        # the smallest workspace the library accepts in some cases, the one sized for the table in others
        nbytes = ld.ld_compress_topk_workspace(seg_off) if rs.rand() < 0.3 else ld.ld_compress_topk_workspace(seg_off, seg_k)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        gi, gv = ld.ld_compress_topk(to_gpu(gt), r_gpu, seg_off, seg_k, workspace=ws, strategy=strategy)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(gi.cpu().numpy(), oi, err_msg=f"idx, call {t}")
        np.testing.assert_array_equal(bits(gv.cpu().numpy()), bits(ov), err_msg=f"val, call {t}")
        np.testing.assert_array_equal(bits(r_gpu.cpu().numpy()), bits(r), err_msg=f"residual, call {t}")
        idxs.append(oi)
        vals.append(ov)
    if n == 0:
        return
    gi, gv = [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals]
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
    for merge in (ld.LD_MERGE_SWEEP, ld.LD_MERGE_SCATTER):
        w = to_gpu(w0)
        ld.ld_merge_sparse(w, gi, gv, 0.1, strategy=merge)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref), err_msg=f"merge strategy {merge}")
    z = np.zeros(n, np.float32)
    wa, ma, va = to_gpu(w0), to_gpu(z), to_gpu(z)
    ld.ld_merge_sparse_adam(wa, ma, va, gi, gv, 3, 1e-3, **synth.ADAM)
    torch.cuda.synchronize()
    for name, got, want in zip("wmv", (wa, ma, va), oracle.sparse_adam_replay(w0, z, z, idxs, vals, 3, 1e-3, **synth.ADAM)):
        x = got.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(x - want) <= 1e-7 + 1e-6 * np.abs(want)), f"sparse Adam {name}"
    ci, cv, cn = ld.ld_combine_sparse(gi, gv, n, 1.0)
    torch.cuda.synchronize()
    ei, ev = oracle.combine_sparse(idxs, vals, n, 1.0)
    c = int(cn.item())
    assert c == ei.size
    np.testing.assert_array_equal(ci[:c].cpu().numpy(), ei)
    np.testing.assert_array_equal(bits(cv[:c].cpu().numpy()), bits(ev))


@pytest.mark.parametrize("seed", range(7100, 7124))
def test_random_long_thin_windows(seed):
    """Windows of more than ten very sparse diffs (the lane-per-diff kernel's domain and the cases
    just outside it), with the workspace that admits that kernel, with the smallest one, and
    through the entry point that brings its own scratch memory."""
    rs = np.random.RandomState(seed)
    n = int(rs.choice([rs.randint(5000, 200000), rs.randint(200000, 6000000)]))
    W = int(rs.choice([11, 12, 40, 64, 65, 70, 100, 128, 130, 200]))
    mode = str(rs.choice(["indep", "shared", "cluster", "mixed", "tiny"]))
    base_k = int(rs.randint(1, max(1, n // 512) + 1))   # at most 16 records per 8192 elements
    pool = np.sort(rs.choice(n, min(n, base_k * 3), replace=False))
    idxs, vals = [], []
    for t in range(W):
        k = base_k if mode != "tiny" else int(rs.randint(0, 4))
        if mode in ("indep", "tiny") or (mode == "mixed" and t % 3 == 0):
            i = np.sort(rs.choice(n, min(k, n), replace=False))
        elif mode in ("shared", "mixed"):   # the diffs keep hitting the same elements
            i = np.sort(rs.choice(pool, min(k, pool.size), replace=False))
        else:                               # half of every diff inside one 5000-element stretch
            c = int(rs.randint(0, max(1, n - 5000)))
            span = min(5000, n - c)
            i = np.unique(np.concatenate([c + rs.choice(span, min(k // 2 + 1, span), replace=False),
                                          rs.choice(n, k // 2 + 1, replace=False)]))[:max(k, 1)]
        idxs.append(i.astype(np.int32))
        vals.append((rs.standard_normal(i.size) * 10.0 ** rs.uniform(-4, 1)).astype(np.float32))
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
    K = [i.size for i in idxs]
    full_ws = ld.ld_merge_sparse_workspace(n, K)
    min_ws = int(ld.load().ld_merge_sparse_workspace(n, len(K), None))
    print(f"[random thin window] seed={seed} n={n} W={W} mode={mode} k={base_k} lane-per-diff={full_ws > min_ws}", flush=True)
    gi, gv = [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals]
    for nbytes in sorted({full_ws, min_ws}):
        w = to_gpu(w0)
        ld.ld_merge_sparse(w, gi, gv, 0.1, workspace=torch.empty(nbytes, dtype=torch.uint8, device=DEV),
                           strategy=ld.LD_MERGE_SWEEP)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref), err_msg=f"workspace {nbytes}")
    if min_ws <= ld.ld_merge_sparse_static_limit():
        w = to_gpu(w0)
        ld.ld_merge_sparse_static(w, gi, gv, 0.1)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref), err_msg="static scratch")

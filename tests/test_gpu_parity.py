"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.

Bars: bit-exact for indices, values, residuals, snapshots and sparse merges;
|x - y| <= 1e-7 + 1e-6 |y| for the dense Adam replay (and a relative-only check
on v, which never cancels).
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


def compress_paths(ws, seg_off):
    """(path, tied flag, overflowed tiles) per segment of the last call on workspace `ws`; also checks
    that the full-segment pass never gave up."""
    paths, over = ld.ld_compress_topk_paths(ws, seg_off)
    torch.cuda.synchronize()
    paths, over = paths.cpu().numpy(), over.cpu().numpy()
    assert not np.any(paths & 0x10000), "the full-segment pass gave up at its barrier"
    return paths & 0xFF, (paths & 0x100) != 0, over


def check_compress(g, r, seg_off, seg_k, select=True, tag="",
                   strategies=(ld.LD_COMPRESS_AUTO, ld.LD_COMPRESS_FULL), want=None):
    """Runs one compress call per strategy on the GPU and once on the oracle;
    returns (idx, val, r_new) of the oracle. `want(path, tied, overflowed)` is called with what
    the AUTO call reports about the way each segment went."""
    print(f"[compress] {tag} n={len(g)} n_seg={len(seg_k)}", flush=True)
    oi, ov, orr = oracle.topk_ef(g, r, seg_off, seg_k, select=select)
    g_gpu = to_gpu(g)
    seg_k = np.asarray(seg_k, np.int32)
    ws = torch.empty(max(256, ld.ld_compress_topk_workspace(seg_off, seg_k)), dtype=torch.uint8, device=DEV)
    for strategy in strategies:
        r_gpu = to_gpu(r)
        idx, val = ld.ld_compress_topk(g_gpu, r_gpu, seg_off, seg_k, workspace=ws, strategy=strategy)
        torch.cuda.synchronize()
        tg = f"{tag} strategy={strategy}"
        np.testing.assert_array_equal(idx.cpu().numpy(), oi, err_msg=f"idx {tg}")
        np.testing.assert_array_equal(bits(val.cpu().numpy()), bits(ov), err_msg=f"val {tg}")
        np.testing.assert_array_equal(bits(r_gpu.cpu().numpy()), bits(orr), err_msg=f"residual {tg}")
        if len(seg_k) and int(np.asarray(seg_off)[-1]) > 0:
            path, tied, over = compress_paths(ws, seg_off)
            if strategy == ld.LD_COMPRESS_FULL:  # every segment that keeps anything went the full way
                assert np.all(path[seg_k > 0] == ld.LD_PATH_FULL), tg
            elif want is not None:
                want(path, tied, over)
    return oi, ov, orr


# ------------------------------------------------------------------ compress

def test_compress_flat_1m_chained():
    wl = synth.workload("flat1m")
    off, k = wl.seg_off, wl.seg_k
    r = np.zeros(wl.n, np.float32)
    for t in range(3):
        g = synth.gradient(wl, t).numpy()
        def usual(path, tied, over):
            assert path[0] == ld.LD_PATH_CANDIDATES and not tied[0] and over[0] == 0
        _, _, r = check_compress(g, r, off, k, select=(t > 0), tag=f"flat1m t={t}", want=usual)


def test_compress_ragged_segments():
    sizes = [1, 3, 64, 0, 4095, 4097, 65535, 65537, 2, 70001, 0, 200000, 131072, 5]
    off = synth.seg_offsets(sizes)
    rs = np.random.RandomState(1)
    n = int(off[-1])
    g = rs.standard_normal(n).astype(np.float32)
    r = (rs.standard_normal(n) * 0.3).astype(np.float32)
    check_compress(g, r, off, synth.seg_topk(sizes, 1, 100) * (np.array(sizes) > 0), tag="rho=1%")
    check_compress(g, r, off, np.array(sizes, np.int32), tag="k=n")
    check_compress(g, r, off, np.zeros(len(sizes), np.int32), tag="k=0")
    check_compress(g, r, off, np.minimum(np.array(sizes), 1).astype(np.int32), tag="k=1")
    check_compress(g, r, off, (np.array(sizes) // 2).astype(np.int32), tag="k=n/2")


def test_compress_thousands_of_small_segments():
    # 3,000 segments (a model of many small tensors): the segment table travels in seven launches,
    # most segments are smaller than the sample and a tile, a few span several tiles
    rs = np.random.RandomState(11)
    sizes = [int(x) for x in rs.randint(0, 2000, size=3000)]
    for j in range(0, 3000, 250):
        sizes[j] = int(rs.randint(5000, 40000))
    off = synth.seg_offsets(sizes)
    n = int(off[-1])
    g = (rs.standard_t(3, n) * 1e-3).astype(np.float32)
    r = (rs.standard_normal(n) * 1e-3).astype(np.float32)
    k = synth.seg_topk(sizes, 1, 100) * (np.array(sizes) > 0)
    check_compress(g, r, off, k, tag="3000 segments rho=1%")
    k2 = np.array([int(rs.randint(0, s + 1)) for s in sizes], np.int32)
    check_compress(g, r, off, k2, tag="3000 segments random k")


@pytest.mark.parametrize("n", [150001])
def test_compress_adversarial(n):
    off = np.array([0, 1000, 70000, n], np.int64)
    for name, g, r in synth.adversarial_cases(n, seed=3):
        for k in ([10, 690, 800], [1000, 1, 80001], [500, 69000, 40000]):
            check_compress(g, r, off, np.array(k, np.int32), tag=f"{name} k={k}")


@pytest.mark.parametrize("rho", [(2, 100), (3, 100), (5, 100), (75, 1000), (10, 100), (25, 100)])
def test_compress_density_range(rho):
    # Densities of the paper's Exp. 10 range and beyond: the candidate passes change shape with
    # the density (lanes per tile, slot size). Once with the workspace the binding sizes for
    # the call's seg_k, once with the minimum one (the tiles then overflow their slots).
    sizes = [300000, 70000, 1200000, 4097, 65536]
    off = synth.seg_offsets(sizes)
    k = synth.seg_topk(sizes, *rho)
    rs = np.random.RandomState(rho[0])
    n = int(off[-1])
    g = (rs.standard_t(3, n) * 1e-3).astype(np.float32)
    r = (rs.standard_t(3, n) * 3e-4).astype(np.float32)
    oi, ov, orr = check_compress(g, r, off, k, tag=f"rho={rho}", strategies=(ld.LD_COMPRESS_AUTO,))
    assert ld.ld_compress_topk_workspace(off, k) >= ld.ld_compress_topk_workspace(off)
    small = torch.empty(ld.ld_compress_topk_workspace(off), dtype=torch.uint8, device=DEV)
    r_gpu = to_gpu(r)
    idx, val = ld.ld_compress_topk(to_gpu(g), r_gpu, off, k, workspace=small)
    torch.cuda.synchronize()
    path, _, over = compress_paths(small, off)
    assert np.all(path == ld.LD_PATH_CANDIDATES)
    if rho[0] * 100 >= 10 * rho[1]:  # 10 % and 25 %: far more candidates per tile than the minimum slot holds
        assert over[2] > 100, "the slots were expected to overflow"
    np.testing.assert_array_equal(idx.cpu().numpy(), oi)
    np.testing.assert_array_equal(bits(val.cpu().numpy()), bits(ov))
    np.testing.assert_array_equal(bits(r_gpu.cpu().numpy()), bits(orr))


def test_compress_massive_ties_at_the_threshold():
    # More equal keys at the threshold than a segment's gather list holds (4096 + n_s / 4096).
    # One repeated value (zeros of a frozen layer, values on a grid): taken by index order without
    # leaving the candidate path. Two adjacent values sharing one overfull bin: the full-segment
    # path. Both must give the oracle's records, bit for bit.
    rs = np.random.RandomState(17)
    n = 1_000_000
    off = np.array([0, n], np.int64)
    k = np.array([10_000], np.int32)
    base = (rs.standard_normal(n) * 1e-3).astype(np.float32)
    order = np.argsort(-np.abs(base), kind="stable")
    cluster = order[7_000:13_000]                 # ranks around k
    lo_val = np.float32(np.abs(base[order[13_000]]))
    one = base.copy()
    one[cluster] = np.where(rs.rand(cluster.size) < 0.5, lo_val, -lo_val)
    # as drawn, a few other keys just below the repeated value share its fine bin: several values in an
    # overfull bin, so the segment is redone in full
    def redone(path, tied, over):
        assert path[0] == ld.LD_PATH_FULL
    check_compress(one, np.zeros(n, np.float32), off, k, tag="one repeated value and close neighbours", want=redone)
    # with the next 300 ranks moved away the repeated value has its bin to itself: candidate path
    def stays(path, tied, over):
        assert path[0] == ld.LD_PATH_CANDIDATES and not tied[0]
    alone = one.copy()
    alone[order[13_000:13_300]] *= np.float32(0.25)
    check_compress(alone, np.zeros(n, np.float32), off, k, tag="one repeated value across the threshold", want=stays)
    # values on a dyadic grid (exact in fp32, so equal magnitudes are equal keys): ~7000 copies of the
    # threshold value, more than the gather list's 4340 entries, one value per bin
    dyadic = (np.round(base * 4096) / 4096).astype(np.float32)
    check_compress(dyadic, np.zeros(n, np.float32), off, k, tag="dyadic grid", want=stays)
    two = one.copy()
    up = np.nextafter(lo_val, np.float32(1.0))
    two[cluster[::2]] = up
    check_compress(two, np.zeros(n, np.float32), off, k, tag="two adjacent values across the threshold", want=redone)
    # frozen layer next to a live one, and values on a coarse grid (heavy duplication everywhere)
    sizes = [600_000, 400_000]
    off2 = synth.seg_offsets(sizes)
    g = base.copy()
    g[:600_000] = 0.0
    g[123] = -0.0
    def frozen(path, tied, over):
        assert path[0] == ld.LD_PATH_TIES and tied[0], "the zeros of the frozen segment: ties by index"
        assert path[1] == ld.LD_PATH_CANDIDATES and not tied[1]
    check_compress(g, np.zeros(n, np.float32), off2, synth.seg_topk(sizes, 1, 100), tag="frozen segment", want=frozen)
    grid = (np.round(base * 3e4) / 3e4).astype(np.float32)
    check_compress(grid, (np.round(base[::-1] * 1e4) / 3e4).astype(np.float32), off2,
                   synth.seg_topk(sizes, 1, 100), tag="values on a grid")


def test_compress_tied_segment_with_and_without_enough_ties():
    # A segment is treated as "tied" when the 16 K-element sample holds the candidate threshold's
    # own key hundreds of times. White-box: the sample positions are rebuilt here (256 jittered runs
    # of 64 elements), so that the sample can be made to see a repeated key X at the threshold.
    # (a) the rest of the segment holds X often enough: X is the threshold, ties by index;
    # (b) it does not: the tied guess is wrong, the threshold lies below X, full-segment path.
    ns, k_s, X = 2_000_000, 20_000, np.float32(0.3)   # a key whose low mantissa bits are not zero
    stride = ns // 256
    pos = []
    for run in range(256):
        x = (run * 2654435761) & 0xFFFFFFFF
        x ^= x >> 16
        x = (x * 0x7FEB352D) & 0xFFFFFFFF
        x ^= x >> 15
        x = (x * 0x846CA68B) & 0xFFFFFFFF
        x ^= x >> 16
        pos.append(run * stride + ((x * (stride - 63)) >> 32) + np.arange(64))
    pos = np.concatenate(pos)
    rs = np.random.RandomState(23)
    sign = lambda m: np.where(rs.rand(m) < 0.5, 1.0, -1.0).astype(np.float32)
    base = (rs.uniform(0.0, 0.25, ns).astype(np.float32) * sign(ns))
    picked = rs.permutation(pos)
    base[picked[:200]] = rs.uniform(2.0, 3.0, 200).astype(np.float32) * sign(200)
    base[picked[200:800]] = X * sign(600)
    off = np.array([0, ns], np.int64)
    k = np.array([k_s], np.int32)
    z = np.zeros(ns, np.float32)
    few = base.copy()                                  # (b): 800 elements reach X, k is 20,000
    def wrong_guess(path, tied, over):
        assert tied[0], "the sample was built to show a massively repeated key at the threshold"
        assert path[0] == ld.LD_PATH_FULL, "too few ties: the segment must have been redone in full"
    check_compress(few, z, off, k, tag="tied guess, too few ties", strategies=(ld.LD_COMPRESS_AUTO,), want=wrong_guess)
    many = base.copy()                                 # (a): 25,000 more copies of +-X elsewhere
    rest = np.setdiff1d(np.arange(ns), pos)
    many[rs.choice(rest, 25_000, replace=False)] = X * sign(25_000)
    def right_guess(path, tied, over):
        assert tied[0] and path[0] == ld.LD_PATH_TIES
    oi, ov, _ = check_compress(many, z, off, k, tag="tied guess, enough ties", strategies=(ld.LD_COMPRESS_AUTO,),
                               want=right_guess)
    assert np.count_nonzero(np.abs(ov) == X) == k_s - 200 and np.count_nonzero(np.abs(ov) > X) == 200


def test_compress_resnet50_shape():
    wl = synth.workload("resnet50")
    g = synth.gradient(wl, 0).numpy()
    r = (synth.gradient(wl, 1).numpy() * np.float32(0.5))
    check_compress(g, r, wl.seg_off, wl.seg_k, tag="resnet50")


def test_compress_is_deterministic_and_reads_only_grad():
    wl = synth.workload("flat1m")
    g = synth.gradient(wl, 5, device=DEV)
    g0 = g.clone()
    outs = []
    for _ in range(2):
        r = torch.zeros(wl.n, device=DEV)
        i, v = ld.ld_compress_topk(g, r, wl.seg_off, wl.seg_k)
        outs.append((i.clone(), v.clone(), r.clone()))
    torch.cuda.synchronize()
    assert torch.equal(g, g0)
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))


# -------------------------------------------------------------- sparse merge

def _diff_chain(wl, W, n=None):
    n = wl.n if n is None else n
    off = wl.seg_off
    k = wl.seg_k
    r = np.zeros(n, np.float32)
    idxs, vals = [], []
    for t in range(W):
        g = synth.gradient(wl, t).numpy()
        i, v, r = oracle.topk_ef(g, r, off, k, select=True)
        idxs.append(i)
        vals.append(v)
    return idxs, vals


@pytest.mark.parametrize("strategy", [ld.LD_MERGE_SWEEP, ld.LD_MERGE_SCATTER, ld.LD_MERGE_AUTO])
def test_merge_flat_window(strategy):
    wl = synth.workload("flat1m")
    idxs, vals = _diff_chain(wl, wl.window)
    w0 = synth.base_weights(wl.n).numpy()
    ref = oracle.merge_sparse(w0, idxs, vals, wl.lr)
    w = to_gpu(w0)
    ld.ld_merge_sparse(w, [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], wl.lr, strategy=strategy)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref))
    # the window in one call == one call per diff == any prefix
    w2 = to_gpu(w0)
    for j in range(wl.window):
        ld.ld_merge_sparse(w2, [to_gpu(idxs[j])], [to_gpu(vals[j])], wl.lr, strategy=strategy)
        if j == 3:
            torch.cuda.synchronize()
            np.testing.assert_array_equal(bits(w2.cpu().numpy()),
                                          bits(oracle.merge_sparse(w0, idxs[:4], vals[:4], wl.lr)))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w2.cpu().numpy()), bits(ref))


@pytest.mark.parametrize("n,W,dens", [(1, 1, 1.0), (4095, 3, 0.5), (4097, 5, 0.02), (1000003, 9, 0.03),
                                      (300000, 140, 0.004), (123457, 2, 1.0), (50000, 4, 0.0),
                                      (2000003, 40, 0.0005), (2000003, 100, 0.0004)])
def test_merge_ragged_and_dense_windows(n, W, dens):
    rs = np.random.RandomState(n % 1000 + W)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    idxs, vals = [], []
    for t in range(W):
        kk = int(round(n * dens)) if t != 1 else min(n, int(round(n * dens * 2)))
        i = np.sort(rs.choice(n, kk, replace=False)).astype(np.int32)
        idxs.append(i)
        vals.append(rs.standard_normal(kk).astype(np.float32))
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
    for strategy in (ld.LD_MERGE_SWEEP, ld.LD_MERGE_SCATTER):
        w = to_gpu(w0)
        ld.ld_merge_sparse(w, [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], 0.1, strategy=strategy)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref), err_msg=f"strategy {strategy}")


@pytest.mark.parametrize("case", ["random", "identical", "pairs", "clustered", "short_then_long"])
def test_merge_thin_long_windows(case):
    # Long windows of very sparse diffs run a lane per diff: every lane holds its diff's records for
    # the wave's sub-tile, elements touched by several diffs are held back and applied in diff order.
    #   random          a few elements shared by two or three diffs
    #   identical       every diff records the same positions: every record is held back, more per
    #                   lane than it keeps (the lanes take turns)
    #   pairs           diffs 2j and 2j+1 share all positions, values far apart in magnitude
    #   clustered       one diff puts 300 records into one sub-tile (more than a lane holds)
    #   short_then_long 70 diffs (two sets of lanes), the first ones empty or tiny
    # Each also with the minimum workspace (no per-sub-tile table: the ordinary sweep) - same bits.
    n = 3_000_017
    rs = np.random.RandomState({"random": 1, "identical": 2, "pairs": 3, "clustered": 4, "short_then_long": 5}[case])
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    W, k = 100, 3000
    idxs, vals = [], []
    if case == "random":
        for t in range(W):
            idxs.append(np.sort(rs.choice(n, k, replace=False)).astype(np.int32))
    elif case == "identical":
        same = np.sort(rs.choice(n, k, replace=False)).astype(np.int32)
        idxs = [same.copy() for _ in range(W)]
    elif case == "pairs":
        for t in range(0, W, 2):
            i = np.sort(rs.choice(n, k, replace=False)).astype(np.int32)
            idxs += [i, i.copy()]
    elif case == "clustered":
        for t in range(W):
            i = rs.choice(n, k, replace=False)
            if t == 37:
                i[:300] = 16_384 + rs.choice(8192, 300, replace=False)   # sub-tile 2
            idxs.append(np.unique(i).astype(np.int32))
    else:
        W = 70
        for t in range(W):
            kk = [0, 1, 2][t] if t < 3 else k
            idxs.append(np.sort(rs.choice(n, kk, replace=False)).astype(np.int32))
    for t, i in enumerate(idxs):
        scale = 1.0 if case != "pairs" else (1e-4 if t % 2 else 10.0)
        vals.append((rs.standard_normal(i.size) * scale).astype(np.float32))
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
    gi, gv = [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals]
    K = [i.size for i in idxs]
    full_ws = ld.ld_merge_sparse_workspace(n, K)
    min_ws = int(ld.load().ld_merge_sparse_workspace(n, len(K), None))
    assert full_ws > min_ws, "this window was meant to qualify for the per-sub-tile table"
    for nbytes in (full_ws, min_ws):
        w = to_gpu(w0)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        ld.ld_merge_sparse(w, gi, gv, 0.1, workspace=ws, strategy=ld.LD_MERGE_SWEEP)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref), err_msg=f"{case}, workspace {nbytes}")


def test_merge_uneven_diffs_across_many_chunks():
    # Record positions are looked up per 49152-element chunk from guesses that assume evenly
    # spread records; these diffs are anything but (dense runs between long gaps, everything
    # in the last percent, only the first half, one record), the window spans several
    # workgroups of the lookup kernel, and two index arrays start at addresses that are
    # only 4-byte aligned.
    n = 60_000_003
    rs = np.random.RandomState(7)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    starts = np.sort(rs.choice(n - 6000, 120, replace=False)).astype(np.int64)
    runs = np.unique(np.concatenate([np.arange(s0, s0 + 5000) for s0 in starts]))
    idxs = [runs.astype(np.int32),
            (n - 600_000 + np.sort(rs.choice(600_000, 400_000, replace=False))).astype(np.int32),
            np.sort(rs.choice(n, 600_000, replace=False)).astype(np.int32),
            np.arange(0, n // 2, 64, dtype=np.int32),
            np.array([n - 1], np.int32),
            np.unique(np.concatenate([np.arange(0, 40_000), np.arange(n - 40_000, n)])).astype(np.int32)]
    vals = [rs.standard_normal(i.size).astype(np.float32) for i in idxs]
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)

    def shifted(a, shift):  # device copy whose first element sits `shift` elements into an allocation
        buf = torch.empty(a.size + shift, dtype=torch.from_numpy(a[:1]).dtype, device=DEV)
        buf[shift:].copy_(torch.from_numpy(a))
        return buf[shift:]

    gi = [shifted(i, (1, 0, 3, 0, 0, 2)[t]) for t, i in enumerate(idxs)]
    gv = [shifted(v, (0, 0, 1, 0, 0, 3)[t]) for t, v in enumerate(vals)]
    w = to_gpu(w0)
    ld.ld_merge_sparse(w, gi, gv, 0.1, strategy=ld.LD_MERGE_SWEEP)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref))


def test_merge_order_and_zero_diff():
    # order sensitivity: swapping two diffs changes the fp32 result; the GPU follows list order
    n = 8192
    w0 = np.ones(n, np.float32)
    i = np.arange(n, dtype=np.int32)
    v1 = np.full(n, -(2.0 ** -24 + 2.0 ** -30), np.float32)
    v2 = np.ones(n, np.float32)
    for order in ((v1, v2), (v2, v1)):
        ref = oracle.merge_sparse(w0, [i, i], list(order), 1.0)
        w = to_gpu(w0)
        ld.ld_merge_sparse(w, [to_gpu(i), to_gpu(i)], [to_gpu(order[0]), to_gpu(order[1])], 1.0,
                           strategy=ld.LD_MERGE_SWEEP)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref))
    # a zero diff leaves w bit-identical, -0.0 weights included
    w0 = np.random.RandomState(0).standard_normal(n).astype(np.float32)
    w0[:100] = -0.0
    w = to_gpu(w0)
    ld.ld_merge_sparse(w, [to_gpu(i)], [to_gpu(np.zeros(n, np.float32))], 0.1, strategy=ld.LD_MERGE_SWEEP)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(w0))


@pytest.mark.timeout(600)
def test_compress_then_merge_end_to_end_resnet_window():
    """Config 2 whole: ResNet-50-shaped, 161 segments, 1 %, the configuration's 50-diff window built by
    50 chained compress calls and merged in one call; every record, residual and weight against the oracle."""
    wl = synth.workload("resnet50")
    W = wl.window
    assert W == 50
    r_cpu = np.zeros(wl.n, np.float32)
    r_gpu = torch.zeros(wl.n, device=DEV)
    ws = torch.empty(ld.ld_compress_topk_workspace(wl.seg_off), dtype=torch.uint8, device=DEV)
    gi, gv, oi, ov = [], [], [], []
    for t in range(W):
        if t % 10 == 0:
            print(f"[resnet50 window] diff {t}", flush=True)
        g = synth.gradient(wl, t).numpy()
        a, b = ld.ld_compress_topk(to_gpu(g), r_gpu, wl.seg_off, wl.seg_k, workspace=ws)
        gi.append(a)
        gv.append(b)
        i, v, r_cpu = oracle.topk_ef(g, r_cpu, wl.seg_off, wl.seg_k, select=True)
        oi.append(i)
        ov.append(v)
    w0 = synth.base_weights(wl.n).numpy()
    w = to_gpu(w0)
    ld.ld_merge_sparse(w, gi, gv, wl.lr)
    torch.cuda.synchronize()
    for t in range(W):
        np.testing.assert_array_equal(gi[t].cpu().numpy(), oi[t], err_msg=f"idx t={t}")
        np.testing.assert_array_equal(bits(gv[t].cpu().numpy()), bits(ov[t]), err_msg=f"val t={t}")
    np.testing.assert_array_equal(bits(r_gpu.cpu().numpy()), bits(r_cpu))
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(oracle.merge_sparse(w0, oi, ov, wl.lr)))


# ------------------------------------------------------------------ snapshot

@pytest.mark.parametrize("n", [0, 1, 7, 8191, 8192, 1 << 20, (1 << 20) + 3, 11008 * 4096])
def test_snapshot_bit_exact(n):
    src = torch.randint(-32768, 32767, (n + 9,), dtype=torch.int16, device=DEV).view(torch.bfloat16)
    for shift in (0, 1):  # 16-byte aligned and 2-byte aligned views
        s = src[shift:shift + n]
        d = torch.zeros(n + 2, dtype=torch.bfloat16, device=DEV)
        ld.ld_snapshot_layer(s, d[1:1 + n] if shift else d[:n])
        torch.cuda.synchronize()
        got = (d[1:1 + n] if shift else d[:n]).view(torch.int16).cpu().numpy().view(np.uint16)
        ref = oracle.snapshot(s.view(torch.int16).cpu().numpy().view(np.uint16))
        np.testing.assert_array_equal(got, ref)
        rest = d[:1] if shift else d[n:]
        assert torch.all(rest.view(torch.int16) == 0)  # nothing written outside


def test_snapshot_many_layers_one_launch():
    wl = synth.workload("llama7b")
    sizes = [s // 64 for s in wl.sizes[:40]] + [0, 1, 17]
    srcs = [torch.randint(-32768, 32767, (s,), dtype=torch.int16, device=DEV).view(torch.bfloat16) for s in sizes]
    dsts = [torch.zeros_like(s) for s in srcs]
    ld.ld_snapshot_layers(srcs, dsts)
    torch.cuda.synchronize()
    for a, b in zip(srcs, dsts):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ---------------------------------------------------------------------- Adam

def _bf16_bits_t(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def check_adam_close(got, ref, tag):
    for name, a, b in zip("wmv", got, ref):
        a = a.cpu().numpy().astype(np.float64)
        b = b.astype(np.float64)
        err = np.abs(a - b)
        assert np.all(err <= 1e-7 + 1e-6 * np.abs(b)), f"{tag} {name}: max err {err.max()}"
    # v is a sum of non-negative terms: hold it to the relative bound alone
    a, b = got[2].cpu().numpy().astype(np.float64), ref[2].astype(np.float64)
    assert np.all(np.abs(a - b) <= 1e-6 * np.abs(b)), f"{tag} v relative"


@pytest.mark.parametrize("n", [1, 7, 8, 1000003])
@pytest.mark.parametrize("W,step0", [(1, 0), (4, 0), (3, 1000)])
def test_adam_replay_parity(n, W, step0):
    rs = np.random.RandomState(n % 97 + W)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    m0 = np.zeros(n, np.float32) if step0 == 0 else (rs.standard_normal(n) * 1e-4).astype(np.float32)
    v0 = np.zeros(n, np.float32) if step0 == 0 else (rs.standard_normal(n) ** 2 * 1e-7).astype(np.float32)
    grads = [to_gpu((rs.standard_normal(n) * 1e-3).astype(np.float32)).to(torch.bfloat16) for _ in range(W)]
    hp = dict(lr=1e-4, **synth.ADAM)
    ref = oracle.adam_replay(w0, m0, v0, [_bf16_bits_t(g) for g in grads], step0, **hp)
    w, m, v = to_gpu(w0), to_gpu(m0), to_gpu(v0)
    ld.ld_merge_dense_adam(w, m, v, grads, step0, **hp)
    torch.cuda.synchronize()
    check_adam_close((w, m, v), ref, f"n={n} W={W} step0={step0}")
    # fused window == chain of single-step calls, bit for bit
    w2, m2, v2 = to_gpu(w0), to_gpu(m0), to_gpu(v0)
    for t in range(W):
        ld.ld_merge_dense_adam(w2, m2, v2, [grads[t]], step0 + t, **hp)
    torch.cuda.synchronize()
    for a, b in ((w, w2), (m, m2), (v, v2)):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))


@pytest.mark.parametrize("eps", [0.0, 1e-20])
def test_adam_with_no_eps_and_denormal_second_moments(eps):
    # With eps = 0 (or far below the root of a denormal) the denominator is sqrt(v / bc2) alone, and for
    # gradients below 1e-19 that argument is a denormal fp32 number: a square root that takes denormals
    # for zero would divide by zero. Gradients from 1e-3 down to 3e-20, no zeros (0 / 0 has no value to
    # compare); dense replay and sparse replay of the same gradients.
    n, W = 40_003, 3
    rs = np.random.RandomState(71)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    z = np.zeros(n, np.float32)
    grads = []
    for _ in range(W):
        mag = 10.0 ** rs.uniform(-19.5, -3.0, n)
        g = (mag * np.where(rs.rand(n) < 0.5, 1.0, -1.0)).astype(np.float32)
        grads.append(to_gpu(g).to(torch.bfloat16))
    assert all(bool((g.float().abs() > 1e-20).all()) for g in grads)
    hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=eps)
    gb = [_bf16_bits_t(g) for g in grads]
    ref = oracle.adam_replay(w0, z, z, gb, 0, **hp)
    assert np.all(np.isfinite(ref[0]))
    assert int((grads[0].float().abs() < 1.0e-19).sum()) > 500   # first step: v / bc2 = g^2 is a denormal for these
    w, m, v = to_gpu(w0), to_gpu(z), to_gpu(z)
    ld.ld_merge_dense_adam(w, m, v, grads, 0, **hp)
    # the same gradients as sparse diffs that record every position
    ws, ms_, vs = to_gpu(w0), to_gpu(z), to_gpu(z)
    allpos = torch.arange(n, dtype=torch.int32, device=DEV)
    ld.ld_merge_sparse_adam(ws, ms_, vs, [allpos] * W, [g.float() for g in grads], 0, **hp)
    torch.cuda.synchronize()
    for got in ((w, m, v), (ws, ms_, vs)):
        for name, a, b in zip("wmv", got, ref):
            a = a.cpu().numpy().astype(np.float64)
            err = np.abs(a - b.astype(np.float64))
            assert np.all(err <= 1e-7 + 1e-6 * np.abs(b)), f"eps={eps} {name}: max err {err.max()}"
        a, b = got[2].cpu().numpy().astype(np.float64), ref[2].astype(np.float64)
        normal = b >= 1.1755e-38   # a denormal v has few bits: the relative bound is for the normal ones
        assert np.all(np.abs(a - b)[normal] <= 1e-6 * b[normal])
        assert np.all(np.abs(a - b)[~normal] <= 3e-45)   # and at most two steps of the denormal grid elsewhere
    for a, b in ((w, ws), (m, ms_), (v, vs)):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_adam_zero_gradient_and_closed_form():
    n = 4096
    hp = dict(lr=1e-2, **synth.ADAM)
    w0 = np.random.RandomState(2).standard_normal(n).astype(np.float32)
    v0 = (np.random.RandomState(3).standard_normal(n) ** 2 * 1e-6).astype(np.float32)
    w, m, v = to_gpu(w0), torch.zeros(n, device=DEV), to_gpu(v0)
    ld.ld_merge_dense_adam(w, m, v, [torch.zeros(n, dtype=torch.bfloat16, device=DEV)], 5, **hp)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(w0))
    assert torch.all(m == 0)
    np.testing.assert_allclose(v.cpu().numpy(), np.float64(np.float32(0.999)) * v0, rtol=1e-6)
    # constant gradient from zero state: every step moves w by lr*c/(|c|+eps)
    c = torch.linspace(-2, 2, n, device=DEV).to(torch.bfloat16)
    T = 20
    w, m, v = torch.ones(n, device=DEV), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    ld.ld_merge_dense_adam(w, m, v, [c] * T, 0, **hp)
    torch.cuda.synchronize()
    cd = c.float().cpu().numpy().astype(np.float64)
    want = 1.0 - T * hp["lr"] * cd / (np.abs(cd) + hp["eps"])
    want[cd == 0] = 1.0
    np.testing.assert_allclose(w.cpu().numpy(), want, rtol=3e-6)


# ------------------------------------------------- sparse diffs through Adam

@pytest.mark.parametrize("n,W,dens,step0", [(1, 1, 1.0, 0), (7, 3, 0.5, 0), (2047, 4, 0.05, 3), (2049, 5, 0.01, 0),
                                            (1000003, 6, 0.01, 1000), (300000, 70, 0.004, 2),
                                            (123457, 3, 1.0, 0), (50000, 4, 0.0, 5)])
def test_sparse_adam_replay_parity(n, W, dens, step0):
    rs = np.random.RandomState(n % 1000 + W)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    m0 = np.zeros(n, np.float32) if step0 == 0 else (rs.standard_normal(n) * 1e-4).astype(np.float32)
    v0 = np.zeros(n, np.float32) if step0 == 0 else (rs.standard_normal(n) ** 2 * 1e-7).astype(np.float32)
    idxs, vals = [], []
    for t in range(W):
        kk = int(round(n * dens)) if t != 1 else min(n, int(round(n * dens * 2)))
        idxs.append(np.sort(rs.choice(n, kk, replace=False)).astype(np.int32))
        vals.append((rs.standard_normal(kk) * 1e-3).astype(np.float32))
    hp = dict(lr=1e-4, **synth.ADAM)
    print(f"[sparse_adam] n={n} W={W} dens={dens} step0={step0}", flush=True)
    ref = oracle.sparse_adam_replay(w0, m0, v0, idxs, vals, step0, **hp)
    gi, gv = [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals]
    w, m, v = to_gpu(w0), to_gpu(m0), to_gpu(v0)
    ld.ld_merge_sparse_adam(w, m, v, gi, gv, step0, **hp)
    torch.cuda.synchronize()
    for name, a, b in zip("wmv", (w, m, v), ref):
        a = a.cpu().numpy().astype(np.float64)
        err = np.abs(a - b.astype(np.float64))
        assert np.all(err <= 1e-7 + 1e-6 * np.abs(b)), f"{name}: max err {err.max()}"
    # v never cancels: hold it to a relative bound alone (W roundings of 2^-24 each)
    a, b = v.cpu().numpy().astype(np.float64), ref[2].astype(np.float64)
    assert np.all(np.abs(a - b) <= max(1e-6, W * 1.2e-7) * np.abs(b)), "v relative"
    # the window in one call == one call per diff, bit for bit
    w2, m2, v2 = to_gpu(w0), to_gpu(m0), to_gpu(v0)
    for t in range(W):
        ld.ld_merge_sparse_adam(w2, m2, v2, [gi[t]], [gv[t]], step0 + t, **hp)
    torch.cuda.synchronize()
    for a, b in ((w, w2), (m, m2), (v, v2)):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_sparse_adam_equals_dense_adam_on_full_diffs():
    # diffs that record every position with bf16-representable values are dense gradients:
    # both entry points must then agree bit for bit (they share the per-element step)
    n, W = 70001, 3
    rs = np.random.RandomState(9)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    gb = [to_gpu((rs.standard_normal(n) * 1e-3).astype(np.float32)).to(torch.bfloat16) for _ in range(W)]
    hp = dict(lr=1e-4, **synth.ADAM)
    w, m, v = to_gpu(w0), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    ld.ld_merge_dense_adam(w, m, v, gb, 0, **hp)
    allidx = torch.arange(n, dtype=torch.int32, device=DEV)
    w2, m2, v2 = to_gpu(w0), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    ld.ld_merge_sparse_adam(w2, m2, v2, [allidx] * W, [g.float() for g in gb], 0, **hp)
    torch.cuda.synchronize()
    for a, b in ((w, w2), (m, m2), (v, v2)):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_sparse_adam_after_compress_resnet_window():
    # diffs as ld_compress_topk emits them (161 segments of very different sizes)
    wl = synth.workload("resnet50")
    W = 4
    r_gpu = torch.zeros(wl.n, device=DEV)
    gi, gv = [], []
    for t in range(W):
        a, b = ld.ld_compress_topk(to_gpu(synth.gradient(wl, t).numpy()), r_gpu, wl.seg_off, wl.seg_k)
        gi.append(a)
        gv.append(b)
    rs = np.random.RandomState(4)
    w0 = synth.base_weights(wl.n).numpy()
    m0 = (rs.standard_normal(wl.n) * 1e-4).astype(np.float32)
    v0 = (rs.standard_normal(wl.n) ** 2 * 1e-7).astype(np.float32)
    hp = dict(lr=1e-4, **synth.ADAM)
    w, m, v = to_gpu(w0), to_gpu(m0), to_gpu(v0)
    ld.ld_merge_sparse_adam(w, m, v, gi, gv, 10, **hp)
    torch.cuda.synchronize()
    ref = oracle.sparse_adam_replay(w0, m0, v0, [i.cpu().numpy() for i in gi], [x.cpu().numpy() for x in gv], 10, **hp)
    check_adam_close((w, m, v), ref, "resnet50 window")


# ------------------------------------------------- combine of per-worker lists

def check_combine(idxs, vals, n, scale=1.0, tag=""):
    print(f"[combine] {tag} n={n} N={len(idxs)} K={[len(i) for i in idxs][:8]}", flush=True)
    oi, ov = oracle.combine_sparse(idxs, vals, n, scale)
    gi, gv, cnt = ld.ld_combine_sparse([to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], n, scale)
    torch.cuda.synchronize()
    c = int(cnt.item())
    assert c == len(oi), f"{tag}: count {c} != {len(oi)}"
    np.testing.assert_array_equal(gi[:c].cpu().numpy(), oi, err_msg=f"idx {tag}")
    np.testing.assert_array_equal(bits(gv[:c].cpu().numpy()), bits(ov), err_msg=f"val {tag}")


@pytest.mark.parametrize("n,N,dens", [(1, 1, 1.0), (100, 3, 0.3), (8191, 4, 0.05), (8193, 5, 0.5),
                                      (1000003, 8, 0.01), (3000000, 64, 0.002), (200000, 2, 1.0),
                                      (50000, 4, 0.0)])
def test_combine_parity(n, N, dens):
    rs = np.random.RandomState(n % 997 + N)
    idxs, vals = [], []
    for r in range(N):
        kk = int(round(n * dens)) if r != 1 else min(n, int(round(n * dens * 1.5)))
        idxs.append(np.sort(rs.choice(n, kk, replace=False)).astype(np.int32))
        vals.append(rs.standard_normal(kk).astype(np.float32))
    check_combine(idxs, vals, n, tag="sum")
    check_combine(idxs, vals, n, scale=1.0 / N, tag="mean")


def test_combine_worker_order_cancellation_and_clusters():
    n = 100000
    one = np.array([77777], np.int32)
    a, b, c = np.float32(1.0), np.float32(2.0 ** -24), np.float32(2.0 ** -24)
    check_combine([one, one, one], [np.array([a]), np.array([b]), np.array([c])], n, tag="order abc")
    check_combine([one, one, one], [np.array([b]), np.array([c]), np.array([a])], n, tag="order bca")
    i = np.arange(100, 5000, 7, dtype=np.int32)
    v = np.random.RandomState(0).standard_normal(len(i)).astype(np.float32)
    check_combine([i, i], [v, -v], n, tag="cancel")  # zeros stay in the list
    # all records of every worker packed into one corner, the rest of the index space empty
    rs = np.random.RandomState(1)
    idxs = [np.sort(rs.choice(9000, 3000, replace=False)).astype(np.int32) + 40000 for _ in range(5)]
    vals = [rs.standard_normal(3000).astype(np.float32) for _ in range(5)]
    check_combine(idxs, vals, n, tag="clustered")
    # nothing at all, and a single empty worker among full ones
    e = np.zeros(0, np.int32)
    check_combine([e, e], [e.astype(np.float32)] * 2, n, tag="empty")
    check_combine([idxs[0], e, idxs[1]], [vals[0], e.astype(np.float32), vals[1]], n, tag="one empty")


def test_combine_of_compressed_diffs_and_truncated_output():
    # lists as ld_compress_topk emits them for 4 "workers" (different gradients, same segments)
    wl = synth.workload("resnet50")
    gi, gv = [], []
    for t in range(4):
        r = torch.zeros(wl.n, device=DEV)
        a, b = ld.ld_compress_topk(to_gpu(synth.gradient(wl, t).numpy()), r, wl.seg_off, wl.seg_k)
        gi.append(a)
        gv.append(b)
    torch.cuda.synchronize()
    idxs, vals = [x.cpu().numpy() for x in gi], [x.cpu().numpy() for x in gv]
    check_combine(idxs, vals, wl.n, scale=0.25, tag="resnet50 x4")
    # an output buffer that is too small: the count still tells the full size, nothing is written past the end
    oi, ov = oracle.combine_sparse(idxs, vals, wl.n, 0.25)
    cap = len(oi) // 2
    out_i = torch.full((cap + 64,), -1, dtype=torch.int32, device=DEV)
    out_v = torch.zeros(cap + 64, device=DEV)
    _, _, cnt = ld.ld_combine_sparse(gi, gv, wl.n, 0.25, out_idx=out_i[:cap], out_val=out_v[:cap])
    torch.cuda.synchronize()
    assert int(cnt.item()) == len(oi)
    np.testing.assert_array_equal(out_i[:cap].cpu().numpy(), oi[:cap])
    assert bool((out_i[cap:] == -1).all())


def test_snapshot_into_pinned_host_memory():
    # the paper's snapshot leaves the GPU: the same entry points with a page-locked host destination
    n = (1 << 22) + 5
    src = torch.randint(-32768, 32767, (n,), dtype=torch.int16, device=DEV).view(torch.bfloat16)
    dst = torch.zeros(n, dtype=torch.bfloat16).pin_memory()
    ld.ld_snapshot_layer(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst.view(torch.int16), src.cpu().view(torch.int16))
    sizes = [1, 4096, 70001, 1 << 20]
    srcs = [torch.randint(-32768, 32767, (k,), dtype=torch.int16, device=DEV).view(torch.bfloat16) for k in sizes]
    dsts = [torch.zeros(k, dtype=torch.bfloat16).pin_memory() for k in sizes]
    ld.ld_snapshot_layers(srcs, dsts)
    torch.cuda.synchronize()
    for a, b in zip(srcs, dsts):
        assert torch.equal(b.view(torch.int16), a.cpu().view(torch.int16))


# ------------------------------------------------------------ pipelined recovery

@pytest.mark.parametrize("group", [1, 2, 3, 64])
def test_merge_from_pinned_host_equals_the_window_merge(group):
    # diffs in page-locked host memory, copied group by group on one stream while the previous
    # group is merged on another: same bits as the one-call merge and as the oracle
    n, W = 3_000_001, 7
    rs = np.random.RandomState(41 + group)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    idxs, vals = [], []
    for t in range(W):
        kk = [30_000, 0, 45_000, 1, 30_000, 60_000, 29_999][t]
        idxs.append(np.sort(rs.choice(n, kk, replace=False)).astype(np.int32))
        vals.append(rs.standard_normal(kk).astype(np.float32))
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
    hi = [torch.from_numpy(i).pin_memory() for i in idxs]
    hv = [torch.from_numpy(v).pin_memory() for v in vals]
    copy_s, merge_s = torch.cuda.Stream(), torch.cuda.Stream()
    w = to_gpu(w0)
    torch.cuda.synchronize()
    ld.ld_merge_sparse_from_host(w, hi, hv, 0.1, group=group, copy_stream=copy_s, merge_stream=merge_s)
    merge_s.synchronize()
    copy_s.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref))
    # both roles on the current stream, twice in a row with the same staging buffers
    w2 = to_gpu(w0)
    K = [i.numel() for i in hi]
    staging = torch.empty(max(256, ld.load().ld_merge_sparse_from_host_staging(
        np.array(K, np.int64).ctypes.data_as(__import__("ctypes").c_void_p), W, min(group, W))), dtype=torch.uint8, device=DEV)
    for _ in range(2):
        w2.copy_(to_gpu(w0))
        ld.ld_merge_sparse_from_host(w2, hi, hv, 0.1, group=group, staging=staging)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w2.cpu().numpy()), bits(ref))
    # with four events of the caller's the call creates none of its own; the same events serve call after call
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    events = []
    for _ in range(4):
        e = ctypes.c_void_p()
        assert hip.hipEventCreateWithFlags(ctypes.byref(e), 2) == 0     # hipEventDisableTiming
        events.append(e.value)
    for _ in range(2):
        w3 = to_gpu(w0)
        torch.cuda.synchronize()
        ld.ld_merge_sparse_from_host(w3, hi, hv, 0.1, group=group, copy_stream=copy_s, merge_stream=merge_s, events=events)
        merge_s.synchronize()
        copy_s.synchronize()
        np.testing.assert_array_equal(bits(w3.cpu().numpy()), bits(ref))
    for e in events:
        assert hip.hipEventDestroy(ctypes.c_void_p(e)) == 0


# ------------------------------------------------- workspaces hold anything on entry

@pytest.mark.parametrize("fill", [0x00, 0xFF, 0x5A, "random"])
def test_workspace_and_output_contents_on_entry_are_irrelevant(fill):
    def dirty(nbytes):
        if fill == "random":
            return torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV)
        return torch.full((nbytes,), fill, dtype=torch.uint8, device=DEV)

    sizes = [70001, 64, 300000, 0, 4097, 200000]
    off = synth.seg_offsets(sizes)
    k = synth.seg_topk(sizes, 1, 100) * (np.array(sizes) > 0)
    n, K = int(off[-1]), int(k.sum())
    rs = np.random.RandomState(9)
    g = rs.standard_normal(n).astype(np.float32)
    g[70065:370065][rs.rand(300000) < 0.7] = np.float32(0.25)     # massive ties in the large segment
    r0 = (rs.standard_normal(n) * 0.1).astype(np.float32)
    r0[70065:370065] = 0
    oi, ov, orr = oracle.topk_ef(g, r0, off, k, select=True)
    for strategy in (ld.LD_COMPRESS_AUTO, ld.LD_COMPRESS_FULL):
        ws = dirty(ld.ld_compress_topk_workspace(off, k))
        out_i = dirty(4 * K).view(torch.int32)
        out_v = dirty(4 * K).view(torch.float32)
        r = to_gpu(r0)
        ld.ld_compress_topk(to_gpu(g), r, off, k, out_i, out_v, ws, strategy=strategy)
        ld.ld_compress_topk(to_gpu(g), to_gpu(r0), off, k, out_i, out_v, ws, strategy=strategy)  # reused as left
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out_i.cpu().numpy(), oi)
        np.testing.assert_array_equal(bits(out_v.cpu().numpy()), bits(ov))
        np.testing.assert_array_equal(bits(r.cpu().numpy()), bits(orr))
    # the replays and the combine on two diffs
    g2 = rs.standard_normal(n).astype(np.float32)
    oi2, ov2, _ = oracle.topk_ef(g2, orr, off, k, select=True)
    idxs, vals = [oi, oi2], [ov, ov2]
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    w = to_gpu(w0)
    ld.ld_merge_sparse(w, [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], 0.1,
                       dirty(ld.ld_merge_sparse_workspace(n, [K, K])), strategy=ld.LD_MERGE_SWEEP)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(oracle.merge_sparse(w0, idxs, vals, 0.1)))
    z = np.zeros(n, np.float32)
    wa, ma, va = to_gpu(w0), to_gpu(z), to_gpu(z)
    ld.ld_merge_sparse_adam(wa, ma, va, [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], 0, 1e-4, **synth.ADAM,
                            workspace=dirty(ld.ld_merge_sparse_adam_workspace(n, [K, K])))
    torch.cuda.synchronize()
    check_adam_close((wa, ma, va), oracle.sparse_adam_replay(w0, z, z, idxs, vals, 0, 1e-4, **synth.ADAM), "sparse adam")
    c_i, c_v, c_n = ld.ld_combine_sparse([to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], n, 1.0,
                                         dirty(8 * K).view(torch.int32), dirty(8 * K).view(torch.float32),
                                         dirty(8).view(torch.int64), dirty(ld.ld_combine_sparse_workspace(n, 2)))
    torch.cuda.synchronize()
    e_i, e_v = oracle.combine_sparse(idxs, vals, n, 1.0)
    cnt = int(c_n.item())
    assert cnt == e_i.size
    np.testing.assert_array_equal(c_i[:cnt].cpu().numpy(), e_i)
    np.testing.assert_array_equal(bits(c_v[:cnt].cpu().numpy()), bits(e_v))


# ------------------------------------------------------ checking a loaded diff

def test_check_diff_counts_match_oracle():
    n = 5_000_000
    rs = np.random.RandomState(3)
    good = np.sort(rs.choice(n, 300_001, replace=False)).astype(np.int32)
    vals = rs.standard_normal(good.size).astype(np.float32)
    cases = {"good": (good, vals), "no values": (good, None), "empty": (good[:0], vals[:0]), "one": (good[:1], vals[:1])}
    bad = good.copy()
    bv = vals.copy()
    # damage at the start, at workgroup boundaries (2048 records each), in the ragged tail
    for j in (0, 1, 2047, 2048, 2049, 4096, 100_000, 299_999, 300_000):
        bad[j] = bad[j - 1] if j and j % 2 else (-7 if j % 3 == 0 else n + j)
    bv[[0, 2048, 123_456, 300_000]] = np.nan
    bv[5] = np.inf
    cases["damaged"] = (bad, bv)
    cases["descending"] = (good[::-1].copy(), vals)
    cases["all equal"] = (np.full(10_000, 17, np.int32), np.zeros(10_000, np.float32))
    counts = torch.empty(3, dtype=torch.int64, device=DEV)
    for name, (i, v) in cases.items():
        got = ld.ld_check_diff(to_gpu(i), None if v is None else to_gpu(v), n, counts)
        torch.cuda.synchronize()
        assert tuple(got.cpu().tolist()) == oracle.check_diff(i, v, n), name
    assert tuple(ld.ld_check_diff(to_gpu(good), to_gpu(vals), int(good[-1])).cpu().tolist()) == (1, 0, 0)


# ------------------------------------------------------------ graph capture

def test_calls_can_be_captured_in_a_graph_and_replayed():
    # The entry points only enqueue kernels on the caller's stream (no allocation, no copy, no
    # memset, no synchronisation), so a compress + merge + Adam sequence can be captured once and
    # replayed. Every replay, with fresh inputs and eager work in between, must give what
    # the oracle gives.
    wl = synth.workload("flat1m")
    off, k = wl.seg_off, wl.seg_k
    K = int(k.sum())
    n = wl.n
    g = torch.zeros(n, device=DEV)
    r = torch.zeros(n, device=DEV)
    w = torch.zeros(n, device=DEV)
    m = torch.zeros(n, device=DEV)
    v = torch.zeros(n, device=DEV)
    gb = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    snap = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    oi = torch.empty(K, dtype=torch.int32, device=DEV)
    ov = torch.empty(K, dtype=torch.float32, device=DEV)
    ws_c = torch.empty(ld.ld_compress_topk_workspace(off, k), dtype=torch.uint8, device=DEV)
    ws_m = torch.empty(ld.ld_merge_sparse_workspace(n, [K]), dtype=torch.uint8, device=DEV)

    def sequence():
        ld.ld_compress_topk(g, r, off, k, oi, ov, ws_c)
        ld.ld_merge_sparse(w, [oi], [ov], wl.lr, ws_m, strategy=ld.LD_MERGE_SWEEP)
        ld.ld_snapshot_layer(gb, snap)
        ld.ld_merge_dense_adam(w, m, v, [snap], 0, 1e-4, **synth.ADAM)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sequence()  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()

    r_host = np.zeros(n, np.float32)
    for rep in range(3):
        g_host = synth.gradient(wl, 10 + rep).numpy()
        w_host = synth.base_weights(n).numpy() * np.float32(1 + rep)
        gb_t = (synth.gradient(wl, 20 + rep) * 1e-3).to(torch.bfloat16)
        g.copy_(torch.from_numpy(g_host))
        r.copy_(torch.from_numpy(r_host))
        w.copy_(torch.from_numpy(w_host))
        m.zero_()
        v.zero_()
        gb.copy_(gb_t)
        graph.replay()
        torch.cuda.synchronize()
        ei, ev, er = oracle.topk_ef(g_host, r_host, off, k, select=True)
        np.testing.assert_array_equal(oi.cpu().numpy(), ei, err_msg=f"replay {rep}")
        np.testing.assert_array_equal(bits(ov.cpu().numpy()), bits(ev), err_msg=f"replay {rep}")
        np.testing.assert_array_equal(bits(r.cpu().numpy()), bits(er), err_msg=f"replay {rep}")
        w_merged = oracle.merge_sparse(w_host, [ei], [ev], wl.lr)
        gbits = gb_t.view(torch.int16).numpy().view(np.uint16)
        np.testing.assert_array_equal(snap.cpu().view(torch.int16).numpy().view(np.uint16), gbits)
        zeros = np.zeros(n, np.float32)
        rw, rm, rv = oracle.adam_replay(w_merged, zeros, zeros, [gbits], 0, 1e-4, **synth.ADAM)
        check_adam_close((w, m, v), (rw, rm, rv), f"replay {rep}")
        r_host = er
        # eager work between the replays, on the same buffers' neighbours
        torch.randn(1 << 20, device=DEV).sum().item()


# ------------------------------------------------------------ two streams

def test_independent_calls_on_two_streams_do_not_interfere():
    # The library keeps no state between calls and works only in the buffers it is handed: two
    # pipelines (chained compress calls, then the window merge), each with buffers and workspaces of
    # its own, enqueued alternately on two streams so that their kernels overlap on the GPU, must
    # each give what the oracle gives for it alone.
    T = 3
    cases = []
    for seed, sizes, rho in ((5, [1_500_000, 70_001, 2_300_000, 4096, 900_000, 3], (1, 100)),
                             (6, [65_537, 3_100_000, 0, 1_000_000, 131_072], (3, 100))):
        rs = np.random.RandomState(seed)
        off = synth.seg_offsets(sizes)
        k = synth.seg_topk(sizes, *rho) * (np.array(sizes) > 0)
        n, K = int(off[-1]), int(k.sum())
        case = dict(
            off=off, k=k, n=n, K=K, lr=0.1 * (seed - 4),
            g=[(rs.standard_t(3, n) * 1e-3).astype(np.float32) for _ in range(T)],
            r0=(rs.standard_normal(n) * 1e-4).astype(np.float32),
            w0=synth.base_weights(n).numpy() * np.float32(seed),
            stream=torch.cuda.Stream())
        case["g_gpu"] = [to_gpu(x) for x in case["g"]]
        case["r_gpu"] = to_gpu(case["r0"])
        case["w_gpu"] = to_gpu(case["w0"])
        case["idx"] = [torch.empty(K, dtype=torch.int32, device=DEV) for _ in range(T)]
        case["val"] = [torch.empty(K, dtype=torch.float32, device=DEV) for _ in range(T)]
        case["ws_c"] = torch.empty(ld.ld_compress_topk_workspace(off, k), dtype=torch.uint8, device=DEV)
        case["ws_m"] = torch.empty(ld.ld_merge_sparse_workspace(n, [K] * T), dtype=torch.uint8, device=DEV)
        cases.append(case)
    torch.cuda.synchronize()
    for t in range(T):
        for c in cases:
            ld.ld_compress_topk(c["g_gpu"][t], c["r_gpu"], c["off"], c["k"], c["idx"][t], c["val"][t], c["ws_c"],
                                stream=c["stream"])
    for c in cases:
        ld.ld_merge_sparse(c["w_gpu"], c["idx"], c["val"], c["lr"], c["ws_m"], stream=c["stream"])
    torch.cuda.synchronize()
    for j, c in enumerate(cases):
        r = c["r0"]
        idxs, vals = [], []
        for t in range(T):
            oi, ov, r = oracle.topk_ef(c["g"][t], r, c["off"], c["k"], select=True)
            np.testing.assert_array_equal(c["idx"][t].cpu().numpy(), oi, err_msg=f"pipeline {j} idx t={t}")
            np.testing.assert_array_equal(bits(c["val"][t].cpu().numpy()), bits(ov), err_msg=f"pipeline {j} val t={t}")
            idxs.append(oi)
            vals.append(ov)
        np.testing.assert_array_equal(bits(c["r_gpu"].cpu().numpy()), bits(r), err_msg=f"pipeline {j} residual")
        w = oracle.merge_sparse(c["w0"], idxs, vals, c["lr"])
        np.testing.assert_array_equal(bits(c["w_gpu"].cpu().numpy()), bits(w), err_msg=f"pipeline {j} w")


# ------------------------------------------------------------ randomised shapes

def _random_case(seed):
    """Segment table, k per segment, gradient and residual drawn from a mixture of shapes and value laws
    (tiny to 2.5 M-element segments; k from 0 to n_s; normal, heavy-tailed, quantised, mostly-zero,
    constant and fp16-rounded values; zero, random or cancelling residual)."""
    rs = np.random.RandomState(seed)
    sizes = []
    for _ in range(int(rs.choice([1, 2, 3, 8, 25]))):
        u = rs.rand()
        sizes.append(int(rs.randint(0, 200) if u < 0.25 else rs.randint(200, 70000) if u < 0.6
                         else rs.randint(70000, 600000) if u < 0.9 else rs.randint(600000, 2500000)))
    off = synth.seg_offsets(sizes)
    n = int(off[-1])
    ks = []
    for s_ in sizes:
        u = rs.rand()
        k_ = (0 if s_ == 0 else max(1, int(np.ceil(s_ * rs.choice([0.001, 0.01, 0.03, 0.1])))) if u < 0.5
              else int(rs.randint(0, s_ + 1)) if u < 0.7 else s_ if u < 0.8 else 1 if u < 0.9 else 0)
        ks.append(min(s_, k_))
    u = rs.rand()
    if u < 0.35:
        g = rs.standard_normal(n).astype(np.float32)
    elif u < 0.5:
        g = (rs.standard_t(3, n) * 1e-3).astype(np.float32)
    elif u < 0.65:
        g = (np.round(rs.standard_normal(n) * rs.choice([2, 8, 64])) / 8).astype(np.float32)
    elif u < 0.8:
        g = rs.standard_normal(n).astype(np.float32)
        g[rs.rand(n) < rs.choice([0.5, 0.9, 0.995])] = 0
    elif u < 0.9:
        g = np.full(n, rs.choice([0.0, 1.5, -2.0]), np.float32)
    else:
        g = rs.standard_normal(n).astype(np.float32).astype(np.float16).astype(np.float32)
    r = np.zeros(n, np.float32) if rs.rand() < 0.4 else (rs.standard_normal(n) * 0.3).astype(np.float32)
    if rs.rand() < 0.2:
        r = (-g).astype(np.float32)
    return rs, off, np.array(ks, np.int32), g, r


def test_configuration_model_fed_with_measured_costs():
    # Sec. V-C closed loop, as bench.py runs it: R_B(b) and C_B(b) measured with this library (window merge
    # fed from page-locked host memory; diffs copied out to it), handed to ld_config_select over the 24
    # candidates of the paper's Example; every T_w and the selection must be what the oracle's Eq. (10) gives
    # for the same measured inputs.
    import bench
    leg = bench.SparseLeg(synth.workload("resnet50"), torch.device(DEV), pool=4)
    leg.step(bench.Timer())            # fills the window's 50 diffs
    torch.cuda.synchronize()
    row = bench.config_model_row(leg)
    st, ms = row["stated"], row["measured_s"]
    fs, bs = (10, 30, 50, 100), row["b_values"]
    assert list(bs) == [1, 2, 3, 4, 5, 6]
    tw = {}
    for f in fs:
        for b in bs:
            tw[(f, b)] = oracle.wasted_time(st["N"], st["T_s"], st["M_s"], st["tau_s"], f, b, ms["R_F"], ms["R_B"][str(b)],
                                            ms["C_F"], ms["C_B"][str(b)])
    best = min(tw, key=tw.get)
    assert (row["selected"]["f"], row["selected"]["b"]) == best
    assert abs(row["selected"]["T_w_s"] - tw[best]) <= 1e-12 * tw[best]
    for f in fs:
        for j, b in enumerate(bs):
            assert abs(row["T_w_normalised"][f"f={f}"][j] - tw[(f, b)] / tw[best]) <= 1e-12 * tw[(f, b)] / tw[best]
    for b in bs:
        want = oracle.critical_interval(st["M_s"], st["tau_s"], b, ms["R_B"][str(b)], ms["C_F"], ms["C_B"][str(b)])
        assert abs(row["f_c"][str(b)] - want) <= 1e-12 * want
        assert 0 < ms["C_replay"][str(b)] <= ms["R_B"][str(b)]      # replay is part of the recovery of a batch
    assert all(ms["R_B"][str(b)] > 0 and ms["C_B"][str(b)] > 0 for b in bs) and ms["C_F"] > 0 and ms["R_F"] > 0


def test_binding_temporaries_outlive_work_on_a_side_stream():
    # The binding allocates a workspace itself when none is given and drops it when the call
    # returns. With the kernels enqueued on a side stream that is still busy, torch's allocator
    # must not hand that block to the next allocation on the default stream: the block is marked as
    # in use on the side stream. Here the default stream grabs and zeroes same-sized blocks right
    # after the call (an all-zero chunk table would make the merge skip every record).
    n, W = 6_000_000, 12
    rs = np.random.RandomState(5)
    w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
    idxs, vals = [], []
    for t in range(W):
        i = np.sort(rs.choice(n, n // 100, replace=False)).astype(np.int32)
        idxs.append(i)
        vals.append(rs.standard_normal(i.size).astype(np.float32))
    ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
    gi, gv = [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals]
    ws_bytes = ld.ld_merge_sparse_workspace(n, [i.size for i in idxs])
    side = torch.cuda.Stream()
    ballast = torch.empty(1 << 28, dtype=torch.float32, device=DEV)  # 1 GiB: each fill keeps the side stream busy
    w = to_gpu(w0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(12):
            ballast.fill_(1.0)
    ld.ld_merge_sparse(w, gi, gv, 0.1, stream=side, strategy=ld.LD_MERGE_SWEEP)   # workspace allocated inside
    grabbed = [torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV) for _ in range(4)]  # default stream, at once
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref))
    del grabbed, ballast


@pytest.mark.parametrize("block", range(4))
def test_randomised_shapes_against_the_oracle(block):
    for seed in range(100 * block, 100 * block + 12):
        rs, off, k, g, r = _random_case(seed)
        n = int(off[-1])
        print(f"[random] seed={seed} n={n} n_seg={len(k)} K={int(k.sum())}", flush=True)
        W = int(rs.choice([1, 2, 5]))
        idxs, vals, r_ref = [], [], r
        r_gpu = to_gpu(r)
        for t in range(W):
            gt = g if t == 0 else (rs.standard_normal(n) * 0.5).astype(np.float32)
            oi, ov, r_ref = oracle.topk_ef(gt, r_ref, off, k, select=True)
            nbytes = ld.ld_compress_topk_workspace(off) if rs.rand() < 0.3 else ld.ld_compress_topk_workspace(off, k)
            gi, gv = ld.ld_compress_topk(to_gpu(gt), r_gpu, off, k,
                                         workspace=torch.empty(nbytes, dtype=torch.uint8, device=DEV))
            torch.cuda.synchronize()
            np.testing.assert_array_equal(gi.cpu().numpy(), oi, err_msg=f"idx seed {seed} t {t}")
            np.testing.assert_array_equal(bits(gv.cpu().numpy()), bits(ov), err_msg=f"val seed {seed} t {t}")
            np.testing.assert_array_equal(bits(r_gpu.cpu().numpy()), bits(r_ref), err_msg=f"residual seed {seed} t {t}")
            idxs.append(oi)
            vals.append(ov)
        if n == 0:
            continue
        w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
        ref = oracle.merge_sparse(w0, idxs, vals, 0.1)
        for strategy in (ld.LD_MERGE_SWEEP, ld.LD_MERGE_SCATTER):
            w = to_gpu(w0)
            ld.ld_merge_sparse(w, [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], 0.1, strategy=strategy)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(bits(w.cpu().numpy()), bits(ref), err_msg=f"merge seed {seed}")
        z = np.zeros(n, np.float32)
        wa, ma, va = to_gpu(w0), to_gpu(z), to_gpu(z)
        ld.ld_merge_sparse_adam(wa, ma, va, [to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], 3, 1e-3, **synth.ADAM)
        torch.cuda.synchronize()
        check_adam_close((wa, ma, va), oracle.sparse_adam_replay(w0, z, z, idxs, vals, 3, 1e-3, **synth.ADAM),
                         f"sparse adam seed {seed}")
        ci, cv, cn = ld.ld_combine_sparse([to_gpu(i) for i in idxs], [to_gpu(v) for v in vals], n, 1.0)
        torch.cuda.synchronize()
        ei, ev = oracle.combine_sparse(idxs, vals, n, 1.0)
        cnt = int(cn.item())
        assert cnt == ei.size, f"combine count seed {seed}"
        np.testing.assert_array_equal(ci[:cnt].cpu().numpy(), ei, err_msg=f"combine idx seed {seed}")
        np.testing.assert_array_equal(bits(cv[:cnt].cpu().numpy()), bits(ev), err_msg=f"combine val seed {seed}")


def test_randomised_dense_replays_against_the_oracle():
    rs = np.random.RandomState(77)
    for case in range(16):
        n = int(rs.choice([1, 3, 4095, 4096, 4097, 65537, 300001, 1500000]))
        W = int(rs.randint(1, 10))
        step0 = int(rs.choice([0, 1, 7, 1000, 123456]))
        hp = dict(lr=float(10.0 ** rs.uniform(-5, -2)), beta1=float(rs.choice([0.0, 0.8, 0.9])),
                  beta2=float(rs.choice([0.9, 0.99, 0.999])), eps=float(rs.choice([1e-8, 1e-6])))
        print(f"[random dense] case={case} n={n} W={W} step0={step0} {hp}", flush=True)
        w0 = (rs.standard_normal(n) * 0.02).astype(np.float32)
        m0 = (rs.standard_normal(n) * 1e-3).astype(np.float32)
        v0 = (rs.standard_normal(n) ** 2 * 1e-6).astype(np.float32)
        scale = float(10.0 ** rs.uniform(-4, 0))
        grads = [torch.from_numpy((rs.standard_normal(n) * scale).astype(np.float32)).to(torch.bfloat16) for _ in range(W)]
        gbits = [g.view(torch.int16).numpy().view(np.uint16) for g in grads]
        src = [g.to(DEV) for g in grads]
        snaps = [torch.empty_like(s) for s in src]
        if case % 2:
            ld.ld_snapshot_layers(src, snaps)
        else:
            for a, b in zip(src, snaps):
                ld.ld_snapshot_layer(a, b)
        w, m, v = to_gpu(w0), to_gpu(m0), to_gpu(v0)
        ld.ld_merge_dense_adam(w, m, v, snaps, step0, **hp)
        torch.cuda.synchronize()
        for s_, b_ in zip(snaps, gbits):
            np.testing.assert_array_equal(s_.cpu().view(torch.int16).numpy().view(np.uint16), b_)
        check_adam_close((w, m, v), oracle.adam_replay(w0, m0, v0, gbits, step0, **hp), f"case {case}")

"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2509_04084_amd import lowdiff as ld

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a non-NULL, 256-byte aligned address that is never dereferenced on an error path


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lowdiff.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ld_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ld.load()
    names = declared_functions()
    assert {"ld_compress_topk", "ld_snapshot_layer", "ld_merge_sparse", "ld_merge_dense_adam"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_status_strings():
    assert ld.status_string(0) == "LD_OK"
    for code in (-1, -2, -3, -4, -5):
        assert ld.status_string(code).startswith("LD_ERR_")
    assert "unknown" in ld.status_string(-99)


def _p(a):
    return ctypes.c_void_p(a.ctypes.data)


def test_compress_argument_errors():
    lib = ld.load()
    off = np.array([0, 100, 300], np.int64)
    k = np.array([1, 2], np.int32)
    ws_bytes = lib.ld_compress_topk_workspace(2, _p(off))
    assert ws_bytes >= 256
    V = ctypes.c_void_p

    def call(grad=FAKE, res=FAKE, off=off, k=k, n_seg=2, oi=FAKE, ov=FAKE, ws=FAKE, wsb=ws_bytes):
        return lib.ld_compress_topk(V(grad), V(res), _p(off) if off is not None else V(0),
                                    _p(k) if k is not None else V(0), n_seg, V(oi), V(ov), V(ws), wsb, V(0))

    assert call(grad=0) == -1 and call(res=0) == -1 and call(oi=0) == -1 and call(off=None) == -1
    assert call(n_seg=-1) == -2
    assert call(k=np.array([1, 201], np.int32)) == -2            # k_s > n_s
    assert call(k=np.array([-1, 2], np.int32)) == -2
    assert call(off=np.array([0, 300, 100], np.int64)) == -2      # decreasing
    assert call(off=np.array([1, 100, 300], np.int64)) == -2      # does not start at 0
    big = np.array([0, 2 ** 31], np.int64)
    assert lib.ld_compress_topk(V(FAKE), V(FAKE), _p(big), _p(np.array([1], np.int32)), 1, V(FAKE), V(FAKE),
                                V(FAKE), 1 << 40, V(0)) == -2     # n > 2^31 - 1
    assert call(grad=FAKE + 4) == -5 and call(res=FAKE + 8) == -5
    assert call(ws=0) == -3 and call(wsb=ws_bytes - 1) == -3 and call(ws=FAKE + 16) == -3
    assert call(n_seg=0) == 0                                     # nothing to do
    assert lib.ld_compress_topk_workspace(2, _p(np.array([0, 300, 100], np.int64))) == 0


def test_compress_workspace_for_density():
    # the density-aware query never asks for less than the minimum, equals it at the usual 1 %,
    # grows with the density of the large segments only, and is 0 for a malformed table
    off = np.array([0, 1000, 2_000_000, 2_100_000], np.int64)
    base = ld.ld_compress_topk_workspace(off)
    sizes = np.diff(off)

    def at(frac):
        return ld.ld_compress_topk_workspace(off, np.maximum(1, (sizes * frac).astype(np.int32)))

    assert at(0.001) == base and at(0.01) == base
    assert base < at(0.05) < at(0.10) < at(0.25)
    dense_small = np.array([1000, 20000, 1000], np.int32)   # only the 1000-element segment is dense
    assert ld.ld_compress_topk_workspace(off, dense_small) == base
    lib = ld.load()
    assert lib.ld_compress_topk_workspace_for(2, _p(np.array([0, 300, 100], np.int64)),
                                              _p(np.array([1, 1], np.int32))) == 0
    assert lib.ld_compress_topk_workspace_for(2, _p(off), ctypes.c_void_p(0)) == 0


def test_check_diff_argument_errors():
    lib = ld.load()
    V = ctypes.c_void_p
    lib.ld_check_diff.restype = ctypes.c_int32
    assert lib.ld_check_diff(V(FAKE), V(FAKE), -1, 10, V(FAKE), V(0)) == -2
    assert lib.ld_check_diff(V(FAKE), V(FAKE), 5, 2 ** 31, V(FAKE), V(0)) == -2
    assert lib.ld_check_diff(V(FAKE), V(FAKE), 5, 10, V(0), V(0)) == -1
    assert lib.ld_check_diff(V(0), V(FAKE), 5, 10, V(FAKE), V(0)) == -1
    assert lib.ld_check_diff(V(FAKE + 2), V(FAKE), 5, 10, V(FAKE), V(0)) == -5
    assert lib.ld_check_diff(V(FAKE), V(FAKE), 5, 10, V(FAKE + 4), V(0)) == -5


def test_merge_sparse_argument_errors():
    lib = ld.load()
    V = ctypes.c_void_p
    K = np.array([10, 20], np.int64)
    ptrs = (ctypes.c_void_p * 2)(FAKE, FAKE)
    wsb = lib.ld_merge_sparse_workspace(1000, 2, _p(K))

    def call(w=FAKE, n=1000, idx=ptrs, val=ptrs, K=K, W=2, ws=FAKE, wsb=wsb, strat=1):
        return lib.ld_merge_sparse_strategy(V(w), n, idx, val, _p(K), W, ctypes.c_float(0.1), V(ws), wsb,
                                            V(0), strat)

    assert call(w=0) == -1
    assert call(n=-1) == -2 and call(n=2 ** 31) == -2 and call(W=-1) == -2 and call(W=ld.LD_MAX_WINDOW + 1) == -2
    assert call(K=np.array([10, 1001], np.int64)) == -2 and call(K=np.array([-1, 5], np.int64)) == -2
    assert call(idx=(ctypes.c_void_p * 2)(FAKE, 0)) == -1
    assert call(w=FAKE + 4) == -5 and call(val=(ctypes.c_void_p * 2)(FAKE, FAKE + 2)) == -5
    assert call(ws=0) == -3 and call(wsb=wsb - 1) == -3
    assert call(strat=7) == -2
    assert call(W=0) == 0 and call(n=0, K=np.array([0, 0], np.int64)) == 0


def test_merge_from_host_argument_errors():
    lib = ld.load()
    V = ctypes.c_void_p
    K = np.array([10, 0, 5], np.int64)
    hp = (ctypes.c_void_p * 3)(FAKE, FAKE, FAKE)
    stg = lib.ld_merge_sparse_from_host_staging(_p(K), 3, 2)
    assert stg == 2 * 2 * 256                                  # two slots, one diff of <= 256 B (idx + val) each... the larger group
    assert lib.ld_merge_sparse_from_host_staging(_p(K), 3, 0) == 0
    assert lib.ld_merge_sparse_from_host_staging(_p(K), 3, 65) == 0

    def call(w=FAKE, n=100, hi=hp, hv=hp, K=K, W=3, group=2, stg_p=FAKE, stg_b=stg, ws=FAKE, wsb=1 << 20):
        return lib.ld_merge_sparse_from_host(V(w), n, hi, hv, _p(K), W, ctypes.c_float(0.1), group, V(stg_p), stg_b,
                                             V(ws), wsb, V(0), V(0))

    assert call(w=0) == -1 and call(hi=None) == -1
    assert call(group=0) == -2 and call(group=65) == -2 and call(n=2 ** 31) == -2
    assert call(K=np.array([10, 101, 5], np.int64)) == -2      # more records than elements
    assert call(stg_p=0) == -3 and call(stg_b=stg - 1) == -3 and call(ws=0) == -3 and call(wsb=8) == -3
    assert call(W=0) == 0 and call(n=0) == 0


def test_dense_argument_errors():
    lib = ld.load()
    V = ctypes.c_void_p
    assert lib.ld_snapshot_layer(V(0), V(FAKE), 10, V(0)) == -1
    assert lib.ld_snapshot_layer(V(FAKE), V(FAKE), -1, V(0)) == -2
    assert lib.ld_snapshot_layer(V(FAKE + 1), V(FAKE), 10, V(0)) == -5
    assert lib.ld_snapshot_layer(V(0), V(0), 0, V(0)) == 0
    g = (ctypes.c_void_p * 2)(FAKE, FAKE)
    f = ctypes.c_float

    def adam(w=FAKE, m=FAKE, v=FAKE, n=100, g=g, W=2, step0=0, b1=0.9, b2=0.999):
        return lib.ld_merge_dense_adam(V(w), V(m), V(v), n, g, W, step0, f(1e-4), f(b1), f(b2), f(1e-8), V(0))

    assert adam(w=0) == -1 and adam(g=(ctypes.c_void_p * 2)(FAKE, 0)) == -1
    assert adam(n=-1) == -2 and adam(W=65) == -2 and adam(step0=-1) == -2 and adam(b1=1.0) == -2
    assert adam(m=FAKE + 4) == -5 and adam(g=(ctypes.c_void_p * 2)(FAKE, FAKE + 2)) == -5
    assert adam(W=0) == 0 and adam(n=0) == 0


def test_sparse_adam_argument_errors():
    lib = ld.load()
    K = np.array([4], np.int64)
    one = ctypes.c_void_p(256)  # never dereferenced: every call below fails its checks first
    ptrs = (ctypes.c_void_p * 1)(256)
    f = ctypes.c_float
    args = lambda **kw: [kw.get("w", one), kw.get("m", one), kw.get("v", one), kw.get("n", 100), ptrs, ptrs,
                         _p(K), kw.get("W", 1), kw.get("step0", 0), f(1e-4), f(kw.get("b1", 0.9)), f(0.999), f(1e-8),
                         kw.get("ws", one), kw.get("wsb", 1 << 20), None]
    assert lib.ld_merge_sparse_adam(*args(n=-1)) == -2
    assert lib.ld_merge_sparse_adam(*args(n=1 << 31)) == -2
    assert lib.ld_merge_sparse_adam(*args(step0=-1)) == -2
    assert lib.ld_merge_sparse_adam(*args(b1=1.0)) == -2
    assert lib.ld_merge_sparse_adam(*args(m=ctypes.c_void_p(0))) == -1
    assert lib.ld_merge_sparse_adam(*args(v=ctypes.c_void_p(8))) == -5
    assert lib.ld_merge_sparse_adam(*args(ws=ctypes.c_void_p(0))) == -3
    assert lib.ld_merge_sparse_adam(*args(wsb=0)) == -3
    assert lib.ld_merge_sparse_adam(*args(W=0)) == 0
    assert lib.ld_merge_sparse_adam_workspace(1 << 20, 20, _p(np.full(20, 100, np.int64))) >= 20 * 22 * 4


def test_combine_argument_errors():
    lib = ld.load()
    V = ctypes.c_void_p
    K = np.array([4, 4], np.int64)
    ptrs = (ctypes.c_void_p * 2)(FAKE, FAKE)
    f = ctypes.c_float

    def call(N=2, n=100, idx=ptrs, K=K, oi=FAKE, ov=FAKE, cap=8, cnt=FAKE, ws=FAKE, wsb=1 << 20):
        return lib.ld_combine_sparse(idx, ptrs, _p(K), N, n, f(1.0), V(oi), V(ov), cap, V(cnt), V(ws), wsb, V(0))

    assert call(n=-1) == -2 and call(n=1 << 31) == -2 and call(N=65) == -2 and call(cap=-1) == -2
    assert call(K=np.array([4, 101], np.int64)) == -2
    assert call(cnt=0) == -1 and call(oi=0) == -1 and call(idx=(ctypes.c_void_p * 2)(FAKE, 0)) == -1
    assert call(cnt=FAKE + 4) == -5 and call(ov=FAKE + 2) == -5
    assert call(ws=0) == -3 and call(wsb=16) == -3
    assert lib.ld_combine_sparse_workspace(1 << 20, 8) >= 8 * 22 * 4 + 128 * 4


def test_config_model_matches_oracle():
    import oracle
    P = dict(N=32.0, T=3.0e5, M=3600.0, tau=2.1, R_F=12.0, C_F=40.0)
    p = ld.ConfigParams(**P)
    cand_f, cand_b, R_B, C_B = [], [], [], []
    for f in (10, 30, 50, 100):
        for b in (1, 2, 3, 4, 5, 6):
            cand_f.append(f)
            cand_b.append(b)
            R_B.append(0.3 * b + 0.05)      # replay of b diffs + a fixed read latency
            C_B.append(0.8 + 0.25 * b)      # one I/O request + b records
    best, tw = ld.ld_config_select(p, cand_f, cand_b, R_B, C_B)
    want = [oracle.wasted_time(P["N"], P["T"], P["M"], P["tau"], f, b, P["R_F"], rb, P["C_F"], cb)
            for f, b, rb, cb in zip(cand_f, cand_b, R_B, C_B)]
    np.testing.assert_allclose(tw, want, rtol=1e-12)
    assert best == int(np.argmin(want))
    for b, rb, cb in ((1, 0.35, 1.05), (4, 1.25, 1.8)):
        got = ld.ld_config_critical_interval(p, b, rb, cb)
        assert abs(got - oracle.critical_interval(P["M"], P["tau"], b, rb, P["C_F"], cb)) < 1e-12 * got
        assert abs(ld.ld_config_wasted_time(p, got, b, rb, cb)
                   - oracle.wasted_time(P["N"], P["T"], P["M"], P["tau"], got, b, P["R_F"], rb, P["C_F"], cb)) < 1e-9
    # invalid arguments
    assert np.isnan(ld.ld_config_wasted_time(p, 2.0, 3.0, 1.0, 1.0))         # b > f
    assert np.isnan(ld.ld_config_critical_interval(p, 2.0, 1.0, 50.0))       # C_B >= C_F
    assert ld.load().ld_config_select(None, 1, None, None, None, None, None) == -1


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    # no built library and no working compiler: the binding must raise, there is nothing to fall back to
    from paper_2509_04084_amd import _build
    monkeypatch.setattr(ld, "_lib", None)
    monkeypatch.setattr(_build, "LIB", str(tmp_path / "liblowdiff.so"))
    monkeypatch.setenv("HIPCC", "/bin/false")
    with pytest.raises(RuntimeError):
        ld.load()
    with pytest.raises(RuntimeError):
        ld.ld_compress_topk_workspace(np.array([0, 10], np.int64))


def test_binding_refuses_mismatched_sizes_and_devices_before_any_launch():
    # The C ABI cannot know how large the caller's buffers are; the binding can, and must refuse
    # what would make a kernel run past an allocation. Nothing is launched (no GPU here).
    import torch
    off = np.array([0, 100, 300], np.int64)
    k = np.array([1, 2], np.int32)
    g, r = torch.zeros(300), torch.zeros(300)
    with pytest.raises(ValueError, match="segment table covers"):
        ld.ld_compress_topk(torch.zeros(299), torch.zeros(299), off, k)     # table longer than the tensors
    with pytest.raises(ValueError, match="segment table covers"):
        ld.ld_compress_topk(g, torch.zeros(301), off, k)                    # residual of another size
    with pytest.raises(ValueError, match="different devices"):
        ld.ld_compress_topk(g, torch.zeros(300, device="meta"), off, k)
    w = torch.zeros(64)
    gb = [torch.zeros(64, dtype=torch.bfloat16)]
    with pytest.raises(ValueError, match="w, m, v differ"):
        ld.ld_merge_dense_adam(w, torch.zeros(63), torch.zeros(64), gb, 0, 1e-4, 0.9, 0.999, 1e-8)
    with pytest.raises(ValueError, match="w, m, v differ"):
        ld.ld_merge_dense_adam(w, torch.zeros(64), torch.zeros(65), gb, 0, 1e-4, 0.9, 0.999, 1e-8)
    with pytest.raises(ValueError, match="sizes differ"):
        ld.ld_merge_dense_adam(w, torch.zeros(64), torch.zeros(64), [torch.zeros(60, dtype=torch.bfloat16)],
                               0, 1e-4, 0.9, 0.999, 1e-8)
    with pytest.raises(ValueError, match="different devices"):
        ld.ld_merge_dense_adam(w, torch.zeros(64, device="meta"), torch.zeros(64), gb, 0, 1e-4, 0.9, 0.999, 1e-8)
    with pytest.raises(ValueError, match="w, m, v differ"):
        ld.ld_merge_sparse_adam(w, torch.zeros(63), torch.zeros(64), [], [], 0, 1e-4, 0.9, 0.999, 1e-8)
    i, v = torch.zeros(4, dtype=torch.int32), torch.zeros(4)
    with pytest.raises(ValueError, match="different devices"):
        ld.ld_merge_sparse(w, [i], [torch.zeros(4, device="meta")], 0.1)


def test_static_merge_refuses_on_the_host():
    lib = ld.load()
    assert lib.ld_merge_sparse_static_limit() == 4 << 20
    V = ctypes.c_void_p
    W = 128
    K = np.full(W, 4, np.int64)
    ip = (ctypes.c_void_p * W)(*[FAKE] * W)
    n_big = 2 ** 31 - 1
    assert ld.ld_merge_sparse_workspace(n_big, K) > 4 << 20
    call = lambda w, n, W_: lib.ld_merge_sparse_static(V(w), n, ip, ip, _p(K), W_, ctypes.c_float(0.1), V(0))
    assert call(FAKE, n_big, W) == -3          # chunk table beyond the library's scratch array
    assert call(0, 1024, 1) == -1
    assert call(FAKE, 2 ** 31, 1) == -2
    assert call(FAKE + 4, 1024, 1) == -5
    assert call(FAKE, 1024, 0) == 0            # empty window: nothing to do, nothing looked up


def test_compress_paths_argument_errors():
    lib = ld.load()
    V = ctypes.c_void_p
    off = np.array([0, 100, 300], np.int64)
    wsb = lib.ld_compress_topk_workspace(2, _p(off))
    assert lib.ld_compress_topk_paths(V(FAKE), wsb, 2, _p(off), V(0), V(0), V(0)) == -1
    assert lib.ld_compress_topk_paths(V(FAKE), wsb - 1, 2, _p(off), V(FAKE), V(0), V(0)) == -3
    assert lib.ld_compress_topk_paths(V(0), wsb, 2, _p(off), V(FAKE), V(0), V(0)) == -3
    assert lib.ld_compress_topk_paths(V(FAKE), wsb, -1, _p(off), V(FAKE), V(0), V(0)) == -2
    assert lib.ld_compress_topk_paths(V(FAKE), wsb, 0, _p(off), V(FAKE), V(0), V(0)) == 0

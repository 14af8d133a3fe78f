"""ctypes binding of the LowDiff C ABI (include/lowdiff.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU, hands their
device addresses and the current HIP stream to the library, and returns.  All
arithmetic happens in the HIP kernels; there is no fallback - if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import _build

LD_OK = 0
LD_MERGE_AUTO, LD_MERGE_SWEEP, LD_MERGE_SCATTER = 0, 1, 2
LD_COMPRESS_AUTO, LD_COMPRESS_FULL = 0, 1
LD_MAX_WINDOW = 4096
LD_MAX_ADAM_WINDOW = 64

_lib = None


class LowDiffError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn}: {status_string(status)} ({status})")


def library_path() -> str:
    return _build.LIB


def load() -> ctypes.CDLL:
    """Loads liblowdiff.so (building it only if no built library is present)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_library(force=True)
    lib = ctypes.CDLL(_build.LIB)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    lib.ld_status_string.argtypes = [i32]
    lib.ld_status_string.restype = ctypes.c_char_p
    lib.ld_compress_topk_workspace.argtypes = [i32, vp]
    lib.ld_compress_topk_workspace.restype = sz
    lib.ld_merge_sparse_from_host_staging.argtypes = [vp, i32, i32]
    lib.ld_merge_sparse_from_host_staging.restype = sz
    lib.ld_merge_sparse_from_host.argtypes = [vp, i64, vp, vp, vp, i32, f32, i32, vp, sz, vp, sz, vp, vp]
    lib.ld_merge_sparse_from_host.restype = i32
    lib.ld_merge_sparse_from_host_events.argtypes = [vp, i64, vp, vp, vp, i32, f32, i32, vp, sz, vp, sz, vp, vp, vp]
    lib.ld_merge_sparse_from_host_events.restype = i32
    lib.ld_check_diff.argtypes = [vp, vp, i64, i64, vp, vp]
    lib.ld_check_diff.restype = i32
    lib.ld_compress_topk_workspace_for.argtypes = [i32, vp, vp]
    lib.ld_compress_topk_workspace_for.restype = sz
    lib.ld_compress_topk.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.ld_compress_topk.restype = i32
    lib.ld_compress_topk_strategy.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, sz, vp, i32]
    lib.ld_compress_topk_strategy.restype = i32
    lib.ld_compress_topk_paths.argtypes = [vp, sz, i32, vp, vp, vp, vp]
    lib.ld_compress_topk_paths.restype = i32
    lib.ld_snapshot_layer.argtypes = [vp, vp, i64, vp]
    lib.ld_snapshot_layer.restype = i32
    lib.ld_snapshot_layers.argtypes = [vp, vp, vp, i32, vp]
    lib.ld_snapshot_layers.restype = i32
    lib.ld_merge_sparse_workspace.argtypes = [i64, i32, vp]
    lib.ld_merge_sparse_workspace.restype = sz
    lib.ld_merge_sparse.argtypes = [vp, i64, vp, vp, vp, i32, f32, vp, sz, vp]
    lib.ld_merge_sparse.restype = i32
    lib.ld_merge_sparse_strategy.argtypes = [vp, i64, vp, vp, vp, i32, f32, vp, sz, vp, i32]
    lib.ld_merge_sparse_strategy.restype = i32
    lib.ld_merge_sparse_static_limit.argtypes = []
    lib.ld_merge_sparse_static_limit.restype = sz
    lib.ld_merge_sparse_static.argtypes = [vp, i64, vp, vp, vp, i32, f32, vp]
    lib.ld_merge_sparse_static.restype = i32
    lib.ld_merge_dense_adam.argtypes = [vp, vp, vp, i64, vp, i32, i64, f32, f32, f32, f32, vp]
    lib.ld_merge_dense_adam.restype = i32
    lib.ld_merge_sparse_adam_workspace.argtypes = [i64, i32, vp]
    lib.ld_merge_sparse_adam_workspace.restype = sz
    lib.ld_merge_sparse_adam.argtypes = [vp, vp, vp, i64, vp, vp, vp, i32, i64, f32, f32, f32, f32, vp, sz, vp]
    lib.ld_merge_sparse_adam.restype = i32
    lib.ld_combine_sparse_workspace.argtypes = [i64, i32]
    lib.ld_combine_sparse_workspace.restype = sz
    lib.ld_combine_sparse.argtypes = [vp, vp, vp, i32, i64, f32, vp, vp, i64, vp, vp, sz, vp]
    lib.ld_combine_sparse.restype = i32
    dbl = ctypes.c_double
    lib.ld_config_wasted_time.argtypes = [vp, dbl, dbl, dbl, dbl]
    lib.ld_config_wasted_time.restype = dbl
    lib.ld_config_critical_interval.argtypes = [vp, dbl, dbl, dbl]
    lib.ld_config_critical_interval.restype = dbl
    lib.ld_config_select.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.ld_config_select.restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().ld_status_string(int(status)).decode()


def _check(fn: str, status: int) -> None:
    if status != LD_OK:
        raise LowDiffError(fn, status)


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t: Optional[torch.Tensor], dtype, name: str) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def _same_device(*tensors) -> None:
    devs = {t.device for t in tensors if t is not None}
    if len(devs) > 1:
        raise ValueError(f"tensors lie on different devices: {sorted(map(str, devs))}")


def _record(t: torch.Tensor, *streams) -> torch.Tensor:
    """Marks a tensor the binding allocated as in use on the streams the library writes it on."""
    for st in streams:
        if st is not None and t.is_cuda:
            t.record_stream(st)
    return t


def _scratch(nbytes: int, device, *streams) -> torch.Tensor:
    """A temporary the binding allocates itself and drops when the call returns. The kernels that use
    it run on `streams`, which need not be the stream torch's caching allocator ties the block to:
    the block is marked as in use on each of them, so that it is not handed out again before they
    have passed this point."""
    return _record(torch.empty(max(1, int(nbytes)), dtype=torch.uint8, device=device), *streams)


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _hp(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def ld_compress_topk_workspace(seg_off, seg_k=None) -> int:
    """Workspace bytes: the minimum, or with `seg_k` the size that keeps calls of that density fast."""
    seg_off = _host(seg_off, np.int64)
    if seg_k is None:
        return int(load().ld_compress_topk_workspace(seg_off.shape[0] - 1, _hp(seg_off)))
    seg_k = _host(seg_k, np.int32)
    if seg_k.shape[0] != seg_off.shape[0] - 1:
        raise ValueError("seg_k must have one entry per segment")
    return int(load().ld_compress_topk_workspace_for(seg_off.shape[0] - 1, _hp(seg_off), _hp(seg_k)))


def ld_compress_topk(grad: torch.Tensor, residual: torch.Tensor, seg_off, seg_k,
                     out_idx: Optional[torch.Tensor] = None, out_val: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None,
                     strategy: int = LD_COMPRESS_AUTO) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per-segment top-k with error feedback; `residual` is updated in place.
    Returns (out_idx int32[K], out_val float32[K])."""
    lib = load()
    seg_off = _host(seg_off, np.int64)
    seg_k = _host(seg_k, np.int32)
    n_seg = int(seg_k.shape[0])
    if seg_off.shape[0] != n_seg + 1:
        raise ValueError("seg_off must have n_seg + 1 entries")
    if int(seg_off[-1]) != grad.numel() or grad.numel() != residual.numel():
        raise ValueError(f"segment table covers {int(seg_off[-1])} elements, grad has {grad.numel()}, "
                         f"residual has {residual.numel()}")
    _same_device(grad, residual, out_idx, out_val, workspace)
    K = int(seg_k.astype(np.int64).sum())
    if out_idx is None:
        out_idx = _record(torch.empty(K, dtype=torch.int32, device=grad.device), stream)
    if out_val is None:
        out_val = _record(torch.empty(K, dtype=torch.float32, device=grad.device), stream)
    if out_idx.numel() < K or out_val.numel() < K:
        raise ValueError("output buffers smaller than sum(seg_k)")
    if workspace is None:
        workspace = _scratch(lib.ld_compress_topk_workspace_for(n_seg, _hp(seg_off), _hp(seg_k)), grad.device, stream)
    st = lib.ld_compress_topk_strategy(
        _dev(grad, torch.float32, "grad"), _dev(residual, torch.float32, "residual"),
        _hp(seg_off), _hp(seg_k), n_seg,
        _dev(out_idx, torch.int32, "out_idx"), _dev(out_val, torch.float32, "out_val"),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream), int(strategy))
    _check("ld_compress_topk", st)
    return out_idx, out_val


LD_PATH_CANDIDATES, LD_PATH_FULL, LD_PATH_TIES = 0, 1, 2


def ld_compress_topk_paths(workspace: torch.Tensor, seg_off, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(paths, overflowed_tiles), int32 device tensors of one entry per segment: which way the last
    ld_compress_topk call that used `workspace` took for each segment (see lowdiff.h)."""
    seg_off = _host(seg_off, np.int64)
    n_seg = int(seg_off.shape[0]) - 1
    paths = torch.empty(max(n_seg, 1), dtype=torch.int32, device=workspace.device)
    over = torch.empty(max(n_seg, 1), dtype=torch.int32, device=workspace.device)
    st = load().ld_compress_topk_paths(_dev(workspace, torch.uint8, "workspace"), workspace.numel(), n_seg,
                                       _hp(seg_off), _dev(paths, torch.int32, "paths"),
                                       _dev(over, torch.int32, "overflowed_tiles"), _stream(stream))
    _check("ld_compress_topk_paths", st)
    return paths[:n_seg], over[:n_seg]


def _dev_or_pinned(t: torch.Tensor, dtype, name: str) -> ctypes.c_void_p:
    """Device tensor, or a pinned host tensor (page-locked memory is mapped into the GPU's address space)."""
    if not t.is_cuda:
        if not t.is_pinned() or t.dtype != dtype or not t.is_contiguous():
            raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU or in pinned host memory")
        return ctypes.c_void_p(t.data_ptr())
    return _dev(t, dtype, name)


def ld_snapshot_layer(grad_bf16: torch.Tensor, snap_bf16: torch.Tensor, stream=None) -> None:
    """Copies one layer's gradient into `snap_bf16`: a device tensor, or a pinned host tensor (the
    paper's device-to-host snapshot; the copy then runs at the host link's speed)."""
    if grad_bf16.numel() != snap_bf16.numel():
        raise ValueError("snapshot source and destination differ in size")
    st = load().ld_snapshot_layer(_dev(grad_bf16, torch.bfloat16, "grad_bf16"),
                                  _dev_or_pinned(snap_bf16, torch.bfloat16, "snap_bf16"),
                                  grad_bf16.numel(), _stream(stream))
    _check("ld_snapshot_layer", st)


def ld_snapshot_layers(srcs: Sequence[torch.Tensor], dsts: Sequence[torch.Tensor], stream=None) -> None:
    n = len(srcs)
    if len(dsts) != n:
        raise ValueError("srcs and dsts differ in length")
    sp = (ctypes.c_void_p * max(n, 1))(*[_dev(t, torch.bfloat16, "src").value or 0 for t in srcs])
    dp = (ctypes.c_void_p * max(n, 1))(*[_dev_or_pinned(t, torch.bfloat16, "dst").value or 0 for t in dsts])
    for a, b in zip(srcs, dsts):
        if a.numel() != b.numel():
            raise ValueError("snapshot source and destination differ in size")
    ne = np.array([t.numel() for t in srcs], dtype=np.int64)
    st = load().ld_snapshot_layers(sp, dp, _hp(ne), n, _stream(stream))
    _check("ld_snapshot_layers", st)


def ld_merge_sparse_workspace(n: int, K: Sequence[int]) -> int:
    K = _host(K, np.int64)
    return int(load().ld_merge_sparse_workspace(int(n), int(K.shape[0]), _hp(K)))


def ld_merge_sparse(w: torch.Tensor, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], lr: float,
                    workspace: Optional[torch.Tensor] = None, stream=None,
                    strategy: int = LD_MERGE_AUTO) -> None:
    """Replays the diffs (idx[t], val[t]) onto `w` in list order, in place."""
    lib = load()
    W = len(idx)
    if len(val) != W:
        raise ValueError("idx and val differ in length")
    K = np.array([t.numel() for t in idx], dtype=np.int64)
    for a, b in zip(idx, val):
        if a.numel() != b.numel():
            raise ValueError("idx[t] and val[t] differ in size")
    _same_device(w, workspace, *idx, *val)
    ip = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.int32, "idx").value or 0 for t in idx])
    vp = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.float32, "val").value or 0 for t in val])
    if workspace is None:
        workspace = _scratch(lib.ld_merge_sparse_workspace(w.numel(), W, _hp(K)), w.device, stream)
    st = lib.ld_merge_sparse_strategy(_dev(w, torch.float32, "w"), w.numel(), ip, vp, _hp(K), W,
                                      ctypes.c_float(lr), _dev(workspace, torch.uint8, "workspace"),
                                      workspace.numel(), _stream(stream), int(strategy))
    _check("ld_merge_sparse", st)


def ld_merge_sparse_static_limit() -> int:
    return int(load().ld_merge_sparse_static_limit())


def ld_merge_sparse_static(w: torch.Tensor, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], lr: float,
                           stream=None) -> None:
    """ld_merge_sparse without a workspace and without any allocation (the chunk table lies in a
    device array of the library); refuses windows beyond ld_merge_sparse_static_limit()."""
    W = len(idx)
    if len(val) != W:
        raise ValueError("idx and val differ in length")
    K = np.array([t.numel() for t in idx], dtype=np.int64)
    for a, b in zip(idx, val):
        if a.numel() != b.numel():
            raise ValueError("idx[t] and val[t] differ in size")
    ip = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.int32, "idx").value or 0 for t in idx])
    vp = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.float32, "val").value or 0 for t in val])
    st = load().ld_merge_sparse_static(_dev(w, torch.float32, "w"), w.numel(), ip, vp, _hp(K), W,
                                       ctypes.c_float(lr), _stream(stream))
    _check("ld_merge_sparse_static", st)


def ld_merge_dense_adam(w: torch.Tensor, m: torch.Tensor, v: torch.Tensor, grads_bf16: Sequence[torch.Tensor],
                        step0: int, lr: float, beta1: float, beta2: float, eps: float, stream=None) -> None:
    """Replays the bf16 gradients as Adam steps step0+1.. onto (w, m, v), in place."""
    W = len(grads_bf16)
    if m.numel() != w.numel() or v.numel() != w.numel():
        raise ValueError("w, m, v differ in size")
    for g in grads_bf16:
        if g.numel() != w.numel():
            raise ValueError("gradient and parameter sizes differ")
    _same_device(w, m, v, *grads_bf16)
    gp = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.bfloat16, "grad").value or 0 for t in grads_bf16])
    st = load().ld_merge_dense_adam(_dev(w, torch.float32, "w"), _dev(m, torch.float32, "m"),
                                    _dev(v, torch.float32, "v"), w.numel(), gp, W, int(step0),
                                    ctypes.c_float(lr), ctypes.c_float(beta1), ctypes.c_float(beta2),
                                    ctypes.c_float(eps), _stream(stream))
    _check("ld_merge_dense_adam", st)


def ld_merge_sparse_from_host(w: torch.Tensor, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], lr: float,
                              group: int = 4, staging: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None, copy_stream=None,
                              merge_stream=None, events: Optional[Sequence[int]] = None) -> None:
    """ld_merge_sparse for diffs in (pinned) host tensors: groups of `group` diffs are copied on
    `copy_stream` while the previous group is merged on `merge_stream` (default: the current stream
    for both, i.e. no overlap). The host tensors must stay alive until the copies are done.
    `events`: four hipEvent_t handles of the caller's (then the call creates none of its own)."""
    lib = load()
    W = len(idx)
    if len(val) != W:
        raise ValueError("idx and val differ in length")
    for i, v in zip(idx, val):
        if i.is_cuda or v.is_cuda or i.dtype != torch.int32 or v.dtype != torch.float32 \
                or not i.is_contiguous() or not v.is_contiguous() or i.numel() != v.numel():
            raise TypeError("host diffs: contiguous CPU int32 / float32 tensors of equal length expected")
    K = np.array([t.numel() for t in idx], dtype=np.int64)
    n = w.numel()
    group = max(1, min(int(group), 64))
    if staging is None:
        staging = _scratch(max(256, int(lib.ld_merge_sparse_from_host_staging(_hp(K), W, group))), w.device,
                           copy_stream, merge_stream)
    if workspace is None:
        workspace = _scratch(max(256, int(lib.ld_merge_sparse_workspace(n, min(group, max(W, 1)), _hp(K)))),
                             w.device, copy_stream, merge_stream)
    ip = (ctypes.c_void_p * max(W, 1))(*[t.data_ptr() for t in idx])
    vp = (ctypes.c_void_p * max(W, 1))(*[t.data_ptr() for t in val])
    ev = None
    if events is not None:
        if len(events) != 4:
            raise ValueError("events: four hipEvent_t handles expected")
        ev = (ctypes.c_void_p * 4)(*[int(e) for e in events])
    st = lib.ld_merge_sparse_from_host_events(_dev(w, torch.float32, "w"), n, ip, vp, _hp(K), W, ctypes.c_float(lr),
                                              group, _dev(staging, torch.uint8, "staging"), staging.numel(),
                                              _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                              _stream(copy_stream), _stream(merge_stream), ev)
    _check("ld_merge_sparse_from_host", st)


def ld_check_diff(idx: torch.Tensor, val: Optional[torch.Tensor], n: int,
                  counts: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Counts (indices out of range, records not strictly ascending, NaN values) of one diff.
    Returns the 3-element int64 device tensor `counts`; all zero means the diff can be merged."""
    if val is not None and val.numel() != idx.numel():
        raise ValueError("idx and val differ in length")
    if counts is None:
        counts = torch.empty(3, dtype=torch.int64, device=idx.device)
    if counts.numel() < 3:
        raise ValueError("counts needs 3 elements")
    st = load().ld_check_diff(_dev(idx, torch.int32, "idx"), _dev(val, torch.float32, "val"),
                              int(idx.numel()), int(n), _dev(counts, torch.int64, "counts"), _stream(stream))
    _check("ld_check_diff", st)
    return counts


def ld_merge_sparse_adam_workspace(n: int, K: Sequence[int]) -> int:
    K = _host(K, np.int64)
    return int(load().ld_merge_sparse_adam_workspace(int(n), int(K.shape[0]), _hp(K)))


def ld_merge_sparse_adam(w: torch.Tensor, m: torch.Tensor, v: torch.Tensor, idx: Sequence[torch.Tensor],
                         val: Sequence[torch.Tensor], step0: int, lr: float, beta1: float, beta2: float,
                         eps: float, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """Replays the sparse diffs (idx[t], val[t]) as Adam steps step0+1.. onto (w, m, v), in place."""
    lib = load()
    W = len(idx)
    if len(val) != W:
        raise ValueError("idx and val differ in length")
    if m.numel() != w.numel() or v.numel() != w.numel():
        raise ValueError("w, m, v differ in size")
    K = np.array([t.numel() for t in idx], dtype=np.int64)
    for a, b in zip(idx, val):
        if a.numel() != b.numel():
            raise ValueError("idx[t] and val[t] differ in size")
    _same_device(w, m, v, workspace, *idx, *val)
    ip = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.int32, "idx").value or 0 for t in idx])
    vp = (ctypes.c_void_p * max(W, 1))(*[_dev(t, torch.float32, "val").value or 0 for t in val])
    if workspace is None:
        workspace = _scratch(lib.ld_merge_sparse_adam_workspace(w.numel(), W, _hp(K)), w.device, stream)
    st = lib.ld_merge_sparse_adam(_dev(w, torch.float32, "w"), _dev(m, torch.float32, "m"),
                                  _dev(v, torch.float32, "v"), w.numel(), ip, vp, _hp(K), W, int(step0),
                                  ctypes.c_float(lr), ctypes.c_float(beta1), ctypes.c_float(beta2),
                                  ctypes.c_float(eps), _dev(workspace, torch.uint8, "workspace"),
                                  workspace.numel(), _stream(stream))
    _check("ld_merge_sparse_adam", st)


def ld_combine_sparse(idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], n: int, scale: float = 1.0,
                      out_idx: Optional[torch.Tensor] = None, out_val: Optional[torch.Tensor] = None,
                      out_count: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      stream=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Combines N per-worker record lists (values at equal indices added in list order).

    Returns (out_idx, out_val, out_count): the buffers (capacity sum K unless given) and a one-element
    int64 device tensor with the number of records; nothing is synchronized."""
    lib = load()
    N = len(idx)
    if len(val) != N:
        raise ValueError("idx and val differ in length")
    for a, b in zip(idx, val):
        if a.numel() != b.numel():
            raise ValueError("idx[r] and val[r] differ in size")
    K = np.array([t.numel() for t in idx], dtype=np.int64)
    dev = idx[0].device if N else torch.device("cuda", torch.cuda.current_device())
    total = int(K.sum())
    if out_idx is None:
        out_idx = _record(torch.empty(total, dtype=torch.int32, device=dev), stream)
    if out_val is None:
        out_val = _record(torch.empty(total, dtype=torch.float32, device=dev), stream)
    if out_count is None:
        out_count = _record(torch.empty(1, dtype=torch.int64, device=dev), stream)
    cap = min(out_idx.numel(), out_val.numel())
    _same_device(out_idx, out_val, out_count, workspace, *idx, *val)
    ip = (ctypes.c_void_p * max(N, 1))(*[_dev(t, torch.int32, "idx").value or 0 for t in idx])
    vp = (ctypes.c_void_p * max(N, 1))(*[_dev(t, torch.float32, "val").value or 0 for t in val])
    if workspace is None:
        workspace = _scratch(lib.ld_combine_sparse_workspace(int(n), N), dev, stream)
    st = lib.ld_combine_sparse(ip, vp, _hp(K), N, int(n), ctypes.c_float(scale),
                               _dev(out_idx, torch.int32, "out_idx"), _dev(out_val, torch.float32, "out_val"),
                               cap, _dev(out_count, torch.int64, "out_count"),
                               _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("ld_combine_sparse", st)
    return out_idx, out_val, out_count


def ld_combine_sparse_workspace(n: int, N: int) -> int:
    return int(load().ld_combine_sparse_workspace(int(n), int(N)))


class ConfigParams(ctypes.Structure):
    """ld_config_params of lowdiff.h (Sec. V-C): N, T, M, tau, R_F, C_F."""
    _fields_ = [(k, ctypes.c_double) for k in ("N", "T", "M", "tau", "R_F", "C_F")]


def ld_config_wasted_time(p: ConfigParams, f: float, b: float, R_B: float, C_B: float) -> float:
    return float(load().ld_config_wasted_time(ctypes.byref(p), f, b, R_B, C_B))


def ld_config_critical_interval(p: ConfigParams, b: float, R_B: float, C_B: float) -> float:
    return float(load().ld_config_critical_interval(ctypes.byref(p), b, R_B, C_B))


def ld_config_select(p: ConfigParams, f: Sequence[int], b: Sequence[int], R_B: Sequence[float],
                     C_B: Sequence[float]) -> Tuple[int, np.ndarray]:
    """Index of the candidate (f[i], b[i]) with the smallest wasted time, and every T_w."""
    fa, ba = _host(f, np.int32), _host(b, np.int32)
    ra, ca = _host(R_B, np.float64), _host(C_B, np.float64)
    if not (len(fa) == len(ba) == len(ra) == len(ca)):
        raise ValueError("candidate arrays differ in length")
    out = np.empty(len(fa), np.float64)
    i = load().ld_config_select(ctypes.byref(p), len(fa), _hp(fa), _hp(ba), _hp(ra), _hp(ca), _hp(out))
    return int(i), out

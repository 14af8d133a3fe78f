"""Seeded synthetic workloads: segment tables and gradient generators.

This module serves both the GPU library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic: it only says how large the
tensors of each workload are, how many records a segment keeps (the caller-side
ceil(rho*n_s) of Sec. VII-A's compression ratio), and how the stand-in gradient
values are drawn.  The paper's gradients came from ImageNet / WikiText /
RedPajama training runs; here they are random draws with the shapes and value
distributions the benchmark configurations name.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch


# --------------------------------------------------------------------------
# Segment tables (tensor sizes of the published architectures, forward order)
# --------------------------------------------------------------------------

def sizes_resnet50() -> List[int]:
    """53 conv + 53x2 batch-norm + fc weight/bias = 161 tensors, 25,557,032 elements."""
    out: List[int] = [7 * 7 * 3 * 64, 64, 64]
    inp = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            out += [inp * width, width, width]                 # 1x1 reduce + BN
            out += [3 * 3 * width * width, width, width]       # 3x3 + BN
            out += [width * width * 4, width * 4, width * 4]   # 1x1 expand + BN
            if b == 0:
                out += [inp * width * 4, width * 4, width * 4]  # downsample 1x1 + BN
            inp = width * 4
    out += [2048 * 1000, 1000]
    return out


def sizes_gpt2(n_layer: int, d: int, vocab: int = 50257, n_ctx: int = 1024) -> List[int]:
    """Token + position embedding, 12 tensors per block, final layer norm (tied head)."""
    out: List[int] = [vocab * d, n_ctx * d]
    for _ in range(n_layer):
        out += [d, d, d * 3 * d, 3 * d, d * d, d, d, d, d * 4 * d, 4 * d, 4 * d * d, d]
    out += [d, d]
    return out


def sizes_llama7b() -> List[int]:
    """Embedding, 32 x (q,k,v,o, gate, up, down, 2 norms), final norm, lm_head = 291."""
    d, f, vocab = 4096, 11008, 32000
    out: List[int] = [vocab * d]
    for _ in range(32):
        out += [d * d] * 4 + [d * f, d * f, f * d, d, d]
    out += [d, vocab * d]
    return out


def seg_offsets(sizes: Sequence[int]) -> np.ndarray:
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(np.asarray(sizes, dtype=np.int64), out=off[1:])
    return off


def seg_topk(sizes: Sequence[int], rho_num: int, rho_den: int) -> np.ndarray:
    """k_s = min(n_s, max(1, ceil(rho * n_s))) with rho = rho_num / rho_den, in integers."""
    s = np.asarray(sizes, dtype=np.int64)
    k = (s * rho_num + rho_den - 1) // rho_den
    return np.minimum(s, np.maximum(1, k)).astype(np.int32)


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    sizes: Tuple[int, ...]
    dist: str                 # "normal" | "laplace" | "student3" | "bf16_normal"
    rho: Optional[Tuple[int, int]]  # (num, den); None for the dense path
    window: int               # W: diffs per merge window
    lr: float
    w_std: float = 0.02
    scale: float = 1.0        # value scale (student3: 1e-3; bf16_normal: 1e-3)

    @property
    def n(self) -> int:
        return int(sum(self.sizes))

    @property
    def seg_off(self) -> np.ndarray:
        return seg_offsets(self.sizes)

    @property
    def seg_k(self) -> np.ndarray:
        assert self.rho is not None
        return seg_topk(self.sizes, *self.rho)


def workload(name: str) -> Workload:
    if name == "flat1m":
        return Workload(name, (1 << 20,), "normal", (1, 100), 10, 0.1)
    if name == "resnet50":
        return Workload(name, tuple(sizes_resnet50()), "laplace", (1, 100), 50, 0.1)
    if name == "gpt2s":
        return Workload(name, tuple(sizes_gpt2(12, 768)), "student3", (1, 1000), 100, 0.1,
                        scale=1e-3)
    if name == "gpt2xl":
        return Workload(name, tuple(sizes_gpt2(48, 1600)), "student3", (1, 100), 20, 0.1,
                        scale=1e-3)
    if name == "llama7b":
        return Workload(name, tuple(sizes_llama7b()), "bf16_normal", None, 4, 1e-4, scale=1e-3)
    raise KeyError(name)


ADAM = dict(beta1=0.9, beta2=0.999, eps=1e-8)

_BASE_W_SEED = 1000
_SCALE_SEED = 2000
_CHUNK = 1 << 24  # elements drawn per call, bounds the float64 temporaries


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _draw(dist: str, count: int, gen: torch.Generator, device, scale: float) -> torch.Tensor:
    """count values of the named distribution as float32 on `device`."""
    wide = torch.float64 if torch.device(device).type == "cpu" else torch.float32
    if dist == "normal":
        x = torch.randn(count, generator=gen, device=device, dtype=wide) * scale
    elif dist == "laplace":
        u = torch.rand(count, generator=gen, device=device, dtype=wide) - 0.5
        x = -scale * torch.sign(u) * torch.log1p(-2.0 * u.abs())
    elif dist == "student3":
        z = torch.randn(count, generator=gen, device=device, dtype=wide)
        c = torch.randn(3, count, generator=gen, device=device, dtype=wide).square_()
        c = (c[0] + c[1]) + c[2]  # elementwise adds (a reduction kernel over three rows gains nothing)
        x = scale * z / torch.sqrt(c / 3.0).clamp_min(1e-30)
    else:
        raise KeyError(dist)
    return x.to(torch.float32)


def segment_scales(wl: Workload) -> np.ndarray:
    """Per-segment value scale.  Laplace: b_s log-uniform in [1e-4, 1e-2]; else wl.scale."""
    if wl.dist == "laplace":
        rs = np.random.RandomState(_SCALE_SEED)
        return 10.0 ** rs.uniform(-4.0, -2.0, size=len(wl.sizes))
    return np.full(len(wl.sizes), wl.scale, dtype=np.float64)


def gradient_segment(wl: Workload, t: int, s: int, device="cpu") -> torch.Tensor:
    """Segment s of iteration t's gradient as fp32; independent of every other segment."""
    count = int(wl.sizes[s])
    scale = float(segment_scales(wl)[s])
    dist = "normal" if wl.dist == "bf16_normal" else wl.dist
    gen = _gen(device, (int(t) * 1_000_003 + s * 7919 + 17) & 0x7FFFFFFFFFFF)
    out = torch.empty(count, dtype=torch.float32, device=device)
    for c0 in range(0, count, _CHUNK):
        c1 = min(count, c0 + _CHUNK)
        out[c0:c1] = _draw(dist, c1 - c0, gen, device, scale)
    return out


def gradient(wl: Workload, t: int, device="cpu", out: Optional[torch.Tensor] = None,
             segments: Optional[Sequence[int]] = None) -> torch.Tensor:
    """Iteration t's flat fp32 gradient (seed = t).  With `segments`, only those
    segments are drawn (others left as they are in `out`)."""
    if out is None:
        out = torch.zeros(wl.n, dtype=torch.float32, device=device)
    off = wl.seg_off
    todo = range(len(wl.sizes)) if segments is None else segments
    for s in todo:
        out[int(off[s]):int(off[s + 1])] = gradient_segment(wl, t, s, device)
    return out


def gradient_layer_bf16(wl: Workload, t: int, s: int, device="cpu") -> torch.Tensor:
    """Dense-path gradient of one layer, rounded (nearest even) to bf16."""
    return gradient_segment(wl, t, s, device).to(torch.bfloat16)


def base_weights(n: int, device="cpu", std: float = 0.02) -> torch.Tensor:
    gen = _gen(device, _BASE_W_SEED)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for c0 in range(0, n, _CHUNK):
        c1 = min(n, c0 + _CHUNK)
        out[c0:c1] = _draw("normal", c1 - c0, gen, device, std)
    return out


# --------------------------------------------------------------------------
# Adversarial inputs for the selection rule (parity tests only)
# --------------------------------------------------------------------------

def adversarial_cases(n: int, seed: int = 0):
    """Yields (name, g float32[n], r float32[n]) stressing ties, zeros and extremes."""
    rs = np.random.RandomState(seed)
    z = np.zeros(n, dtype=np.float32)
    yield "all_zero", z.copy(), z.copy()
    yield "all_equal", np.full(n, 0.5, dtype=np.float32), z.copy()
    g = rs.choice(np.array([-2.0, -1.0, 1.0, 2.0], dtype=np.float32), size=n)
    yield "four_values", g, z.copy()
    g = rs.standard_normal(n).astype(np.float32)
    g[rs.rand(n) < 0.5] = np.float32(1.25)
    yield "half_at_one_value", g, z.copy()
    g = np.where(rs.rand(n) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
    yield "signed_zeros", g, z.copy()
    g = (rs.standard_normal(n) * 1e-41).astype(np.float32)  # all denormal
    yield "denormals", g, (rs.standard_normal(n) * 1e-42).astype(np.float32)
    g = (rs.standard_normal(n) * 1e-3).astype(np.float32)
    g[rs.randint(0, n)] = np.float32(3.0e38)
    yield "one_outlier", g, z.copy()
    g = rs.standard_normal(n).astype(np.float32)
    r = (-g + (rs.standard_normal(n) * 1e-6).astype(np.float32)).astype(np.float32)
    yield "cancelling_residual", g, r
    g = np.round(rs.standard_normal(n) * 4).astype(np.float32) / 4  # heavy duplication
    yield "quantised", g, np.round(rs.standard_normal(n) * 2).astype(np.float32) / 4
    g = rs.standard_normal(n).astype(np.float32)
    g[: n // 2] = np.float32(0.0)
    yield "half_zero_block", g, z.copy()
    g = np.sort(np.abs(rs.standard_normal(n))).astype(np.float32)  # winners all at the end
    yield "ascending", g, z.copy()
    yield "descending", g[::-1].copy(), z.copy()
    # infinities are ordinary keys (the largest); finite residuals keep r + g free of NaN. Enough
    # of them that some segments select only infinities and tie among them by index.
    g = (rs.standard_normal(n) * 1e-3).astype(np.float32)
    at = rs.choice(n, max(1, n // 50), replace=False)
    g[at] = np.where(rs.rand(at.size) < 0.5, np.float32(np.inf), np.float32(-np.inf))
    yield "infinities", g, (rs.standard_normal(n) * 1e-3).astype(np.float32)
    # sparse gradient (most rows untouched, as an embedding's): fewer non-zeros than k in places
    g = np.zeros(n, dtype=np.float32)
    at = rs.choice(n, max(1, n // 300), replace=False)
    g[at] = rs.standard_normal(at.size).astype(np.float32)
    yield "mostly_zero", g, z.copy()

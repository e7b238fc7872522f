"""Seeded synthetic inputs for the Monarch multiply, shared by tests and bench.

This module holds no arithmetic of the method itself: only a counter-based
normal generator, the bf16 storage conversions, and the table of workload
shapes.  Both the GPU path and the CPU oracle are fed from here, so that they
see bit-identical inputs.

Value distributions (dense i.i.d.; the paper's weights are dense inside each
block and its activations have no exploitable structure):
  x, dy ~ N(0, 1);  R ~ N(0, 1/p);  L ~ N(0, 1/q)   (second argument = variance,
  i.e. 1/fan_in, fan_in being the last dimension of the factor).
For bf16 workloads the float32 draws are rounded once to bf16 (round to nearest
even) and both implementations consume those bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 220400595
_TENSOR_ID = {"x": 0, "R": 1, "L": 2, "dy": 3, "R2": 4, "L2": 5}


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def normal(seed: int, shape, std: float = 1.0, chunk: int = 1 << 22) -> np.ndarray:
    """Counter-based N(0, std^2) float32 array: element n depends on (seed, n) only."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.float32)
    with np.errstate(over="ignore"):
        key = _mix64(np.array([seed], dtype=np.uint64) + np.uint64(0x9E3779B97F4A7C15))[0]
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            ctr = np.arange(lo, hi, dtype=np.uint64)
            a = _mix64((ctr * np.uint64(2) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15) ^ key)
            b = _mix64((ctr * np.uint64(2) + np.uint64(2)) * np.uint64(0x9E3779B97F4A7C15) ^ key)
            # 53-bit uniforms in (0, 1] and [0, 1)
            u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
            u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
            g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
            out[lo:hi] = (g * std).astype(np.float32)
    return out.reshape(shape)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    with np.errstate(over="ignore"):
        r = (u + rounding) >> np.uint32(16)
    # NaN stays NaN (not produced by the generator, kept for completeness)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    """The float32 values the storage dtype actually holds ('f32' or 'bf16')."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    raise ValueError(dtype)


@dataclass(frozen=True)
class Shape:
    """One Monarch layer: x (B, k*p) -> y (B, k*s) with R (k,q,p), L (k,s,q)."""
    name: str
    dtype: str
    B: int
    k: int
    p: int
    q: int
    s: int
    config: int = 0      # workload number (seeds depend on it)
    second: bool = False  # second layer of an MLP pair (uses the R2/L2 seeds)

    @property
    def n_in(self) -> int:
        return self.k * self.p

    @property
    def n_out(self) -> int:
        return self.k * self.s

    @property
    def esize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def fwd_flops(self) -> int:
        return 2 * self.k * self.q * (self.p + self.s) * self.B

    def bwd_flops(self) -> int:
        return 2 * self.fwd_flops()

    def fwd_bytes(self) -> int:
        e = self.esize
        return e * (self.B * (self.n_in + self.n_out) + self.k * self.q * (self.p + self.s))

    def bwd_bytes(self, wgrad_esize: int | None = None) -> int:
        e = self.esize
        eg = e if wgrad_esize is None else wgrad_esize
        w = self.k * self.q * (self.p + self.s)
        return e * (self.B * (self.n_out + 2 * self.n_in) + w) + eg * w


# The five workloads: square n = m^2 transforms (Definition 3.1) and
# Transformer projection / MLP layers with 4 blocks (the paper's ViT-B,
# GPT-2 small and GPT-2 medium layer shapes).
WORKLOADS = {
    "sq256_f32": Shape("sq256_f32", "f32", 64, 16, 16, 16, 16, config=1),
    "vitb_proj": Shape("vitb_proj", "bf16", 64 * 197, 4, 192, 192, 192, config=2),
    "gpt2s_fc1": Shape("gpt2s_fc1", "bf16", 8 * 1024, 4, 192, 192, 768, config=3),
    "sq4096": Shape("sq4096", "bf16", 16384, 64, 64, 64, 64, config=4),
    "gpt2m_fc1": Shape("gpt2m_fc1", "bf16", 16384, 4, 256, 256, 1024, config=5),
    "gpt2m_fc2": Shape("gpt2m_fc2", "bf16", 16384, 4, 1024, 256, 256, config=5, second=True),
    # the m = 16 fp32 shape at a batch large enough to be bandwidth-bound
    "sq256_f32_big": Shape("sq256_f32_big", "f32", 1 << 20, 16, 16, 16, 16, config=1),
}


# The remaining four-block layer shapes of the same models (attention output projection of
# GPT-2 medium, fused q,k,v projections, second MLP layer of GPT-2 small), at the batch of the
# workload of the same model above.  Timed by `bench.py --layers`; not part of the headline step.
MODEL_LAYERS = {
    "vitb_qkv": Shape("vitb_qkv", "bf16", 64 * 197, 4, 192, 192, 576, config=6),
    "gpt2s_fc2": Shape("gpt2s_fc2", "bf16", 8 * 1024, 4, 768, 192, 192, config=7),
    "gpt2m_proj": Shape("gpt2m_proj", "bf16", 16384, 4, 256, 256, 256, config=8),
    "gpt2m_qkv": Shape("gpt2m_qkv", "bf16", 16384, 4, 256, 256, 768, config=9),
    # width 512 (MLP-Mixer-S channel mixing, 64 images x 196 patches)
    "w512_fc1": Shape("w512_fc1", "bf16", 64 * 196, 4, 128, 128, 512, config=10),
    "w512_fc2": Shape("w512_fc2", "bf16", 64 * 196, 4, 512, 128, 128, config=11),
    # ViT-S (width 384 = 4 x 96: no tuned kernel, served by the shape-generic matrix-core kernels)
    "vits_proj": Shape("vits_proj", "bf16", 64 * 197, 4, 96, 96, 96, config=12),
    "vits_qkv": Shape("vits_qkv", "bf16", 64 * 197, 4, 96, 96, 288, config=13),
    "vits_fc1": Shape("vits_fc1", "bf16", 64 * 197, 4, 96, 96, 384, config=14),
    "vits_fc2": Shape("vits_fc2", "bf16", 64 * 197, 4, 384, 96, 96, config=15),
}


def workload(name: str) -> Shape:
    return WORKLOADS[name] if name in WORKLOADS else MODEL_LAYERS[name]


def tensor_seed(config: int, which: str) -> int:
    return BASE_SEED + 1000 * config + _TENSOR_ID[which]


def make_inputs(sh: Shape, rows: int | None = None, seed_shift: int = 0):
    """Return float32 arrays (x, R, L, dy) holding exactly-representable values of sh.dtype.

    ``rows`` overrides the batch (the first ``rows`` rows of the full workload:
    the generator is counter-based, so a prefix is a prefix).
    """
    B = sh.B if rows is None else rows
    rk, lk = ("R2", "L2") if sh.second else ("R", "L")
    cfg = sh.config + seed_shift
    x = normal(tensor_seed(cfg, "x") + (7 if sh.second else 0), (B, sh.n_in))
    R = normal(tensor_seed(cfg, rk), (sh.k, sh.q, sh.p), std=sh.p ** -0.5)
    L = normal(tensor_seed(cfg, lk), (sh.k, sh.s, sh.q), std=sh.q ** -0.5)
    dy = normal(tensor_seed(cfg, "dy") + (7 if sh.second else 0), (B, sh.n_out))
    return tuple(quantize(a, sh.dtype) for a in (x, R, L, dy))

"""Seeded synthetic inputs shaped like the paper's workloads.

Holds none of the method's arithmetic: only shapes, a counter-based random generator and
bf16 rounding, so that the CPU oracle and the HIP library can be fed the very same values.

Generator: ``numpy.random.Generator(Philox(key=seed))`` with
``seed = 1000 * config_index + tensor_index``; ``standard_normal(float32) * scale``; for
bf16 workloads the values are rounded to bf16 (round-to-nearest-even) on the host, and the
oracle is given those rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# tensor indices within a workload
T_Q, T_K, T_V, T_SWA_Q, T_SWA_K, T_SWA_V = 0, 1, 2, 3, 4, 5
T_DECODE = 10  # decode token streams start here: 10 q, 11 k, 12 v, 13 swa q, 14 swa k, 15 swa v


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    B: int
    H: int
    N: int            # prefill tokens per sequence
    d_feat: int       # d' (projected feature dim of q, k for linear attention)
    d_v: int          # value / head dim of linear attention
    d_h: int          # head dim of sliding-window attention
    w: int            # window
    dtype: str        # "f32" or "bf16"
    qk_scale: float   # scale applied to N(0,1) for linear-attention q, k
    v_scale: float
    swa_qk_scale: float
    decode_steps: int = 0

    @property
    def units(self) -> int:
        return self.B * self.H

    @property
    def D(self) -> int:
        return 1 + self.d_feat + self.d_feat * self.d_feat


WORKLOADS = {
    # tiny fp32 case the oracle finishes in well under a second
    "tiny": Workload(0, "tiny", 1, 1, 256, 16, 64, 64, 64, "f32", 0.25, 1.0, 1.0),
    # 360M-layer-shaped prefill
    "prefill_360m": Workload(1, "prefill_360m", 8, 16, 2048, 16, 64, 64, 64, "bf16", 0.5, 0.5, 0.5),
    # 1.3B-layer-shaped prefill
    "prefill_1p3b": Workload(2, "prefill_1p3b", 16, 16, 2048, 16, 128, 128, 64, "bf16", 0.5, 0.5, 0.5),
    # 1.3B-layer-shaped decode: state from a 512-token prefill, then 1024 steps
    "decode_1p3b": Workload(3, "decode_1p3b", 128, 16, 512, 16, 128, 128, 64, "bf16", 0.5, 0.5, 0.5,
                            decode_steps=1024),
    # long sequence, larger state
    "prefill_long": Workload(4, "prefill_long", 2, 16, 16384, 32, 64, 64, 128, "bf16", 0.5, 0.5, 0.5),
}


def seed_for(config_index: int, tensor_index: int) -> int:
    return 1000 * int(config_index) + int(tensor_index)


def normal(seed: int, shape, scale: float) -> np.ndarray:
    """float32 N(0, 1) * scale from a Philox stream keyed by ``seed``."""
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even; NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the float32 values they denote (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Values of ``x`` as representable in ``dtype`` ("f32" | "bf16"), returned as float32."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(x))
    raise ValueError(dtype)


def tensor(wl: Workload, tensor_index: int, shape, scale: float, dtype: str | None = None) -> np.ndarray:
    """One seeded input tensor of a workload, already rounded to the workload's dtype (float32 array)."""
    return round_to(normal(seed_for(wl.index, tensor_index), shape, scale), dtype or wl.dtype)


def linattn_inputs(wl: Workload, units: int | None = None, N: int | None = None):
    """q, k ``[U, N, d']`` and v ``[U, N, d_v]`` for the linear-attention prefill.

    ``units`` / ``N`` cut the workload down (the leading units / tokens of the full tensors
    are NOT what you get: a cut-down draw is its own seeded tensor of that shape).
    """
    U = wl.units if units is None else units
    N = wl.N if N is None else N
    q = tensor(wl, T_Q, (U, N, wl.d_feat), wl.qk_scale)
    k = tensor(wl, T_K, (U, N, wl.d_feat), wl.qk_scale)
    v = tensor(wl, T_V, (U, N, wl.d_v), wl.v_scale)
    return q, k, v


def swa_inputs(wl: Workload, units: int | None = None, N: int | None = None):
    """q, k, v ``[U, N, d_h]`` for sliding-window attention (own seeds)."""
    U = wl.units if units is None else units
    N = wl.N if N is None else N
    q = tensor(wl, T_SWA_Q, (U, N, wl.d_h), wl.swa_qk_scale)
    k = tensor(wl, T_SWA_K, (U, N, wl.d_h), wl.swa_qk_scale)
    # the tiny case runs its window attention on the linear-attention V (d_h == d_v there)
    v_index = T_V if (wl.name == "tiny" and wl.d_h == wl.d_v) else T_SWA_V
    v = tensor(wl, v_index, (U, N, wl.d_h), wl.v_scale)
    return q, k, v


def decode_inputs(wl: Workload, steps: int, units: int | None = None):
    """Per-step decode tokens: dict of ``[steps, U, dim]`` arrays (q, k, v, swa_q, swa_k, swa_v)."""
    U = wl.units if units is None else units
    return {
        "q": tensor(wl, T_DECODE + 0, (steps, U, wl.d_feat), wl.qk_scale),
        "k": tensor(wl, T_DECODE + 1, (steps, U, wl.d_feat), wl.qk_scale),
        "v": tensor(wl, T_DECODE + 2, (steps, U, wl.d_v), wl.v_scale),
        "swa_q": tensor(wl, T_DECODE + 3, (steps, U, wl.d_h), wl.swa_qk_scale),
        "swa_k": tensor(wl, T_DECODE + 4, (steps, U, wl.d_h), wl.swa_qk_scale),
        "swa_v": tensor(wl, T_DECODE + 5, (steps, U, wl.d_h), wl.v_scale),
    }


T_LINEAR = 40   # tensor indices of the projection inputs


def linear_inputs(index: int, M: int, K: int, N: int, dtype: str = "bf16"):
    """Inputs of a bias-free projection y = x W^T: activations x ``[M, K]`` ~ N(0, 1) and weights W ``[N, K]`` ~
    N(0, 1) / sqrt(K) (unit-variance outputs), rounded to ``dtype``; ``index`` keys the draw."""
    x = round_to(normal(seed_for(index, T_LINEAR), (M, K), 1.0), dtype)
    W = round_to(normal(seed_for(index, T_LINEAR + 1), (N, K), 1.0 / np.sqrt(K)), dtype)
    return x, W


T_BASECONV = 50   # tensor indices of the BaseConv gate inputs


def baseconv_gate_inputs(index: int, B: int, N: int, Dc: int, dtype: str = "bf16"):
    """Inputs of the BaseConv gate: the two projected activations a, c ``[B, N, Dc]`` ~ N(0, 1) (unit-variance
    outputs of the input projections), rounded to ``dtype``; filter taps h ``[3, Dc]`` ~ N(0, 1) / sqrt(3) and
    biases b1, b2 ``[Dc]`` ~ N(0, 0.1), fp32; ``index`` keys the draw."""
    a = round_to(normal(seed_for(index, T_BASECONV), (B, N, Dc), 1.0), dtype)
    c = round_to(normal(seed_for(index, T_BASECONV + 1), (B, N, Dc), 1.0), dtype)
    h = normal(seed_for(index, T_BASECONV + 2), (3, Dc), 1.0 / np.sqrt(3.0))
    b1 = normal(seed_for(index, T_BASECONV + 3), (Dc,), 0.1)
    b2 = normal(seed_for(index, T_BASECONV + 4), (Dc,), 0.1)
    return a, c, h, b1, b2

"""CPU oracle for the Based sequence mixer (arXiv 2402.18668) -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``based_oracle.c`` (plain C, fp64).  It shares no code
with the HIP library; only the tests, the smoke check and the benchmark's CPU-baseline
leg may import it.  The product path never does.

Array conventions: ``q, k`` are ``[U, N, d']``, ``v, y`` are ``[U, N, d_v]`` float64,
``S`` is ``[U, D, d_v]`` and ``z`` is ``[U, D]`` with ``D = 1 + d' + d'^2`` (Sec. 4) in the
feature order ``[1, x_a, x_a x_b / sqrt(2) at 1 + d' + a d' + b]`` (Eq. 4).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "based_oracle.c")
_LIB = os.path.join(_HERE, "libbased_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (``-O2 -fopenmp``); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        i = ctypes.c_int
        lib.oracle_threads.restype = i
        lib.oracle_feature_dim.restype = i
        lib.oracle_feature_dim.argtypes = [i]
        lib.oracle_state_size_symmetric.restype = ctypes.c_long
        lib.oracle_state_size_symmetric.argtypes = [i, i]
        lib.oracle_feature_map.argtypes = [dp, i, dp]
        lib.oracle_linattn_quadratic.argtypes = [dp, dp, dp, dp, i, i, i, i]
        lib.oracle_linattn_rows.argtypes = [dp, dp, dp, ip, i, dp, i, i, i, i]
        lib.oracle_linattn_state.argtypes = [dp, dp, dp, dp, i, i, i, i]
        lib.oracle_linattn_recurrent.argtypes = [dp, dp, dp, dp, dp, dp, i, i, i, i]
        lib.oracle_swa.argtypes = [dp, dp, dp, dp, i, i, i, i, ctypes.c_double]
        lib.oracle_swa_rows.argtypes = [dp, dp, dp, ip, i, dp, i, i, i, i, ctypes.c_double]
        for name in ("oracle_feature_map", "oracle_linattn_quadratic", "oracle_linattn_rows",
                     "oracle_linattn_state", "oracle_linattn_recurrent", "oracle_swa",
                     "oracle_swa_rows"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def threads() -> int:
    """OpenMP threads the oracle will use."""
    return int(_load().oracle_threads())


def feature_dim(dp: int) -> int:
    """D = 1 + d' + d'^2 (Sec. 4)."""
    return int(_load().oracle_feature_dim(int(dp)))


def state_size_symmetric(dp: int, dv: int) -> int:
    """(d + 1)(1 + 3d'/2 + d'^2/2): the recurrent-state size of the state-size appendix."""
    return int(_load().oracle_state_size_symmetric(int(dp), int(dv)))


def feature_map(x) -> np.ndarray:
    """phi(x) of Eq. 4 applied along the last axis."""
    x = np.asarray(x, dtype=np.float64)
    dp = x.shape[-1]
    D = feature_dim(dp)
    flat = np.ascontiguousarray(x.reshape(-1, dp))
    out = np.empty((flat.shape[0], D), dtype=np.float64)
    lib = _load()
    for r in range(flat.shape[0]):
        _, pin = _d(flat[r])
        lib.oracle_feature_map(pin, dp, out[r].ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out.reshape(x.shape[:-1] + (D,))


def _shapes(q, k, v):
    assert q.ndim == 3 and k.shape == q.shape and v.ndim == 3 and v.shape[:2] == q.shape[:2]
    return q.shape[0], q.shape[1], q.shape[2], v.shape[2]


def linattn_quadratic(q, k, v) -> np.ndarray:
    """Eq. 2 with the kernel of Eq. 4, every row, zero initial state."""
    q, pq = _d(q); k, pk = _d(k); v, pv = _d(v)
    U, N, dp, dv = _shapes(q, k, v)
    y = np.empty((U, N, dv), dtype=np.float64)
    _load().oracle_linattn_quadratic(pq, pk, pv, y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                     U, N, dp, dv)
    return y


def linattn_rows(q, k, v, rows) -> np.ndarray:
    """Eq. 2 at the listed token indices only; returns ``[U, len(rows), d_v]``."""
    q, pq = _d(q); k, pk = _d(k); v, pv = _d(v)
    U, N, dp, dv = _shapes(q, k, v)
    rows, pr = _i64(rows)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < N).all()
    y = np.empty((U, rows.shape[0], dv), dtype=np.float64)
    _load().oracle_linattn_rows(pq, pk, pv, pr, rows.shape[0],
                                y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), U, N, dp, dv)
    return y


def linattn_state(k, v, S=None, z=None):
    """S = S0 + sum_j phi(k_j) v_j^T and z = z0 + sum_j phi(k_j) (Sec. 3.1); returns copies."""
    k, pk = _d(k); v, pv = _d(v)
    U, N, dp = k.shape
    dv = v.shape[2]
    D = feature_dim(dp)
    S = np.zeros((U, D, dv)) if S is None else np.array(S, dtype=np.float64, order="C")
    z = np.zeros((U, D)) if z is None else np.array(z, dtype=np.float64, order="C")
    assert S.shape == (U, D, dv) and z.shape == (U, D)
    p = ctypes.POINTER(ctypes.c_double)
    _load().oracle_linattn_state(pk, pv, S.ctypes.data_as(p), z.ctypes.data_as(p), U, N, dp, dv)
    return S, z


def linattn_recurrent(q, k, v, S=None, z=None):
    """Eq. 3 from a given state (zero if omitted); returns ``(y, S_final, z_final)``."""
    q, pq = _d(q); k, pk = _d(k); v, pv = _d(v)
    U, N, dp, dv = _shapes(q, k, v)
    D = feature_dim(dp)
    S = np.zeros((U, D, dv)) if S is None else np.array(S, dtype=np.float64, order="C")
    z = np.zeros((U, D)) if z is None else np.array(z, dtype=np.float64, order="C")
    assert S.shape == (U, D, dv) and z.shape == (U, D)
    y = np.empty((U, N, dv), dtype=np.float64)
    p = ctypes.POINTER(ctypes.c_double)
    _load().oracle_linattn_recurrent(pq, pk, pv, y.ctypes.data_as(p), S.ctypes.data_as(p),
                                     z.ctypes.data_as(p), U, N, dp, dv)
    return y, S, z


def linattn_numerator(q, k, v, S=None) -> np.ndarray:
    """The numerator of Eq. 2 alone, every row (what Alg. 1 and Alg. 2 output as printed, and what the
    captions of the kernel timing figures say is timed):
    ``y_i = sum_{j<=i} (1 + q_i.k_j + (q_i.k_j)^2 / 2) v_j``, plus ``phi(q_i) S0`` for an initial
    KV-state ``S`` ``[U, D, d_v]``.  The definition written out with library matrix products."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    _shapes(q, k, v)
    A = np.einsum("uia,uja->uij", q, k)
    W = np.tril(1.0 + A + 0.5 * A * A)
    y = np.einsum("uij,ujc->uic", W, v)
    if S is not None:
        y = y + np.einsum("uif,ufc->uic", feature_map(q), np.asarray(S, dtype=np.float64))
    return y


def linattn_decay(q, k, v, gamma, S=None, z=None, gate=None):
    """Taylor linear attention with a fixed decay rate per unit (appendix paragraph on decay: one rate per
    head, the same for all inputs; the formula is the customary one of the works that paragraph cites):
    the recurrence of Eq. 3 with the state multiplied by gamma at every token,
        S_i = gamma S_{i-1} + phi(k_i) v_i^T,   z_i = gamma z_{i-1} + phi(k_i),   y_i = phi(q_i) S_i / phi(q_i).z_i,
    token by token in fp64; ``gamma [U]``; ``gate [U, N]`` (optional) scales row i of y (the input-dependent
    weight with which that paragraph combines the heads).  Returns ``(y, S_final, z_final)``."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    U, N, dp, dv = _shapes(q, k, v)
    gamma = np.asarray(gamma, dtype=np.float64)
    if gamma.shape != (U,):
        raise ValueError("gamma [U]")
    D = feature_dim(dp)
    S = np.zeros((U, D, dv)) if S is None else np.array(S, dtype=np.float64)
    z = np.zeros((U, D)) if z is None else np.array(z, dtype=np.float64)
    pq, pk = feature_map(q), feature_map(k)
    y = np.empty((U, N, dv))
    for i in range(N):
        S = gamma[:, None, None] * S + pk[:, i, :, None] * v[:, i, None, :]
        z = gamma[:, None] * z + pk[:, i]
        y[:, i] = np.einsum("uf,ufc->uc", pq[:, i], S) / np.einsum("uf,uf->u", pq[:, i], z)[:, None]
    if gate is not None:
        y = y * np.asarray(gate, dtype=np.float64)[:, :, None]
    return y, S, z


def swa(q, k, v, w: int, scale: float) -> np.ndarray:
    """Causal sliding-window softmax attention (Sec. 3.2 on Eq. 1), every row."""
    q, pq = _d(q); k, pk = _d(k); v, pv = _d(v)
    U, N, dh = q.shape
    assert k.shape == q.shape and v.shape == q.shape and w >= 1
    y = np.empty((U, N, dh), dtype=np.float64)
    _load().oracle_swa(pq, pk, pv, y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), U, N, dh,
                       int(w), float(scale))
    return y


def swa_rows(q, k, v, w: int, scale: float, rows) -> np.ndarray:
    """The same at the listed token indices only; returns ``[U, len(rows), d_h]``."""
    q, pq = _d(q); k, pk = _d(k); v, pv = _d(v)
    U, N, dh = q.shape
    rows, pr = _i64(rows)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < N).all()
    y = np.empty((U, rows.shape[0], dh), dtype=np.float64)
    _load().oracle_swa_rows(pq, pk, pv, pr, rows.shape[0],
                            y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), U, N, dh, int(w),
                            float(scale))
    return y


def project_heads(x, W, H: int) -> np.ndarray:
    """A projection of the layer input into per-head rows (Sec. 3; the layer listing of the appendix
    projects, splits the features into H heads and moves the head axis in front of the token axis):
    ``x [B, N, d_model]``, ``W [H d, d_model]`` (row ``h d + j`` is feature j of head h) -> ``[B, H, N, d]``."""
    x = np.asarray(x, dtype=np.float64)
    B, N, dm = x.shape
    y = linear(x.reshape(B * N, dm), W)
    d = y.shape[1] // H
    return np.ascontiguousarray(y.reshape(B, N, H, d).transpose(0, 2, 1, 3))


def project_out(y_heads, W) -> np.ndarray:
    """The output projection of a mixer layer: the heads of ``y_heads [B, H, N, d_v]`` are concatenated along
    the feature axis (head h at columns ``h d_v ..``) and projected with ``W [d_model, H d_v]`` -> ``[B, N, d_model]``."""
    y = np.asarray(y_heads, dtype=np.float64)
    B, H, N, dv = y.shape
    cat = y.transpose(0, 2, 1, 3).reshape(B * N, H * dv)
    return linear(cat, W).reshape(B, N, -1)


def rotary(x, positions, base: float = 10000.0) -> np.ndarray:
    """Rotary position encoding of the sliding-window layers (the training-settings table names it for
    those layers only; the paper gives no formula, so this is the published definition of the encoding
    it names): the head dimension is split into d_h / 2 adjacent pairs (x_{2i}, x_{2i+1}); pair i of the
    token at position p is rotated by the angle p * base^(-2i / d_h):
        x'_{2i}   = x_{2i} cos - x_{2i+1} sin,     x'_{2i+1} = x_{2i} sin + x_{2i+1} cos.
    ``x [..., N, d_h]``, ``positions [N]`` (integers).  fp64."""
    x = np.asarray(x, dtype=np.float64)
    pos = np.asarray(positions, dtype=np.float64)
    dh = x.shape[-1]
    if dh % 2 or pos.shape != (x.shape[-2],):
        raise ValueError("x [..., N, d_h] with even d_h, positions [N]")
    theta = base ** (-2.0 * np.arange(dh // 2) / dh)
    ang = pos[:, None] * theta[None, :]
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
    out[..., 1::2] = x[..., 0::2] * s + x[..., 1::2] * c
    return out


def swa_rotary(q, k, v, w: int, scale: float, pos0: int = 0, base: float = 10000.0) -> np.ndarray:
    """Sliding-window attention with rotary-encoded queries and keys: token i of the arrays sits at
    position pos0 + i.  The composition of the two definitions above, nothing else."""
    N = np.asarray(q).shape[1]
    pos = pos0 + np.arange(N)
    return swa(rotary(q, pos, base), rotary(k, pos, base), v, w, scale)


def short_conv_gate(a, c, h, b1, b2, c_prev=None) -> np.ndarray:
    """The gate of a BaseConv layer (appendix on the gated convolution; training-settings table: filter
    size 3, SiLU) between its input projections and its output projection:
        g[t] = (a[t] + b1) * silu(sum_{j<K} h[j] * c[t - j] + b2),     silu(x) = x / (1 + exp(-x)),
    every product per channel, ``a = u W1`` and ``c = u W2`` ``[B, N, Dc]``, filter ``h [K, Dc]`` (tap j
    looks j tokens back: the convolution is causal), biases ``[Dc]``.  Rows before the start of the
    sequence are zero, or the last K - 1 rows of an earlier part ``c_prev [B, K - 1, Dc]`` (oldest first).
    fp64."""
    a = np.asarray(a, dtype=np.float64); c = np.asarray(c, dtype=np.float64); h = np.asarray(h, dtype=np.float64)
    b1 = np.asarray(b1, dtype=np.float64); b2 = np.asarray(b2, dtype=np.float64)
    B, N, Dc = a.shape
    K = h.shape[0]
    if c.shape != a.shape or h.shape != (K, Dc) or b1.shape != (Dc,) or b2.shape != (Dc,):
        raise ValueError("a, c [B, N, Dc]; h [K, Dc]; b1, b2 [Dc]")
    hist = np.zeros((B, K - 1, Dc)) if c_prev is None else np.asarray(c_prev, dtype=np.float64)
    if hist.shape != (B, K - 1, Dc):
        raise ValueError("c_prev [B, K - 1, Dc]")
    ext = np.concatenate([hist, c], axis=1)          # ext[:, K - 1 + t] = c[:, t]
    conv = np.zeros_like(c)
    for j in range(K):
        conv += h[j][None, None, :] * ext[:, K - 1 - j:K - 1 - j + N]
    pre = conv + b2
    return (a + b1) * (pre / (1.0 + np.exp(-pre)))


def baseconv(u, W1, b1, W2, b2, h, W3, b3) -> np.ndarray:
    """A whole BaseConv layer as the appendix writes it: ((u W1 + b1) * silu(h * (u W2) + b2)) W3 + b3 with
    ``u [B, N, d]``, ``W1, W2 [Dc, d]``, ``W3 [d, Dc]`` (weights stored output-major like ``linear``)."""
    u = np.asarray(u, dtype=np.float64)
    B, N, d = u.shape
    a = linear(u.reshape(B * N, d), W1).reshape(B, N, -1)
    c = linear(u.reshape(B * N, d), W2).reshape(B, N, -1)
    g = short_conv_gate(a, c, h, b1, b2)
    return linear(g.reshape(B * N, -1), W3).reshape(B, N, -1) + np.asarray(b3, dtype=np.float64)


def linear(x, W) -> np.ndarray:
    """Bias-free linear projection ``y = x W^T`` (the q / k / v / output projections around the mixers,
    Sec. 3; the architecture listing gives them as bias-free linear layers): ``x [M, K]``, ``W [N, K]`` ->
    ``[M, N]``, fp64.  The definition written out with the library matrix product."""
    x = np.asarray(x, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    if x.ndim != 2 or W.ndim != 2 or x.shape[1] != W.shape[1]:
        raise ValueError("x [M, K], W [N, K]")
    return x @ W.T

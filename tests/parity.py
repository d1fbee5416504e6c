"""Shared helpers of the GPU parity tests: upload, error metric, tolerances."""
import numpy as np
import torch

TOL = {"f32": 1e-4, "bf16": 2e-2}   # fp32 paths / bf16-input fp32-accumulate paths
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def up(a: np.ndarray, dtype: str, shape=None) -> torch.Tensor:
    """Upload already-rounded float32 values as a device tensor of the workload dtype (exact)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if shape is not None:
        t = t.reshape(shape)
    return t.to(TORCH_DTYPE[dtype]).cuda().contiguous()


def down(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def check_close(got: np.ndarray, want: np.ndarray, tol: float, what: str, unit_axes=1):
    """Parity criterion.  The leading ``unit_axes`` axes index independent results ("groups"): an
    output row y_i (Eq. 2 and Eq. 1 define every row on its own, and its scale shrinks like
    1/sqrt(i)), or one unit's state tensor.  For every group
         |got - want| <= tol * (|want| + rms(want over the group))   element by element, and
         max|got - want| / max|want| <= tol.
    Returns (max elementwise excess ratio, max normwise error) for reporting."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    U = int(np.prod(want.shape[:unit_axes]))
    g = got.reshape(U, -1)
    w = want.reshape(U, -1)
    rms = np.sqrt((w * w).mean(axis=1, keepdims=True))
    err = np.abs(g - w)
    bound = tol * (np.abs(w) + rms)
    ratio = err / np.maximum(bound, 1e-300)
    worst = ratio.max()
    normwise = (err.max(axis=1) / np.maximum(np.abs(w).max(axis=1), 1e-300)).max()
    if not (worst <= 1.0 and normwise <= tol):
        idx = np.unravel_index(ratio.argmax(), ratio.shape)
        raise AssertionError(
            f"{what}: elementwise ratio {worst:.3g} (unit {idx[0]}, flat {idx[1]}: got {g[idx]:.6g} want {w[idx]:.6g}), "
            f"normwise {normwise:.3g}, tol {tol}")
    return worst, normwise

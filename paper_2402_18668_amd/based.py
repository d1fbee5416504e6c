"""ctypes binding of the C-ABI HIP library (``include/based.h``): argument marshalling only.

Every function takes torch CUDA tensors (used purely as device memory), checks their shapes and
dtypes on the host, and forwards raw pointers plus the current HIP stream to the library.  No
step of the method runs in Python or in torch; if the built library is missing the import
fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# BASED_HIP_LIB lets a developer point the binding at another build of the same library
LIB_PATH = os.environ.get("BASED_HIP_LIB") or os.path.join(_HERE, "lib", "libbased_hip.so")

F32, BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_LAUNCH, ERR_TOO_LARGE = 0, 1, 2, 3, 4
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "based_strerror", "based_version", "based_feature_dim", "based_state_bytes",
    "based_state_stride_floats", "based_state_export", "based_state_import",
    "based_prefill_workspace_bytes", "based_prefill", "based_prefill_status", "based_debug_set_poll_limit",
    "based_prefill_static",
    "based_decode_step", "based_swa_ring_bytes",
    "based_swa_prefill", "based_swa_decode", "based_decode_fused",
    "based_packed_feature_dim", "based_packed_state_stride_floats", "based_packed_state_bytes",
    "based_state_pack", "based_state_unpack", "based_decode_step_packed", "based_decode_fused_packed",
    "based_prefill_packed", "based_prefill_numerator", "based_decode_step_numerator",
    "based_swa_decode_ragged", "based_decode_fused_ragged", "based_positions_advance", "based_linear",
    "based_project_qkv", "based_project_out",
    "based_short_conv_gate", "based_rotary_table", "based_swa_prefill_rotary", "based_swa_decode_rotary",
    "based_decode_fused_rotary",
    "based_prefill_decay_workspace_bytes", "based_prefill_decay", "based_decode_step_decay",
]


class BasedError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {strerror(status)} (status {status})")
        self.status = status


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -m paper_2402_18668_amd.build` (there is no fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.based_strerror.restype = ctypes.c_char_p
    lib.based_strerror.argtypes = [i]
    lib.based_version.restype = i
    lib.based_feature_dim.restype = i
    lib.based_feature_dim.argtypes = [i]
    lib.based_state_bytes.restype = sz
    lib.based_state_bytes.argtypes = [i, i, i, i]
    lib.based_state_stride_floats.restype = sz
    lib.based_state_stride_floats.argtypes = [i, i]
    lib.based_state_export.restype = i
    lib.based_state_export.argtypes = [vp, vp, vp, i, i, i, i, vp]
    lib.based_state_import.restype = i
    lib.based_state_import.argtypes = [vp, vp, vp, i, i, i, i, vp]
    lib.based_prefill_workspace_bytes.restype = sz
    lib.based_prefill_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.based_prefill.restype = i
    lib.based_prefill.argtypes = [vp, vp, vp, vp, vp, i, vp, i, i, i, i, i, i, vp]
    lib.based_prefill_static.restype = i
    lib.based_prefill_static.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
    lib.based_prefill_status.restype = i
    lib.based_prefill_status.argtypes = [vp, i, i, i, i, i, i, vp]
    lib.based_debug_set_poll_limit.restype = None
    lib.based_debug_set_poll_limit.argtypes = [i]
    lib.based_decode_step.restype = i
    lib.based_decode_step.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    lib.based_swa_ring_bytes.restype = sz
    lib.based_swa_ring_bytes.argtypes = [i, i, i, i, i]
    lib.based_swa_prefill.restype = i
    lib.based_swa_prefill.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
    lib.based_swa_decode.restype = i
    lib.based_swa_decode.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
    lib.based_decode_fused.restype = i
    lib.based_decode_fused.argtypes = [vp, vp, vp, vp, vp, i, i, vp, vp, vp, vp, vp, i, i, i, f, i, i, i, vp]
    lib.based_packed_feature_dim.restype = i
    lib.based_packed_feature_dim.argtypes = [i]
    lib.based_packed_state_stride_floats.restype = sz
    lib.based_packed_state_stride_floats.argtypes = [i, i]
    lib.based_packed_state_bytes.restype = sz
    lib.based_packed_state_bytes.argtypes = [i, i, i, i]
    lib.based_state_pack.restype = i
    lib.based_state_pack.argtypes = [vp, vp, i, i, i, i, vp]
    lib.based_state_unpack.restype = i
    lib.based_state_unpack.argtypes = [vp, vp, i, i, i, i, vp]
    lib.based_decode_step_packed.restype = i
    lib.based_decode_step_packed.argtypes = lib.based_decode_step.argtypes
    lib.based_decode_fused_packed.restype = i
    lib.based_decode_fused_packed.argtypes = lib.based_decode_fused.argtypes
    lib.based_swa_decode_ragged.restype = i
    lib.based_swa_decode_ragged.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, f, i, vp]
    lib.based_decode_fused_ragged.restype = i
    lib.based_decode_fused_ragged.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, vp, vp, vp, vp, vp, i, i, f, i, i, i, vp]
    lib.based_prefill_packed.restype = i
    lib.based_prefill_packed.argtypes = lib.based_prefill.argtypes
    lib.based_prefill_numerator.restype = i
    lib.based_prefill_numerator.argtypes = lib.based_prefill.argtypes
    lib.based_decode_step_numerator.restype = i
    lib.based_decode_step_numerator.argtypes = lib.based_decode_step.argtypes
    lib.based_linear.restype = i
    lib.based_linear.argtypes = [vp, vp, vp, i, i, i, i, vp]
    lib.based_rotary_table.restype = i
    lib.based_rotary_table.argtypes = [vp, i, i, i, f, vp]
    lib.based_swa_prefill_rotary.restype = i
    lib.based_swa_prefill_rotary.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
    lib.based_swa_decode_rotary.restype = i
    lib.based_swa_decode_rotary.argtypes = [vp, vp, vp, vp, vp, vp, i, i, vp, i, i, i, i, f, i, vp]
    lib.based_project_qkv.restype = i
    lib.based_project_qkv.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
    lib.based_project_out.restype = i
    lib.based_project_out.argtypes = [vp, vp, vp, i, i, i, i, i, i, vp]
    lib.based_decode_fused_rotary.restype = i
    lib.based_decode_fused_rotary.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, vp, vp, vp, vp, vp, i, i, vp, i, i, f, i, i, i, vp]
    lib.based_prefill_decay_workspace_bytes.restype = sz
    lib.based_prefill_decay_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.based_prefill_decay.restype = i
    lib.based_prefill_decay.argtypes = [vp, vp, vp, vp, vp, i, vp, vp, vp, i, i, i, i, i, i, vp]
    lib.based_decode_step_decay.restype = i
    lib.based_decode_step_decay.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    lib.based_short_conv_gate.restype = i
    lib.based_short_conv_gate.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
    lib.based_positions_advance.restype = i
    lib.based_positions_advance.argtypes = [vp, i, vp]
    return lib


lib = _load()


def strerror(status: int) -> str:
    return lib.based_strerror(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, what: str):
    if status != OK:
        raise BasedError(status, what)


def _dev(*ts):
    for t in ts:
        if t is not None:
            if not t.is_cuda:
                raise ValueError("tensors must live on the GPU")
            if not t.is_contiguous():
                raise ValueError("tensors must be contiguous")


def feature_dim(d_feat: int) -> int:
    return int(lib.based_feature_dim(int(d_feat)))


def state_bytes(B: int, H: int, d_feat: int, d_v: int) -> int:
    return int(lib.based_state_bytes(B, H, d_feat, d_v))


def state_stride_floats(d_feat: int, d_v: int) -> int:
    return int(lib.based_state_stride_floats(d_feat, d_v))


def alloc_state(B: int, H: int, d_feat: int, d_v: int, device="cuda") -> torch.Tensor:
    """Zero-filled state buffer (an opaque fp32 tensor of the size the library asks for)."""
    n = state_bytes(B, H, d_feat, d_v)
    if n == 0:
        raise BasedError(ERR_UNSUPPORTED, "based_state_bytes")
    return torch.zeros(n // 4, dtype=torch.float32, device=device)


def state_export(state: torch.Tensor, B: int, H: int, d_feat: int, d_v: int):
    """Returns canonical ``S [B, H, D, d_v]`` and ``z [B, H, D]`` (fp32 device tensors)."""
    _dev(state)
    D = feature_dim(d_feat)
    S = torch.empty((B, H, D, d_v), dtype=torch.float32, device=state.device)
    z = torch.empty((B, H, D), dtype=torch.float32, device=state.device)
    _check(lib.based_state_export(_ptr(state), _ptr(S), _ptr(z), B, H, d_feat, d_v, _stream()),
           "based_state_export")
    return S, z


def state_import(state: torch.Tensor, S: torch.Tensor, z: torch.Tensor, d_feat: int):
    _dev(state, S, z)
    B, H, D, d_v = S.shape
    if S.dtype != torch.float32 or z.dtype != torch.float32 or tuple(z.shape) != (B, H, D) or D != feature_dim(d_feat):
        raise ValueError("S must be [B,H,D,d_v] fp32 and z [B,H,D] fp32")
    _check(lib.based_state_import(_ptr(state), _ptr(S), _ptr(z), B, H, d_feat, d_v, _stream()),
           "based_state_import")


def prefill_workspace_bytes(B, H, N, d_feat, d_v, dtype_code) -> int:
    return int(lib.based_prefill_workspace_bytes(B, H, N, d_feat, d_v, dtype_code))


def alloc_prefill_workspace(B, H, N, d_feat, d_v, dtype_code, device="cuda"):
    """Workspace of the size the library asks for, zero-filled once as its contract requires."""
    n = prefill_workspace_bytes(B, H, N, d_feat, d_v, dtype_code)
    if n == 0:
        return None
    return torch.zeros((n + 3) // 4, dtype=torch.float32, device=device)


def prefill_static(q, k, v, y, state=None, has_init=False):
    """based_prefill_static: based_prefill on the library's own static scratch.  Allocates nothing, so
    ``y`` must be given.  Returns the status code (the caller decides what an error means)."""
    _dev(q, k, v, y, state)
    B, H, N, dp = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or tuple(v.shape[:3]) != (B, H, N) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    if y.shape != v.shape or y.dtype != v.dtype:
        raise ValueError("y must match v")
    if state is not None and (state.dtype != torch.float32 or state.numel() * 4 < state_bytes(B, H, dp, dv)):
        raise ValueError("state buffer too small or not fp32")
    return int(lib.based_prefill_static(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(state), int(bool(has_init)),
                                        B, H, N, dp, dv, _dtype_code(q), _stream()))


def prefill_status(workspace, B, H, N, d_feat, d_v, dtype_code) -> int:
    """based_prefill_status: OK, or ERR_LAUNCH if a call on this workspace gave up a bounded wait
    (host-synchronous; clears the condition)."""
    _dev(workspace)
    return int(lib.based_prefill_status(_ptr(workspace), B, H, N, d_feat, d_v, dtype_code, _stream()))


def debug_set_poll_limit(polls: int) -> None:
    """based_debug_set_poll_limit (testing hook)."""
    lib.based_debug_set_poll_limit(int(polls))


def prefill(q, k, v, y=None, state=None, has_init=False, workspace=None, packed=False, numerator_only=False):
    """based_prefill, based_prefill_packed (``packed=True``: ``state`` is a packed-state buffer) or
    based_prefill_numerator (``numerator_only=True``: y is the numerator of Eq. 2, not divided).
    q, k ``[B,H,N,d']``; v ``[B,H,N,d_v]``; returns y (allocated if not given)."""
    _dev(q, k, v, y, state, workspace)
    B, H, N, dp = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or tuple(v.shape[:3]) != (B, H, N) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    code = _dtype_code(q)
    if y is None:
        y = torch.empty_like(v)
    elif y.shape != v.shape or y.dtype != v.dtype:
        raise ValueError("y must match v")
    sbytes = packed_state_bytes(B, H, dp, dv) if packed else state_bytes(B, H, dp, dv)
    if state is not None and (state.dtype != torch.float32 or state.numel() * 4 < sbytes):
        raise ValueError("state buffer too small or not fp32")
    need = prefill_workspace_bytes(B, H, N, dp, dv, code)
    if need and workspace is None:
        workspace = alloc_prefill_workspace(B, H, N, dp, dv, code, q.device)
    if need and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    if packed and numerator_only:
        raise ValueError("there is no packed numerator-only prefill")
    fn, what = (lib.based_prefill_packed, "based_prefill_packed") if packed else (lib.based_prefill, "based_prefill")
    if numerator_only:
        fn, what = lib.based_prefill_numerator, "based_prefill_numerator"
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(state), int(bool(has_init)),
              _ptr(workspace), B, H, N, dp, dv, code, _stream()), what)
    return y


def prefill_decay(q, k, v, gamma, y=None, state=None, has_init=False, gate=None):
    """based_prefill_decay: per-head decay ``gamma [H]`` (fp32), optional ``gate [B,N,H]`` in the input dtype."""
    _dev(q, k, v, y, state, gamma, gate)
    B, H, N, dp = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or tuple(v.shape[:3]) != (B, H, N) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    if gamma.dtype != torch.float32 or tuple(gamma.shape) != (H,) or not gamma.is_contiguous():
        raise ValueError("gamma must be contiguous fp32 [H]")
    if gate is not None and (gate.dtype != q.dtype or tuple(gate.shape) != (B, N, H) or not gate.is_contiguous()):
        raise ValueError("gate must be contiguous [B, N, H] of the input dtype")
    code = _dtype_code(q)
    if y is None:
        y = torch.empty_like(v)
    if state is not None and (state.dtype != torch.float32 or state.numel() * 4 < state_bytes(B, H, dp, dv)):
        raise ValueError("state buffer too small or not fp32")
    need = int(lib.based_prefill_decay_workspace_bytes(B, H, N, dp, dv, code))
    workspace = torch.zeros((need + 3) // 4, dtype=torch.int32, device=q.device) if need else None
    _check(lib.based_prefill_decay(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(state), int(bool(has_init)),
                                   _ptr(workspace), _ptr(gamma), _ptr(gate), B, H, N, dp, dv, code, _stream()),
           "based_prefill_decay")
    return y


def decode_step_decay(q, k, v, state, gamma, y=None, gate=None):
    """based_decode_step_decay: per-head decay ``gamma [H]`` (fp32), optional ``gate [B,H]`` in the input dtype."""
    _dev(q, k, v, y, state, gamma, gate)
    B, H, dp = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or tuple(v.shape[:2]) != (B, H) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    if gamma.dtype != torch.float32 or tuple(gamma.shape) != (H,) or not gamma.is_contiguous():
        raise ValueError("gamma must be contiguous fp32 [H]")
    if gate is not None and (gate.dtype != q.dtype or tuple(gate.shape) != (B, H) or not gate.is_contiguous()):
        raise ValueError("gate must be contiguous [B, H] of the input dtype")
    if state.dtype != torch.float32 or state.numel() * 4 < state_bytes(B, H, dp, dv):
        raise ValueError("state buffer too small or not fp32")
    if y is None:
        y = torch.empty_like(v)
    _check(lib.based_decode_step_decay(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(state), _ptr(gamma), _ptr(gate), B, H,
                                       dp, dv, _dtype_code(q), _stream()), "based_decode_step_decay")
    return y


def packed_state_bytes(B, H, d_feat, d_v) -> int:
    return int(lib.based_packed_state_bytes(B, H, d_feat, d_v))


def alloc_packed_state(B, H, d_feat, d_v, device="cuda") -> torch.Tensor:
    """Zeroed packed-state buffer ``[B*H, stride]`` (fp32)."""
    stride = int(lib.based_packed_state_stride_floats(d_feat, d_v))
    if stride == 0:
        raise BasedError(ERR_UNSUPPORTED, "based_packed_state_stride_floats")
    return torch.zeros((B * H, stride), dtype=torch.float32, device=device)


def state_pack(state, packed, B, H, d_feat, d_v):
    """based_state_pack: state buffer -> packed state buffer."""
    _dev(state, packed)
    if state.numel() * 4 < state_bytes(B, H, d_feat, d_v) or packed.numel() * 4 < packed_state_bytes(B, H, d_feat, d_v):
        raise ValueError("state buffer too small")
    _check(lib.based_state_pack(_ptr(state), _ptr(packed), B, H, d_feat, d_v, _stream()), "based_state_pack")
    return packed


def state_unpack(packed, state, B, H, d_feat, d_v):
    """based_state_unpack: packed state buffer -> state buffer."""
    _dev(state, packed)
    if state.numel() * 4 < state_bytes(B, H, d_feat, d_v) or packed.numel() * 4 < packed_state_bytes(B, H, d_feat, d_v):
        raise ValueError("state buffer too small")
    _check(lib.based_state_unpack(_ptr(packed), _ptr(state), B, H, d_feat, d_v, _stream()), "based_state_unpack")
    return state


def decode_step(q, k, v, state, y=None, packed=False, numerator_only=False):
    """based_decode_step (``packed=True``: based_decode_step_packed on a packed state;
    ``numerator_only=True``: based_decode_step_numerator, y = phi(q) S undivided).
    q, k ``[B,H,d']``; v ``[B,H,d_v]``; state updated in place."""
    _dev(q, k, v, y, state)
    B, H, dp = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or tuple(v.shape[:2]) != (B, H) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    need = packed_state_bytes(B, H, dp, dv) if packed else state_bytes(B, H, dp, dv)
    if state.dtype != torch.float32 or state.numel() * 4 < need:
        raise ValueError("state buffer too small or not fp32")
    if y is None:
        y = torch.empty_like(v)
    if packed and numerator_only:
        raise ValueError("there is no packed numerator-only decode step")
    fn, what = (lib.based_decode_step_packed, "based_decode_step_packed") if packed else (lib.based_decode_step, "based_decode_step")
    if numerator_only:
        fn, what = lib.based_decode_step_numerator, "based_decode_step_numerator"
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(state), B, H, dp, dv, _dtype_code(q), _stream()), what)
    return y


def swa_ring_bytes(B, H, w, d_h, dtype_code) -> int:
    return int(lib.based_swa_ring_bytes(B, H, w, d_h, dtype_code))


def alloc_swa_ring(B, H, w, d_h, dtype, device="cuda") -> torch.Tensor:
    code = F32 if dtype == torch.float32 else BF16
    n = swa_ring_bytes(B, H, w, d_h, code)
    if n == 0:
        raise BasedError(ERR_UNSUPPORTED, "based_swa_ring_bytes")
    return torch.zeros((B, H, 2, w, d_h), dtype=dtype, device=device)


def rotary_table(N: int, d_h: int, pos0: int = 0, base: float = 10000.0, device="cuda") -> torch.Tensor:
    """based_rotary_table: ``[N, d_h / 2, 2]`` fp32 (cos, sin) for positions pos0 .. pos0 + N - 1."""
    table = torch.empty((N, d_h // 2, 2), dtype=torch.float32, device=device)
    _check(lib.based_rotary_table(_ptr(table), int(pos0), int(N), int(d_h), float(base), _stream()),
           "based_rotary_table")
    return table


def swa_prefill(q, k, v, w: int, scale: float, y=None, ring=None, rotary=None):
    """based_swa_prefill, or based_swa_prefill_rotary (``rotary``: a table from ``rotary_table`` whose row t
    belongs to token t).  q, k, v ``[B,H,N,d_h]``."""
    _dev(q, k, v, y, ring)
    B, H, N, dh = q.shape
    if k.shape != q.shape or v.shape != q.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    if y is None:
        y = torch.empty_like(v)
    if ring is not None and (ring.dtype != q.dtype or ring.numel() != B * H * 2 * w * dh):
        raise ValueError("ring must be [B,H,2,w,d_h] of the input dtype")
    if rotary is not None:
        _dev(rotary)
        if rotary.dtype != torch.float32 or tuple(rotary.shape) != (N, dh // 2, 2) or not rotary.is_contiguous():
            raise ValueError("rotary table must be contiguous fp32 [N, d_h / 2, 2]")
        _check(lib.based_swa_prefill_rotary(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(ring), _ptr(rotary), B, H, N,
                                            dh, int(w), float(scale), _dtype_code(q), _stream()),
               "based_swa_prefill_rotary")
        return y
    _check(lib.based_swa_prefill(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(ring), B, H, N, dh, int(w),
                                 float(scale), _dtype_code(q), _stream()), "based_swa_prefill")
    return y


def _check_pos(pos, B):
    if pos.dtype != torch.int32 or pos.numel() != B or not pos.is_cuda or not pos.is_contiguous():
        raise ValueError("per-sequence positions must be a contiguous int32 device tensor of B elements")


def linear(x, W, y=None):
    """based_linear: ``y = x W^T``; x ``[..., K]``, W ``[N, K]`` (bf16); returns y ``[..., N]``."""
    _dev(x, W, y)
    K = x.shape[-1]
    N = W.shape[0]
    M = x.numel() // K
    if W.shape != (N, K) or W.dtype != x.dtype or not x.is_contiguous() or not W.is_contiguous():
        raise ValueError("x [..., K] and W [N, K] must be contiguous and of one dtype")
    if y is None:
        y = torch.empty((*x.shape[:-1], N), dtype=x.dtype, device=x.device)
    elif y.numel() != M * N or y.dtype != x.dtype or not y.is_contiguous():
        raise ValueError("y must be [..., N], contiguous, of x's dtype")
    _check(lib.based_linear(_ptr(x), _ptr(W), _ptr(y), M, K, N, _dtype_code(x), _stream()), "based_linear")
    return y


def project_qkv(x, W, H: int, d_feat: int, d_v: int):
    """based_project_qkv: x ``[B,N,d_model]``, W ``[H (2 d' + d_v), d_model]`` (rows of Wq, Wk, Wv) ->
    head-major q, k ``[B,H,N,d']`` and v ``[B,H,N,d_v]``."""
    _dev(x, W)
    B, N, dm = x.shape
    if tuple(W.shape) != (H * (2 * d_feat + d_v), dm) or W.dtype != x.dtype or not x.is_contiguous() \
            or not W.is_contiguous():
        raise ValueError("x [B, N, d_model] and W [H (2 d' + d_v), d_model] must be contiguous and of one dtype")
    q = torch.empty((B, H, N, d_feat), dtype=x.dtype, device=x.device)
    k = torch.empty_like(q)
    v = torch.empty((B, H, N, d_v), dtype=x.dtype, device=x.device)
    _check(lib.based_project_qkv(_ptr(x), _ptr(W), _ptr(q), _ptr(k), _ptr(v), B, N, dm, H, d_feat, d_v,
                                 _dtype_code(x), _stream()), "based_project_qkv")
    return q, k, v


def project_out(y_heads, W):
    """based_project_out: head-major ``[B,H,N,d_v]`` times W ``[d_model, H d_v]`` -> ``[B,N,d_model]``."""
    _dev(y_heads, W)
    B, H, N, dv = y_heads.shape
    dm = W.shape[0]
    if tuple(W.shape) != (dm, H * dv) or W.dtype != y_heads.dtype or not y_heads.is_contiguous() \
            or not W.is_contiguous():
        raise ValueError("y [B, H, N, d_v] and W [d_model, H d_v] must be contiguous and of one dtype")
    out = torch.empty((B, N, dm), dtype=y_heads.dtype, device=y_heads.device)
    _check(lib.based_project_out(_ptr(y_heads), _ptr(W), _ptr(out), B, N, H, dv, dm, _dtype_code(y_heads),
                                 _stream()), "based_project_out")
    return out


def short_conv_gate(a, c, h, b1, b2, c_prev=None, c_last=None, out=None):
    """based_short_conv_gate: ``(a + b1) * silu(causal 3-tap conv of c + b2)``; a, c ``[B,N,Dc]``, h ``[3,Dc]``
    and b1, b2 ``[Dc]`` fp32; c_prev / c_last ``[B,2,Dc]`` (rows before / at the end of the sequence)."""
    _dev(a, c, h, b1, b2, c_prev, c_last, out)
    B, N, Dc = a.shape
    if c.shape != a.shape or c.dtype != a.dtype or not a.is_contiguous() or not c.is_contiguous():
        raise ValueError("a, c must be contiguous [B, N, Dc] of one dtype")
    for t_, shp in ((h, (3, Dc)), (b1, (Dc,)), (b2, (Dc,))):
        if tuple(t_.shape) != shp or t_.dtype != torch.float32 or not t_.is_contiguous():
            raise ValueError("h [3, Dc], b1, b2 [Dc] must be contiguous fp32")
    for t_ in (c_prev, c_last):
        if t_ is not None and (tuple(t_.shape) != (B, 2, Dc) or t_.dtype != a.dtype or not t_.is_contiguous()):
            raise ValueError("c_prev / c_last must be contiguous [B, 2, Dc] of a's dtype")
    if out is None:
        out = torch.empty_like(a)
    elif out.shape != a.shape or out.dtype != a.dtype or not out.is_contiguous():
        raise ValueError("out must match a")
    _check(lib.based_short_conv_gate(_ptr(a), _ptr(c), _ptr(h), _ptr(b1), _ptr(b2), _ptr(c_prev), _ptr(out),
                                     _ptr(c_last), B, N, Dc, _dtype_code(a), _stream()), "based_short_conv_gate")
    return out


def positions_advance(pos):
    """based_positions_advance: pos[b] += 1 where pos[b] >= 1, on the current stream."""
    _check_pos(pos, pos.numel())
    _check(lib.based_positions_advance(_ptr(pos), pos.numel(), _stream()), "based_positions_advance")


def swa_decode(q, k, v, ring, pos, w: int, scale: float, y=None, rotary=None):
    """based_swa_decode (``pos`` an int) or based_swa_decode_ragged (``pos`` an int32 device tensor
    ``[B]``); with ``rotary`` (a table from position 0) based_swa_decode_rotary for either kind of ``pos``.
    q, k, v ``[B,H,d_h]``; ring updated in place."""
    _dev(q, k, v, y, ring)
    B, H, dh = q.shape
    if k.shape != q.shape or v.shape != q.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes / dtypes disagree")
    if ring.dtype != q.dtype or ring.numel() != B * H * 2 * w * dh:
        raise ValueError("ring must be [B,H,2,w,d_h] of the input dtype")
    if y is None:
        y = torch.empty_like(v)
    if rotary is not None:
        _dev(rotary)
        if rotary.dtype != torch.float32 or rotary.dim() != 3 or tuple(rotary.shape[1:]) != (dh // 2, 2) \
                or not rotary.is_contiguous():
            raise ValueError("rotary table must be contiguous fp32 [rows, d_h / 2, 2]")
        ragged = isinstance(pos, torch.Tensor)
        if ragged:
            _check_pos(pos, B)
        _check(lib.based_swa_decode_rotary(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(ring), _ptr(rotary),
                                           int(rotary.shape[0]), 0 if ragged else int(pos),
                                           _ptr(pos) if ragged else None, B, H, dh, int(w), float(scale),
                                           _dtype_code(q), _stream()), "based_swa_decode_rotary")
        return y
    if isinstance(pos, torch.Tensor):   # per-sequence positions in device memory
        _check_pos(pos, B)
        _check(lib.based_swa_decode_ragged(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(ring), _ptr(pos), B, H, dh,
                                           int(w), float(scale), _dtype_code(q), _stream()),
               "based_swa_decode_ragged")
        return y
    _check(lib.based_swa_decode(_ptr(q), _ptr(k), _ptr(v), _ptr(y), _ptr(ring), int(pos), B, H, dh,
                                int(w), float(scale), _dtype_code(q), _stream()), "based_swa_decode")
    return y


def decode_fused(q, k, v, state, swa_q, swa_k, swa_v, ring, pos, w: int, scale: float,
                 y_lin=None, y_swa=None, packed=False, rotary=None):
    """based_decode_fused (``packed=True``: based_decode_fused_packed; ``pos`` a device tensor:
    based_decode_fused_ragged; ``rotary``: a table from position 0, based_decode_fused_rotary): both decode
    steps in one launch; returns ``(y_lin, y_swa)``."""
    _dev(q, k, v, state, swa_q, swa_k, swa_v, ring, y_lin, y_swa)
    B, H, dp = q.shape
    dv = v.shape[-1]
    dh = swa_q.shape[-1]
    if k.shape != q.shape or tuple(v.shape[:2]) != (B, H) or tuple(swa_q.shape[:2]) != (B, H):
        raise ValueError("shapes disagree")
    if swa_k.shape != swa_q.shape or swa_v.shape != swa_q.shape:
        raise ValueError("window attention shapes disagree")
    for t in (k, v, swa_q, swa_k, swa_v, ring):
        if t.dtype != q.dtype:
            raise ValueError("dtypes disagree")
    need = packed_state_bytes(B, H, dp, dv) if packed else state_bytes(B, H, dp, dv)
    if state.dtype != torch.float32 or state.numel() * 4 < need:
        raise ValueError("state buffer too small or not fp32")
    if ring.numel() != B * H * 2 * w * dh:
        raise ValueError("ring must be [B,H,2,w,d_h]")
    if y_lin is None:
        y_lin = torch.empty_like(v)
    if y_swa is None:
        y_swa = torch.empty_like(swa_v)
    if rotary is not None:
        _dev(rotary)
        if rotary.dtype != torch.float32 or rotary.dim() != 3 or tuple(rotary.shape[1:]) != (dh // 2, 2) \
                or not rotary.is_contiguous():
            raise ValueError("rotary table must be contiguous fp32 [rows, d_h / 2, 2]")
        ragged = isinstance(pos, torch.Tensor)
        if ragged:
            _check_pos(pos, B)
        _check(lib.based_decode_fused_rotary(_ptr(q), _ptr(k), _ptr(v), _ptr(y_lin), _ptr(state), int(bool(packed)),
                                             dp, dv, _ptr(swa_q), _ptr(swa_k), _ptr(swa_v), _ptr(y_swa), _ptr(ring),
                                             _ptr(rotary), int(rotary.shape[0]), 0 if ragged else int(pos),
                                             _ptr(pos) if ragged else None, dh, int(w), float(scale), B, H,
                                             _dtype_code(q), _stream()), "based_decode_fused_rotary")
        return y_lin, y_swa
    if isinstance(pos, torch.Tensor):   # per-sequence positions in device memory
        _check_pos(pos, B)
        _check(lib.based_decode_fused_ragged(_ptr(q), _ptr(k), _ptr(v), _ptr(y_lin), _ptr(state), int(bool(packed)),
                                             dp, dv, _ptr(swa_q), _ptr(swa_k), _ptr(swa_v), _ptr(y_swa), _ptr(ring),
                                             _ptr(pos), dh, int(w), float(scale), B, H, _dtype_code(q), _stream()),
               "based_decode_fused_ragged")
        return y_lin, y_swa
    fn = lib.based_decode_fused_packed if packed else lib.based_decode_fused
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(y_lin), _ptr(state), dp, dv, _ptr(swa_q), _ptr(swa_k),
              _ptr(swa_v), _ptr(y_swa), _ptr(ring), int(pos), dh, int(w), float(scale), B, H,
              _dtype_code(q), _stream()),
           "based_decode_fused_packed" if packed else "based_decode_fused")
    return y_lin, y_swa

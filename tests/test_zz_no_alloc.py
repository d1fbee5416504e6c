"""based_prefill_static (the entry point for callers that cannot allocate device memory) against
based_prefill on a caller-allocated workspace: same inputs, outputs compared at the parity bar and bit
for bit, on two calls in a row, the second with a smaller input; then the size limit."""
import numpy as np
import pytest
import torch

from paper_2402_18668_amd import synth
from parity import TOL, check_close, down, up

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def based():
    from paper_2402_18668_amd import based as b
    return b


def _wl(dp, dv, dtype):
    base = synth.WORKLOADS["prefill_360m"]
    fields = {f: getattr(base, f) for f in base.__dataclass_fields__}
    fields.update(d_feat=dp, d_v=dv, dtype=dtype)
    return synth.Workload(**fields)


def _both(based, wl, B, H, N, with_state):
    dtype, dp, dv = wl.dtype, wl.d_feat, wl.d_v
    q, k, v = synth.linattn_inputs(wl, units=B * H, N=N)
    tq, tk, tv = up(q, dtype, (B, H, N, dp)), up(k, dtype, (B, H, N, dp)), up(v, dtype, (B, H, N, dv))
    st_a = based.alloc_state(B, H, dp, dv) if with_state else None
    st_b = based.alloc_state(B, H, dp, dv) if with_state else None
    if with_state:
        # a non-trivial initial state: the state after the first 100 tokens of the same draw
        based.prefill(tq[:, :, :100].contiguous(), tk[:, :, :100].contiguous(), tv[:, :, :100].contiguous(), state=st_a)
        st_b.copy_(st_a)
    y_a = based.prefill(tq, tk, tv, state=st_a, has_init=with_state)
    y_b = torch.full_like(y_a, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    status = based.prefill_static(tq, tk, tv, y_b, state=st_b, has_init=with_state)
    torch.cuda.synchronize()
    assert status == based.OK, based.strerror(status)
    assert torch.cuda.memory_allocated() == before
    code = based.F32 if dtype == "f32" else based.BF16
    assert based.prefill_status(None, B, H, N, dp, dv, code) == based.OK
    what = f"static scratch vs workspace: {dtype} d'={dp} dv={dv} B={B} H={H} N={N} state={with_state}"
    check_close(down(y_b).reshape(B * H * N, dv), down(y_a).reshape(B * H * N, dv), TOL[dtype], what)
    assert torch.equal(y_a, y_b), what
    if with_state:
        assert torch.equal(st_a, st_b), what


@pytest.mark.parametrize("dtype,dp,dv", [("bf16", 16, 64), ("bf16", 16, 128), ("bf16", 32, 64), ("f32", 16, 64)])
def test_static_scratch_two_calls_second_smaller(based, dtype, dp, dv):
    wl = _wl(dp, dv, dtype)
    _both(based, wl, 1, 2, 2048, with_state=False)   # segmented: increments travel through the scratch
    _both(based, wl, 1, 2, 700, with_state=True)     # smaller, right after, on the same scratch
    _both(based, wl, 2, 3, 130, with_state=False)


def test_static_scratch_size_limit(based):
    """Sizes whose workspace exceeds the static scratch are refused with their own status, before any launch."""
    B, H, N, dp, dv = 64, 16, 8192, 32, 128
    assert based.prefill_workspace_bytes(B, H, N, dp, dv, based.BF16) > based.STATIC_SCRATCH_BYTES
    null = None
    import ctypes
    p = ctypes.c_void_p(0x1000)   # never dereferenced: the call is refused on the host
    assert based.lib.based_prefill_static(p, p, p, p, null, 0, B, H, N, dp, dv, based.BF16, null) == based.ERR_TOO_LARGE
    assert "scratch" in based.strerror(based.ERR_TOO_LARGE)
    # the largest benchmark shapes fit
    for name in ("prefill_360m", "prefill_1p3b", "prefill_long"):
        w = synth.WORKLOADS[name]
        assert based.prefill_workspace_bytes(w.B, w.H, w.N, w.d_feat, w.d_v, based.BF16) <= based.STATIC_SCRATCH_BYTES, name

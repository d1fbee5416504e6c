"""GPU parity: every entry point of the C-ABI library against the CPU oracle on the same seeded
inputs, element by element.  Sizes span several chunks / tiles and a ragged tail."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2402_18668_amd import synth
from parity import TOL, TORCH_DTYPE, check_close, down, up

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def based():
    from paper_2402_18668_amd import based as b
    return b


def make_wl(name, **kw):
    base = synth.WORKLOADS[name]
    fields = {f: getattr(base, f) for f in base.__dataclass_fields__}
    fields.update(kw)
    return synth.Workload(**fields)


def rows(a):
    """[U, N, d] -> [U * N, d]: every output row is its own group for the parity criterion."""
    return np.asarray(a).reshape(-1, a.shape[-1])


def lin_case(wl, B, H, N):
    q, k, v = synth.linattn_inputs(wl, units=B * H, N=N)
    return q, k, v


# ------------------------------------------------------------------------------------------------
# linear attention prefill
# ------------------------------------------------------------------------------------------------
def run_prefill(based, wl, B, H, N, q, k, v, state=None, has_init=False):
    tq = up(q, wl.dtype, (B, H, N, wl.d_feat)); tk = up(k, wl.dtype, (B, H, N, wl.d_feat))
    tv = up(v, wl.dtype, (B, H, N, wl.d_v))
    y = based.prefill(tq, tk, tv, state=state, has_init=has_init)
    torch.cuda.synchronize()
    return down(y).reshape(B * H, N, wl.d_v)


def test_prefill_tiny_fp32(based):
    wl = synth.WORKLOADS["tiny"]
    q, k, v = synth.linattn_inputs(wl)
    state = based.alloc_state(wl.B, wl.H, wl.d_feat, wl.d_v)
    y = run_prefill(based, wl, wl.B, wl.H, wl.N, q, k, v, state=state)
    want = oracle.linattn_quadratic(q, k, v)
    check_close(rows(y), rows(want), TOL["f32"], "tiny prefill y")
    S, z = based.state_export(state, wl.B, wl.H, wl.d_feat, wl.d_v)
    Sw, zw = oracle.linattn_state(k, v)
    check_close(down(S).reshape(Sw.shape), Sw, TOL["f32"], "tiny prefill S")
    check_close(down(z).reshape(zw.shape), zw, TOL["f32"], "tiny prefill z")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dp,dv,B,H,N", [
    (16, 64, 2, 3, 333), (16, 128, 1, 2, 200), (32, 64, 1, 2, 150), (32, 128, 1, 1, 70),
    (16, 64, 1, 1, 1), (16, 64, 1, 2, 63), (16, 64, 1, 2, 64), (16, 128, 1, 1, 65),
    # long enough for the sequence to be cut into segments (ragged last segment and chunk)
    (16, 64, 1, 2, 1100), (16, 128, 1, 1, 1500), (16, 64, 1, 1, 2048),
    (32, 64, 1, 2, 1100), (32, 128, 1, 1, 1500), (32, 64, 1, 1, 1), (32, 128, 1, 2, 64), (32, 64, 2, 1, 65),
    # the other feature dimensions of the ablation table (fp32 vector kernel for both dtypes)
    (8, 64, 2, 2, 333), (8, 128, 1, 2, 1100), (24, 64, 1, 2, 150), (24, 128, 1, 1, 1100), (8, 64, 1, 1, 1),
    (24, 64, 1, 1, 5),
])
def test_prefill_shapes(based, dtype, dp, dv, B, H, N):
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv, dtype=dtype)
    q, k, v = lin_case(wl, B, H, N)
    state = based.alloc_state(B, H, dp, dv)
    y = run_prefill(based, wl, B, H, N, q, k, v, state=state)
    want = oracle.linattn_quadratic(q, k, v)
    check_close(rows(y), rows(want), TOL[dtype], f"prefill y {dtype} d'={dp} dv={dv} N={N}")
    S, z = based.state_export(state, B, H, dp, dv)
    Sw, zw = oracle.linattn_state(k, v)
    check_close(down(S).reshape(Sw.shape), Sw, TOL[dtype], "prefill S")
    check_close(down(z).reshape(zw.shape), zw, TOL[dtype], "prefill z")


@pytest.mark.parametrize("dtype,dp,dv,N,N1", [("f32", 16, 64, 300, 130), ("bf16", 16, 64, 300, 130),
                                               ("bf16", 16, 128, 300, 130), ("bf16", 32, 64, 300, 130),
                                               ("bf16", 16, 64, 1400, 130), ("bf16", 16, 128, 1300, 1100),
                                               # segmented second part on the fp32 vector-ALU path
                                               ("f32", 16, 64, 1400, 130), ("bf16", 32, 64, 1200, 100),
                                               ("bf16", 32, 128, 1700, 1100),
                                               ("f32", 8, 64, 300, 130), ("bf16", 24, 128, 1300, 200)])
def test_prefill_split_with_state(based, dtype, dp, dv, N, N1):
    """prefill(N) == prefill(N1) then prefill(N - N1 | state); state import/export round trip."""
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv, dtype=dtype)
    B, H = 1, 3
    q, k, v = lin_case(wl, B, H, N)
    want = oracle.linattn_quadratic(q, k, v)
    state = based.alloc_state(B, H, dp, dv)
    y1 = run_prefill(based, wl, B, H, N1, q[:, :N1], k[:, :N1], v[:, :N1], state=state)
    # round trip through the canonical layout into a fresh buffer
    S, z = based.state_export(state, B, H, dp, dv)
    state2 = based.alloc_state(B, H, dp, dv)
    based.state_import(state2, S, z, dp)
    torch.cuda.synchronize()
    assert torch.equal(state, state2)
    y2 = run_prefill(based, wl, B, H, N - N1, q[:, N1:], k[:, N1:], v[:, N1:], state=state2, has_init=True)
    check_close(rows(y1), rows(want[:, :N1]), TOL[dtype], "split prefill part 1")
    check_close(rows(y2), rows(want[:, N1:]), TOL[dtype], "split prefill part 2")
    S2, z2 = based.state_export(state2, B, H, dp, dv)
    Sw, zw = oracle.linattn_state(k, v)
    check_close(down(S2).reshape(Sw.shape), Sw, TOL[dtype], "split prefill final S")
    check_close(down(z2).reshape(zw.shape), zw, TOL[dtype], "split prefill final z")


@pytest.mark.parametrize("dtype,dp,dv", [("bf16", 16, 64), ("bf16", 16, 128), ("f32", 16, 64), ("bf16", 32, 64),
                                          ("bf16", 32, 128)])
def test_prefill_initial_state_symmetric_part(based, dtype, dp, dv):
    """y depends only on the sum of the state rows (a, b) and (b, a): an antisymmetric
    perturbation of the initial state leaves y (and the symmetric part of the final state) unchanged."""
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv, dtype=dtype)
    B, H, N, N1 = 1, 2, 700, 90
    q, k, v = lin_case(wl, B, H, N)
    want = oracle.linattn_quadratic(q, k, v)
    Sw, zw = oracle.linattn_state(k, v)
    state = based.alloc_state(B, H, dp, dv)
    run_prefill(based, wl, B, H, N1, q[:, :N1], k[:, :N1], v[:, :N1], state=state)
    S, z = based.state_export(state, B, H, dp, dv)
    D = 1 + dp + dp * dp
    S2 = S.clone().reshape(B, H, D, dv)
    pert = torch.linspace(0.5, 2.0, dv, device=S2.device)
    for a in range(dp):
        for b in range(a + 1, dp):
            S2[:, :, 1 + dp + a * dp + b] += pert
            S2[:, :, 1 + dp + b * dp + a] -= pert
    state2 = based.alloc_state(B, H, dp, dv)
    based.state_import(state2, S2.reshape(S.shape), z, dp)
    y2 = run_prefill(based, wl, B, H, N - N1, q[:, N1:], k[:, N1:], v[:, N1:], state=state2, has_init=True)
    check_close(rows(y2), rows(want[:, N1:]), TOL[dtype], "y after an antisymmetric perturbation of S0")
    Sf, zf = based.state_export(state2, B, H, dp, dv)
    Sf = down(Sf).reshape(B * H, D, dv)
    pair = Sf[:, 1 + dp:].reshape(B * H, dp, dp, dv)
    Sf_sym = Sf.copy()
    Sf_sym[:, 1 + dp:] = (0.5 * (pair + pair.transpose(0, 2, 1, 3))).reshape(B * H, dp * dp, dv)
    check_close(Sf_sym.reshape(Sw.shape), Sw, TOL[dtype], "symmetric part of the final S")
    check_close(down(zf).reshape(zw.shape), zw, TOL[dtype], "final z")


@pytest.mark.parametrize("dp", [16, 32])
@pytest.mark.parametrize("scale", [2.0, 4.0])
def test_prefill_large_magnitudes(based, dp, scale):
    """Inputs 4 and 8 times larger than the workloads' (q.k of the order of +-100, kernel values up to 1e4):
    the bf16 matrix-core kernels stay finite and inside the same tolerance."""
    wl = make_wl("prefill_360m", d_feat=dp, qk_scale=scale, v_scale=scale)
    B, H, N = 1, 2, 700
    q, k, v = lin_case(wl, B, H, N)
    y = run_prefill(based, wl, B, H, N, q, k, v)
    check_close(rows(y), rows(oracle.linattn_quadratic(q, k, v)), TOL["bf16"], f"prefill at input scale {scale}, d'={dp}")


def test_prefill_deterministic(based):
    wl = synth.WORKLOADS["prefill_360m"]
    B, H, N = 2, 4, 512
    q, k, v = lin_case(wl, B, H, N)
    a = run_prefill(based, wl, B, H, N, q, k, v)
    b = run_prefill(based, wl, B, H, N, q, k, v)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------------------------------------
# linear attention decode
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,dp,dv", [("f32", 16, 64), ("bf16", 16, 128), ("bf16", 16, 64), ("bf16", 32, 64),
                                         ("f32", 32, 128), ("f32", 8, 64), ("bf16", 8, 128), ("bf16", 24, 64),
                                         ("f32", 24, 128)])
def test_decode_steps(based, dtype, dp, dv):
    wl = make_wl("decode_1p3b", d_feat=dp, d_v=dv, dtype=dtype)
    B, H, N0, T = 2, 3, 40, 12
    U = B * H
    q, k, v = lin_case(wl, B, H, N0)
    dec = synth.decode_inputs(wl, T, units=U)
    # oracle: state after the prefill, then the recurrent view token by token
    S, z = oracle.linattn_state(k, v)
    state = based.alloc_state(B, H, dp, dv)
    based.state_import(state, up(S, "f32", (B, H, S.shape[1], dv)), up(z, "f32", (B, H, z.shape[1])), dp)
    Sd, zd = S.astype(np.float32).astype(np.float64), z.astype(np.float32).astype(np.float64)
    for t in range(T):
        qt, kt, vt = dec["q"][t], dec["k"][t], dec["v"][t]
        y = based.decode_step(up(qt, dtype, (B, H, dp)), up(kt, dtype, (B, H, dp)), up(vt, dtype, (B, H, dv)), state)
        yw, Sd, zd = oracle.linattn_recurrent(qt[:, None], kt[:, None], vt[:, None], Sd, zd)
        check_close(down(y).reshape(U, dv), yw[:, 0], TOL[dtype], f"decode step {t}")
    Sg, zg = based.state_export(state, B, H, dp, dv)
    check_close(down(Sg).reshape(Sd.shape), Sd, TOL["f32"], "decode final S")
    check_close(down(zg).reshape(zd.shape), zd, TOL["f32"], "decode final z")


def test_prefill_then_decode_equals_longer_prefill(based):
    """prefill(N) + one decode step == last row of the quadratic form over N + 1 tokens."""
    wl = synth.WORKLOADS["prefill_360m"]
    B, H, N = 1, 4, 129
    q, k, v = lin_case(wl, B, H, N + 1)
    state = based.alloc_state(B, H, wl.d_feat, wl.d_v)
    run_prefill(based, wl, B, H, N, q[:, :N], k[:, :N], v[:, :N], state=state)
    y = based.decode_step(up(q[:, N], "bf16", (B, H, 16)), up(k[:, N], "bf16", (B, H, 16)),
                          up(v[:, N], "bf16", (B, H, 64)), state)
    want = oracle.linattn_rows(q, k, v, np.array([N]))[:, 0]
    check_close(down(y).reshape(B * H, 64), want, TOL["bf16"], "prefill + decode")


# ------------------------------------------------------------------------------------------------
# numerator-only variants (the undivided output of Alg. 1 / Alg. 2)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,dp,dv,N,N1", [("f32", 16, 64, 300, 130), ("bf16", 16, 64, 300, 130),
                                               ("bf16", 16, 128, 1400, 1100), ("bf16", 32, 64, 1200, 100),
                                               ("f32", 8, 64, 200, 70), ("bf16", 24, 128, 200, 70),
                                               ("f32", 32, 128, 1300, 64)])
def test_prefill_numerator_only(based, dtype, dp, dv, N, N1):
    """based_prefill_numerator over a split sequence (the second part from the state of the first, both
    long and short enough to be cut into segments or not) against the oracle's undivided rows; the state
    it leaves is the same as based_prefill's."""
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv, dtype=dtype)
    B, H = 1, 3
    U = B * H
    q, k, v = lin_case(wl, B, H, N)
    want = oracle.linattn_numerator(q, k, v)

    def part(a, lo, hi, d):
        return up(a[:, lo:hi], dtype, (B, H, hi - lo, d))

    state = based.alloc_state(B, H, dp, dv)
    y1 = based.prefill(part(q, 0, N1, dp), part(k, 0, N1, dp), part(v, 0, N1, dv), state=state, numerator_only=True)
    ref = based.alloc_state(B, H, dp, dv)
    based.prefill(part(q, 0, N1, dp), part(k, 0, N1, dp), part(v, 0, N1, dv), state=ref)
    torch.cuda.synchronize()
    assert torch.equal(state, ref)
    y2 = based.prefill(part(q, N1, N, dp), part(k, N1, N, dp), part(v, N1, N, dv), state=state, has_init=True,
                       numerator_only=True)
    torch.cuda.synchronize()
    check_close(rows(down(y1).reshape(U, N1, dv)), rows(want[:, :N1]), TOL[dtype], "numerator prefill part 1")
    check_close(rows(down(y2).reshape(U, N - N1, dv)), rows(want[:, N1:]), TOL[dtype], "numerator prefill part 2")
    Sg, zg = based.state_export(state, B, H, dp, dv)
    Sw, zw = oracle.linattn_state(k, v)
    check_close(down(Sg).reshape(Sw.shape), Sw, TOL[dtype], "numerator prefill final S")
    check_close(down(zg).reshape(zw.shape), zw, TOL[dtype], "numerator prefill final z")


@pytest.mark.parametrize("dtype,dp,dv", [("f32", 16, 64), ("bf16", 16, 128), ("bf16", 32, 64), ("f32", 8, 128)])
def test_decode_steps_numerator_only(based, dtype, dp, dv):
    """based_decode_step_numerator: y = phi(q) S after the update, token by token (Alg. 2 as printed)."""
    wl = make_wl("decode_1p3b", d_feat=dp, d_v=dv, dtype=dtype)
    B, H, N0, T = 2, 3, 40, 8
    U = B * H
    q, k, v = lin_case(wl, B, H, N0)
    dec = synth.decode_inputs(wl, T, units=U)
    S, z = oracle.linattn_state(k, v)
    state = based.alloc_state(B, H, dp, dv)
    based.state_import(state, up(S, "f32", (B, H, S.shape[1], dv)), up(z, "f32", (B, H, z.shape[1])), dp)
    Sd, zd = S.astype(np.float32).astype(np.float64), z.astype(np.float32).astype(np.float64)
    for t in range(T):
        qt, kt, vt = dec["q"][t], dec["k"][t], dec["v"][t]
        y = based.decode_step(up(qt, dtype, (B, H, dp)), up(kt, dtype, (B, H, dp)), up(vt, dtype, (B, H, dv)), state,
                              numerator_only=True)
        # one token on top of the state so far: the oracle's numerator with that state as S0
        yw = oracle.linattn_numerator(qt[:, None], kt[:, None], vt[:, None], Sd)[:, 0]
        Sd, zd = oracle.linattn_state(kt[:, None], vt[:, None], Sd, zd)
        check_close(down(y).reshape(U, dv), yw, TOL[dtype], f"numerator decode step {t}")
    Sg, zg = based.state_export(state, B, H, dp, dv)
    check_close(down(Sg).reshape(Sd.shape), Sd, TOL["f32"], "numerator decode final S")
    check_close(down(zg).reshape(zd.shape), zd, TOL["f32"], "numerator decode final z")


# ------------------------------------------------------------------------------------------------
# decay variant
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,dp,dv,N,N1,with_gate", [("f32", 16, 64, 300, 130, False), ("bf16", 16, 128, 300, 130, True),
                                                         ("f32", 16, 64, 1400, 1100, True), ("bf16", 32, 64, 700, 64, False),
                                                         ("f32", 8, 64, 1, 0, False)])
def test_prefill_and_decode_with_decay(based, dtype, dp, dv, N, N1, with_gate):
    """based_prefill_decay over a split sequence (second part from the state of the first; long enough to be
    cut into segments in one case), then based_decode_step_decay token by token, against the oracle's decayed
    recurrence; a per-head rate, heads cycling over the units."""
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv, dtype=dtype)
    B, H, T = 2, 3, 3
    U = B * H
    q, k, v = lin_case(wl, B, H, N + T)
    gam_h = np.array([0.999, 0.97, 0.9], dtype=np.float32)
    gamma_u = np.tile(gam_h.astype(np.float64), B)
    gate = synth.round_to(synth.normal(4242, (B, N + T, H), 1.0), dtype) if with_gate else None
    gate_u = None if gate is None else np.ascontiguousarray(gate.transpose(0, 2, 1)).reshape(U, N + T).astype(np.float64)
    want, Sw, zw = oracle.linattn_decay(q, k, v, gamma_u, gate=gate_u)
    tg = up(gam_h, "f32")

    def part(a, lo, hi, d):
        return up(a[:, lo:hi], dtype, (B, H, hi - lo, d))

    def gpart(lo, hi):
        return None if gate is None else up(gate[:, lo:hi], dtype)

    state = based.alloc_state(B, H, dp, dv)
    has = False
    if N1 > 0:
        y1 = based.prefill_decay(part(q, 0, N1, dp), part(k, 0, N1, dp), part(v, 0, N1, dv), tg, state=state, gate=gpart(0, N1))
        check_close(rows(down(y1).reshape(U, N1, dv)), rows(want[:, :N1]), TOL[dtype], "decay prefill part 1")
        has = True
    y2 = based.prefill_decay(part(q, N1, N, dp), part(k, N1, N, dp), part(v, N1, N, dv), tg, state=state, has_init=has,
                             gate=gpart(N1, N))
    torch.cuda.synchronize()
    check_close(rows(down(y2).reshape(U, N - N1, dv)), rows(want[:, N1:N]), TOL[dtype], "decay prefill part 2")
    for t in range(N, N + T):
        gt = None if gate is None else up(gate[:, t], dtype)
        y = based.decode_step_decay(up(q[:, t], dtype, (B, H, dp)), up(k[:, t], dtype, (B, H, dp)),
                                    up(v[:, t], dtype, (B, H, dv)), state, tg, gate=gt)
        check_close(down(y).reshape(U, dv), want[:, t], TOL[dtype], f"decay decode token {t}")
    Sg, zg = based.state_export(state, B, H, dp, dv)
    check_close(down(Sg).reshape(Sw.shape), Sw, TOL[dtype], "decay final S")
    check_close(down(zg).reshape(zw.shape), zw, TOL[dtype], "decay final z")


def test_decay_of_one_is_the_plain_method(based):
    """gamma = 1 and no gate: bit-identical to based_prefill on the fp32 path, and to based_decode_step."""
    wl = make_wl("tiny")
    B, H, N = 1, 2, 150
    q, k, v = lin_case(wl, B, H, N + 1)
    tq, tk, tv = (up(a[:, :N], "f32", (B, H, N, d)) for a, d in ((q, 16), (k, 16), (v, 64)))
    ones = torch.ones((H,), dtype=torch.float32, device="cuda")
    s1, s2 = based.alloc_state(B, H, 16, 64), based.alloc_state(B, H, 16, 64)
    y1 = based.prefill(tq, tk, tv, state=s1)
    y2 = based.prefill_decay(tq, tk, tv, ones, state=s2)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(s1, s2)
    a = [up(x[:, N], "f32", (B, H, d)) for x, d in ((q, 16), (k, 16), (v, 64))]
    assert torch.equal(based.decode_step(a[0], a[1], a[2], s1), based.decode_step_decay(a[0], a[1], a[2], s2, ones))
    assert torch.equal(s1, s2)


# ------------------------------------------------------------------------------------------------
# sliding-window attention
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dh,w,B,H,N", [(64, 64, 2, 2, 300), (128, 64, 1, 2, 150), (64, 128, 1, 2, 333),
                                        (128, 128, 1, 1, 260), (64, 64, 1, 1, 1), (64, 64, 1, 2, 17),
                                        (128, 64, 1, 1, 64), (64, 64, 1, 1, 65),
                                        # the small windows (the paper's 1.4B model uses 16)
                                        (64, 16, 2, 2, 300), (128, 16, 1, 2, 150), (64, 32, 1, 2, 333),
                                        (128, 32, 1, 1, 260), (64, 16, 1, 1, 1), (128, 16, 1, 2, 15),
                                        (64, 16, 1, 1, 16), (64, 16, 1, 2, 17), (64, 32, 1, 1, 33),
                                        # d_h 128 with window 64 or 32 (bf16: 16 queries to a wave, steps of 64):
                                        # one token, less than a tile, a step and one more, several
                                        # segments with a ragged last step
                                        (128, 64, 1, 1, 1), (128, 64, 1, 2, 17), (128, 64, 3, 1, 129),
                                        (128, 64, 1, 1, 65), (128, 64, 2, 3, 1000),
                                        (128, 32, 1, 2, 17), (128, 32, 1, 1, 65), (128, 32, 2, 3, 1000)])
def test_swa_prefill(based, dtype, dh, w, B, H, N):
    wl = make_wl("prefill_360m", d_h=dh, w=w, dtype=dtype)
    q, k, v = synth.swa_inputs(wl, units=B * H, N=N)
    scale = 1.0 / math.sqrt(dh)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    y = based.swa_prefill(up(q, dtype, (B, H, N, dh)), up(k, dtype, (B, H, N, dh)), up(v, dtype, (B, H, N, dh)),
                          w, scale, ring=ring)
    torch.cuda.synchronize()
    want = oracle.swa(q, k, v, w, scale)
    check_close(down(y).reshape(B * H * N, dh), rows(want), TOL[dtype], f"swa prefill {dtype} dh={dh} w={w} N={N}")
    # ring holds the last min(N, w) rows at slot j mod w, bit-exact copies
    r = down(ring).reshape(B * H, 2, w, dh)
    for j in range(max(0, N - w), N):
        assert np.array_equal(r[:, 0, j % w], k[:, j].astype(np.float64))
        assert np.array_equal(r[:, 1, j % w], v[:, j].astype(np.float64))


def test_swa_tiny_fp32_on_the_linear_attention_values(based):
    """The tiny fp32 case as the workload list states it: one unit, 256 tokens, window 64, 64-dim q and k
    of their own and the SAME v as the linear-attention leg; every element, and the ring it leaves."""
    wl = synth.WORKLOADS["tiny"]
    B, H, N, dh, w = wl.B, wl.H, wl.N, wl.d_h, wl.w
    q, k, v = synth.swa_inputs(wl)
    assert np.array_equal(v, synth.linattn_inputs(wl)[2]) and q.shape == (1, 256, 64)
    scale = 1.0 / math.sqrt(dh)
    ring = based.alloc_swa_ring(B, H, w, dh, torch.float32)
    y = based.swa_prefill(up(q, "f32", (B, H, N, dh)), up(k, "f32", (B, H, N, dh)), up(v, "f32", (B, H, N, dh)),
                          w, scale, ring=ring)
    torch.cuda.synchronize()
    check_close(down(y).reshape(N, dh), rows(oracle.swa(q, k, v, w, scale)), TOL["f32"], "tiny window attention")
    r = down(ring).reshape(1, 2, w, dh)
    for j in range(N - w, N):
        assert np.array_equal(r[:, 0, j % w], k[:, j].astype(np.float64))
        assert np.array_equal(r[:, 1, j % w], v[:, j].astype(np.float64))


@pytest.mark.parametrize("dtype,dh,w", [("f32", 64, 64), ("bf16", 128, 64), ("bf16", 64, 128), ("f32", 128, 128),
                                        ("bf16", 64, 64), ("bf16", 64, 16), ("bf16", 128, 16), ("f32", 64, 16),
                                        ("f32", 128, 16), ("bf16", 128, 32), ("f32", 64, 32)])
def test_swa_decode_from_empty_and_wrapping(based, dtype, dh, w):
    """Decode from an empty ring through the wrap-around: every step equals the prefill row."""
    wl = make_wl("decode_1p3b", d_h=dh, w=w, dtype=dtype)
    B, H = 1, 3
    U = B * H
    T = w + 9
    dec = synth.decode_inputs(wl, T, units=U)
    q, k, v = (np.ascontiguousarray(dec[n].transpose(1, 0, 2)) for n in ("swa_q", "swa_k", "swa_v"))
    scale = 1.0 / math.sqrt(dh)
    want = oracle.swa(q, k, v, w, scale)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    for t in range(T):
        y = based.swa_decode(up(q[:, t], dtype, (B, H, dh)), up(k[:, t], dtype, (B, H, dh)),
                             up(v[:, t], dtype, (B, H, dh)), ring, t + 1, w, scale)
        check_close(down(y).reshape(U, dh), want[:, t], TOL[dtype], f"swa decode pos {t + 1}")


@pytest.mark.parametrize("w", [64, 16, 32])
def test_swa_prefill_then_decode(based, w):
    wl = make_wl("decode_1p3b", w=w)
    dtype, dh = wl.dtype, wl.d_h
    B, H, N, T = 2, 2, 100, 5
    U = B * H
    q, k, v = synth.swa_inputs(wl, units=U, N=N + T)
    scale = 1.0 / math.sqrt(dh)
    want = oracle.swa(q, k, v, w, scale)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    based.swa_prefill(up(q[:, :N], dtype, (B, H, N, dh)), up(k[:, :N], dtype, (B, H, N, dh)),
                      up(v[:, :N], dtype, (B, H, N, dh)), w, scale, ring=ring)
    for t in range(N, N + T):
        y = based.swa_decode(up(q[:, t], dtype, (B, H, dh)), up(k[:, t], dtype, (B, H, dh)),
                             up(v[:, t], dtype, (B, H, dh)), ring, t + 1, w, scale)
        check_close(down(y).reshape(U, dh), want[:, t], TOL[dtype], f"swa prefill+decode pos {t + 1}")


# ------------------------------------------------------------------------------------------------
# fused decode launch
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,dp,dv,dh,w", [("bf16", 16, 128, 128, 64), ("f32", 16, 64, 64, 64),
                                              ("bf16", 32, 64, 64, 128), ("bf16", 16, 128, 128, 16),
                                              ("f32", 16, 64, 64, 32)])
def test_decode_fused_equals_separate_calls(based, dtype, dp, dv, dh, w):
    wl = make_wl("decode_1p3b", d_feat=dp, d_v=dv, d_h=dh, w=w, dtype=dtype)
    B, H, N0, T = 2, 2, 70, 6
    U = B * H
    q, k, v = lin_case(wl, B, H, N0)
    sq, sk, sv = synth.swa_inputs(wl, units=U, N=N0)
    dec = synth.decode_inputs(wl, T, units=U)
    scale = 1.0 / math.sqrt(dh)
    td = TORCH_DTYPE[dtype]

    def fresh():
        state = based.alloc_state(B, H, dp, dv)
        run_prefill(based, wl, B, H, N0, q, k, v, state=state)
        ring = based.alloc_swa_ring(B, H, w, dh, td)
        based.swa_prefill(up(sq, dtype, (B, H, N0, dh)), up(sk, dtype, (B, H, N0, dh)),
                          up(sv, dtype, (B, H, N0, dh)), w, scale, ring=ring)
        return state, ring

    state_a, ring_a = fresh()
    state_b, ring_b = fresh()
    # oracle for the window attention over the concatenated history
    allq = np.concatenate([sq, dec["swa_q"].transpose(1, 0, 2)], axis=1)
    allk = np.concatenate([sk, dec["swa_k"].transpose(1, 0, 2)], axis=1)
    allv = np.concatenate([sv, dec["swa_v"].transpose(1, 0, 2)], axis=1)
    want_swa = oracle.swa_rows(allq, allk, allv, w, scale, np.arange(N0, N0 + T))
    allq_l = np.concatenate([q, dec["q"].transpose(1, 0, 2)], axis=1)
    allk_l = np.concatenate([k, dec["k"].transpose(1, 0, 2)], axis=1)
    allv_l = np.concatenate([v, dec["v"].transpose(1, 0, 2)], axis=1)
    want_lin = oracle.linattn_rows(allq_l, allk_l, allv_l, np.arange(N0, N0 + T))
    for t in range(T):
        args = [up(dec[n][t], dtype, (B, H, -1)) for n in ("q", "k", "v", "swa_q", "swa_k", "swa_v")]
        y1 = based.decode_step(args[0], args[1], args[2], state_a)
        y2 = based.swa_decode(args[3], args[4], args[5], ring_a, N0 + t + 1, w, scale)
        f1, f2 = based.decode_fused(args[0], args[1], args[2], state_b, args[3], args[4], args[5], ring_b,
                                    N0 + t + 1, w, scale)
        torch.cuda.synchronize()
        assert torch.equal(y1, f1) and torch.equal(y2, f2)
        check_close(down(f1).reshape(U, dv), want_lin[:, t], TOL[dtype], f"fused lin step {t}")
        check_close(down(f2).reshape(U, dh), want_swa[:, t], TOL[dtype], f"fused swa step {t}")
    assert torch.equal(state_a, state_b) and torch.equal(ring_a, ring_b)


# ------------------------------------------------------------------------------------------------
# full-size workloads, in the launch configuration the benchmark times: sampled rows
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["prefill_360m", "prefill_1p3b"])
def test_full_size_prefill_sampled_rows(based, name):
    wl = synth.WORKLOADS[name]
    B, H, N, U = wl.B, wl.H, wl.N, wl.units
    q, k, v = synth.linattn_inputs(wl)
    y = run_prefill(based, wl, B, H, N, q, k, v)
    units = np.array([0, 1, U // 2, U - 1])
    # chunk boundaries, and every place where the launcher may cut the sequence into segments (multiples of
    # the chunk length between a quarter and three quarters of the sequence, rows on both sides)
    sample = np.array([0, 1, 63, 64, 65, 127, 128, 447, 448, 511, 512, 513, 575, 576, 577, 639, 640, 1023, 1024, 1025,
                       1087, 1088, 1089, 1151, 1152, 1535, 1536, 1537, 1599, 1600, 1601, 1663, 1664, N - 2, N - 1])
    want = oracle.linattn_rows(q[units], k[units], v[units], sample)
    check_close(rows(y[units][:, sample]), rows(want), TOL[wl.dtype], f"{name} sampled rows")
    sq, sk, sv = synth.swa_inputs(wl)
    scale = 1.0 / math.sqrt(wl.d_h)
    ys = based.swa_prefill(up(sq, wl.dtype, (B, H, N, wl.d_h)), up(sk, wl.dtype, (B, H, N, wl.d_h)),
                           up(sv, wl.dtype, (B, H, N, wl.d_h)), wl.w, scale)
    torch.cuda.synchronize()
    ys = down(ys).reshape(U, N, wl.d_h)
    want = oracle.swa_rows(sq[units], sk[units], sv[units], wl.w, scale, sample)
    check_close(rows(ys[units][:, sample]), rows(want), TOL[wl.dtype], f"{name} swa sampled rows")
    # property that holds at any size: outputs are convex combinations of the values seen so far
    hi = np.maximum.accumulate(v[units].astype(np.float64), axis=1)
    lo = np.minimum.accumulate(v[units].astype(np.float64), axis=1)
    slack = TOL[wl.dtype] * np.abs(v).max()
    assert (y[units] <= hi + slack).all() and (y[units] >= lo - slack).all()


def test_full_size_window16_sampled_rows(based):
    """The 1.3B-layer-shaped window attention at the window the paper's 1.4B model uses (16; training
    table in the appendix), full size: sampled rows of sampled units, and the decode ring it leaves."""
    wl = make_wl("prefill_1p3b", w=16)
    B, H, N, U, dh, w = wl.B, wl.H, wl.N, wl.units, wl.d_h, wl.w
    sq, sk, sv = synth.swa_inputs(wl)
    scale = 1.0 / math.sqrt(dh)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[wl.dtype])
    ys = based.swa_prefill(up(sq, wl.dtype, (B, H, N, dh)), up(sk, wl.dtype, (B, H, N, dh)),
                           up(sv, wl.dtype, (B, H, N, dh)), w, scale, ring=ring)
    torch.cuda.synchronize()
    units = np.array([0, 1, U // 2, U - 1])
    sample = np.array([0, 1, 14, 15, 16, 17, 127, 128, 129, 1023, 1024, N - 2, N - 1])
    want = oracle.swa_rows(sq[units], sk[units], sv[units], w, scale, sample)
    check_close(rows(down(ys).reshape(U, N, dh)[units][:, sample]), rows(want), TOL[wl.dtype], "window-16 sampled rows")
    r = down(ring).reshape(U, 2, w, dh)
    for j in range(N - w, N):
        assert np.array_equal(r[units, 0, j % w], sk[units, j].astype(np.float64))
        assert np.array_equal(r[units, 1, j % w], sv[units, j].astype(np.float64))


def test_full_size_decode_sampled_units(based):
    """The batch-128 decode workload in the launch shape the benchmark times (2048 units): a short
    prefill builds state and ring, then fused decode steps; sampled units against the oracle."""
    wl = synth.WORKLOADS["decode_1p3b"]
    B, H, U = wl.B, wl.H, wl.units
    dp, dv, dh, w, dtype = wl.d_feat, wl.d_v, wl.d_h, wl.w, wl.dtype
    N0, T = 80, 3
    q, k, v = lin_case(wl, B, H, N0)
    sq, sk, sv = synth.swa_inputs(wl, units=U, N=N0)
    dec = synth.decode_inputs(wl, T)
    scale = 1.0 / math.sqrt(dh)
    state = based.alloc_state(B, H, dp, dv)
    run_prefill(based, wl, B, H, N0, q, k, v, state=state)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    based.swa_prefill(up(sq, dtype, (B, H, N0, dh)), up(sk, dtype, (B, H, N0, dh)), up(sv, dtype, (B, H, N0, dh)),
                      w, scale, ring=ring)
    units = np.array([0, 1, 777, U // 2, U - 2, U - 1])
    cat = lambda a, b: np.concatenate([a[units], b.transpose(1, 0, 2)[units]], axis=1)
    steps = np.arange(N0, N0 + T)
    want_lin = oracle.linattn_rows(cat(q, dec["q"]), cat(k, dec["k"]), cat(v, dec["v"]), steps)
    want_swa = oracle.swa_rows(cat(sq, dec["swa_q"]), cat(sk, dec["swa_k"]), cat(sv, dec["swa_v"]), w, scale, steps)
    for t in range(T):
        args = [up(dec[n][t], dtype, (B, H, -1)) for n in ("q", "k", "v", "swa_q", "swa_k", "swa_v")]
        f1, f2 = based.decode_fused(args[0], args[1], args[2], state, args[3], args[4], args[5], ring,
                                    N0 + t + 1, w, scale)
        torch.cuda.synchronize()
        check_close(down(f1).reshape(U, dv)[units], want_lin[:, t], TOL[dtype], f"full-size fused lin step {t}")
        check_close(down(f2).reshape(U, dh)[units], want_swa[:, t], TOL[dtype], f"full-size fused swa step {t}")
    # state after the steps, sampled units
    S, z = based.state_export(state, B, H, dp, dv)
    kk, vv = cat(k, dec["k"]), cat(v, dec["v"])
    Sw, zw = oracle.linattn_state(kk, vv)
    D = Sw.shape[1]
    check_close(down(S).reshape(U, D, dv)[units], Sw, TOL[dtype], "full-size decode final S")
    check_close(down(z).reshape(U, D)[units], zw, TOL[dtype], "full-size decode final z")


def test_decode_workload_as_stated(based):
    """The batch-128 decode workload exactly as the workload list states it: state and ring from a seeded
    512-token prefill of all 2048 units, then 1024 sequential fused steps on 1024 distinct seeded tokens.
    Rows of Eq. 2 / Eq. 1 over the 1536-token history are independent, so sampled units at sampled steps
    are compared with the oracle directly; the final state of those units as well.  Three chains run side
    by side: (a) the state as based_prefill leaves it (bf16 matrix-core arithmetic: bf16 tolerance on the
    state); (b) the same, but the sampled units start from the oracle's 512-token state rounded to fp32,
    which isolates the 1024-step fp32 read-modify-write chain (fp32 tolerance on the final state);
    (c) chain (b) on the packed state."""
    from concurrent.futures import ThreadPoolExecutor
    wl = synth.WORKLOADS["decode_1p3b"]
    B, H, U = wl.B, wl.H, wl.units
    dp, dv, dh, w, dtype = wl.d_feat, wl.d_v, wl.d_h, wl.w, wl.dtype
    N0, T = wl.N, wl.decode_steps
    assert (B, H, N0, T, dp, dv, dh, w) == (128, 16, 512, 1024, 16, 128, 128, 64)
    D = 1 + dp + dp * dp
    scale = 1.0 / math.sqrt(dh)
    q, k, v = synth.linattn_inputs(wl)
    sq, sk, sv = synth.swa_inputs(wl)
    # synth.decode_inputs(wl, T), its six tensors drawn side by side (same seeds, same values)
    names = ("q", "k", "v", "swa_q", "swa_k", "swa_v")
    dims = (dp, dp, dv, dh, dh, dh)
    scales = (wl.qk_scale, wl.qk_scale, wl.v_scale, wl.swa_qk_scale, wl.swa_qk_scale, wl.v_scale)
    with ThreadPoolExecutor(6) as pool:
        futs = [pool.submit(synth.tensor, wl, synth.T_DECODE + i, (T, U, dims[i]), scales[i]) for i in range(6)]
        dec = {n: f.result() for n, f in zip(names, futs)}
    dev = {n: up(dec[n], dtype, (T, B, H, -1)) for n in names}

    state_a = based.alloc_state(B, H, dp, dv)
    run_prefill(based, wl, B, H, N0, q, k, v, state=state_a)
    ring_a = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    based.swa_prefill(up(sq, dtype, (B, H, N0, dh)), up(sk, dtype, (B, H, N0, dh)), up(sv, dtype, (B, H, N0, dh)),
                      w, scale, ring=ring_a)
    units = np.array([0, 1, 15, 16, 777, U // 2, U - 2, U - 1])
    # chain (b): sampled units start from the oracle's state of the 512 prefill tokens
    S0, z0 = oracle.linattn_state(k[units], v[units])
    S, z = based.state_export(state_a, B, H, dp, dv)
    S = S.reshape(U, D, dv).clone(); z = z.reshape(U, D).clone()
    S[torch.from_numpy(units).cuda()] = up(S0, "f32")
    z[torch.from_numpy(units).cuda()] = up(z0, "f32")
    state_b = based.alloc_state(B, H, dp, dv)
    based.state_import(state_b, S.reshape(B, H, D, dv), z.reshape(B, H, D), dp)
    packed_c = based.alloc_packed_state(B, H, dp, dv)
    based.state_pack(state_b, packed_c, B, H, dp, dv)
    ring_b, ring_c = ring_a.clone(), ring_a.clone()
    torch.cuda.synchronize()

    steps = np.array([1, 2, 64, 65, 512, 1023, 1024])   # 1-based step numbers
    keep = {int(t) - 1 for t in steps}
    got = {c: {} for c in "abc"}
    for t in range(T):
        a = [dev[n][t] for n in names]
        for c, st, rg, pk in (("a", state_a, ring_a, False), ("b", state_b, ring_b, False), ("c", packed_c, ring_c, True)):
            f1, f2 = based.decode_fused(a[0], a[1], a[2], st, a[3], a[4], a[5], rg, N0 + t + 1, w, scale, packed=pk)
            if t in keep:
                got[c][t] = (down(f1).reshape(U, dv)[units], down(f2).reshape(U, dh)[units])
    torch.cuda.synchronize()

    cat = lambda x, y: np.concatenate([x[units], y.transpose(1, 0, 2)[units]], axis=1)
    hist_rows = N0 + steps - 1
    allk, allv = cat(k, dec["k"]), cat(v, dec["v"])
    want_lin = oracle.linattn_rows(cat(q, dec["q"]), allk, allv, hist_rows)
    want_swa = oracle.swa_rows(cat(sq, dec["swa_q"]), cat(sk, dec["swa_k"]), cat(sv, dec["swa_v"]), w, scale, hist_rows)
    for c in "abc":
        for i, step in enumerate(steps):
            yl, ys = got[c][int(step) - 1]
            check_close(yl, want_lin[:, i], TOL[dtype], f"decode workload, chain {c}, step {step}: linear attention")
            check_close(ys, want_swa[:, i], TOL[dtype], f"decode workload, chain {c}, step {step}: window attention")
    Sw, zw = oracle.linattn_state(allk, allv)
    back = based.alloc_state(B, H, dp, dv)
    based.state_unpack(packed_c, back, B, H, dp, dv)
    for c, st, tol in (("a", state_a, TOL[dtype]), ("b", state_b, TOL["f32"]), ("c", back, TOL["f32"])):
        Sg, zg = based.state_export(st, B, H, dp, dv)
        check_close(down(Sg).reshape(U, D, dv)[units], Sw, tol, f"decode workload, chain {c}: S after 1024 steps")
        check_close(down(zg).reshape(U, D)[units], zw, tol, f"decode workload, chain {c}: z after 1024 steps")
    # the rings of the three chains saw the same tokens
    assert torch.equal(ring_a, ring_b) and torch.equal(ring_a, ring_c)
    r = down(ring_a).reshape(U, 2, w, dh)[units]
    for j in range(N0 + T - w, N0 + T):
        assert np.array_equal(r[:, 0, j % w], dec["swa_k"][j - N0, units].astype(np.float64))
        assert np.array_equal(r[:, 1, j % w], dec["swa_v"][j - N0, units].astype(np.float64))


def test_decode_state_beyond_the_cache(based):
    """A state well beyond the last-level cache (704 units x 545 KB = 384 MB at d' = 32, d_v = 128): the
    launches then walk the units in alternating directions and the fused launch streams the ring past the
    cache.  Four steps from an empty state (both directions at least once in each entry point), sampled
    units against the oracle, for the state update alone and for the fused step."""
    wl = make_wl("decode_1p3b", d_feat=32, d_v=128)
    B, H = 44, 16
    U = B * H
    dp, dv, dh, w, dtype = wl.d_feat, wl.d_v, wl.d_h, wl.w, wl.dtype
    T = 4
    dec = synth.decode_inputs(wl, T, units=U)
    scale = 1.0 / math.sqrt(dh)
    units = np.array([0, 1, 2, 351, 352, U - 2, U - 1])
    tr = lambda a: np.ascontiguousarray(a.transpose(1, 0, 2)[units])
    steps = np.arange(T)
    want_lin = oracle.linattn_rows(tr(dec["q"]), tr(dec["k"]), tr(dec["v"]), steps)
    want_swa = oracle.swa_rows(tr(dec["swa_q"]), tr(dec["swa_k"]), tr(dec["swa_v"]), w, scale, steps)
    state_a = based.alloc_state(B, H, dp, dv)
    state_b = based.alloc_state(B, H, dp, dv)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    toks = [[up(dec[n][t], dtype, (B, H, -1)) for n in ("q", "k", "v", "swa_q", "swa_k", "swa_v")] for t in range(T)]
    # consecutive launches of one entry point, so that each of them runs in both directions
    for t in range(T):
        y = based.decode_step(toks[t][0], toks[t][1], toks[t][2], state_a)
        torch.cuda.synchronize()
        check_close(down(y).reshape(U, dv)[units], want_lin[:, t], TOL[dtype], f"large-state update step {t}")
    for t in range(T):
        f1, f2 = based.decode_fused(*toks[t][:3], state_b, *toks[t][3:], ring, t + 1, w, scale)
        torch.cuda.synchronize()
        check_close(down(f1).reshape(U, dv)[units], want_lin[:, t], TOL[dtype], f"large-state fused lin step {t}")
        check_close(down(f2).reshape(U, dh)[units], want_swa[:, t], TOL[dtype], f"large-state fused swa step {t}")
    assert torch.equal(state_a, state_b)


@pytest.mark.parametrize("dh,w,N", [(64, 64, 1100), (128, 128, 1300), (64, 128, 2100), (128, 16, 1300),
                                    (64, 32, 1100),
                                    # 16 queries to a wave: many short segments, a last step of 20 and of 63 queries
                                    (128, 64, 1300), (128, 64, 2047), (128, 32, 1300)])
def test_swa_prefill_segmented(based, dh, w, N):
    """Sequences long enough to be cut into segments (ragged last step), every element checked."""
    wl = make_wl("prefill_360m", d_h=dh, w=w, dtype="bf16")
    B, H = 1, 2
    q, k, v = synth.swa_inputs(wl, units=B * H, N=N)
    scale = 1.0 / math.sqrt(dh)
    ring = based.alloc_swa_ring(B, H, w, dh, torch.bfloat16)
    y = based.swa_prefill(up(q, "bf16", (B, H, N, dh)), up(k, "bf16", (B, H, N, dh)), up(v, "bf16", (B, H, N, dh)),
                          w, scale, ring=ring)
    torch.cuda.synchronize()
    want = oracle.swa(q, k, v, w, scale)
    check_close(down(y).reshape(B * H * N, dh), rows(want), TOL["bf16"], f"segmented swa dh={dh} w={w} N={N}")
    r = down(ring).reshape(B * H, 2, w, dh)
    for j in range(N - w, N):
        assert np.array_equal(r[:, 0, j % w], k[:, j].astype(np.float64))
        assert np.array_equal(r[:, 1, j % w], v[:, j].astype(np.float64))


@pytest.mark.parametrize("scale", [-0.11, 0.0])
def test_swa_prefill_non_positive_scale(based, scale):
    """A non-positive softmax scale is legal (Eq. 1 with any temperature) and takes the vector-ALU kernel."""
    wl = make_wl("prefill_360m", d_h=64, w=64, dtype="bf16")
    B, H, N = 1, 2, 200
    q, k, v = synth.swa_inputs(wl, units=B * H, N=N)
    y = based.swa_prefill(up(q, "bf16", (B, H, N, 64)), up(k, "bf16", (B, H, N, 64)), up(v, "bf16", (B, H, N, 64)),
                          64, scale)
    torch.cuda.synchronize()
    want = oracle.swa(q, k, v, 64, scale)
    check_close(down(y).reshape(B * H * N, 64), rows(want), TOL["bf16"], f"swa scale {scale}")


def test_long_sequence_sampled_rows(based):
    """Few units, long sequences (8 segments in the linear-attention prefill, window 128): sampled rows."""
    wl = make_wl("prefill_long", d_feat=16, d_v=64, dtype="bf16")
    B, H, N = 1, 4, 16384
    U = B * H
    q, k, v = lin_case(wl, B, H, N)
    state = based.alloc_state(B, H, 16, 64)
    y = run_prefill(based, wl, B, H, N, q, k, v, state=state)
    sample = np.array([0, 63, 64, 2047, 2048, 2112, 4095, 4096, 8191, 8192, 12287, 12288, N - 65, N - 1])
    want = oracle.linattn_rows(q, k, v, sample)
    check_close(rows(y[:, sample]), rows(want), TOL["bf16"], "long sequence sampled rows")
    S, z = based.state_export(state, B, H, 16, 64)
    Sw, zw = oracle.linattn_state(k, v)
    check_close(down(S).reshape(Sw.shape), Sw, TOL["bf16"], "long sequence final S")
    check_close(down(z).reshape(zw.shape), zw, TOL["bf16"], "long sequence final z")
    sq, sk, sv = synth.swa_inputs(wl, units=U, N=N)
    scale = 1.0 / math.sqrt(wl.d_h)
    ys = based.swa_prefill(up(sq, "bf16", (B, H, N, wl.d_h)), up(sk, "bf16", (B, H, N, wl.d_h)),
                           up(sv, "bf16", (B, H, N, wl.d_h)), wl.w, scale)
    torch.cuda.synchronize()
    want = oracle.swa_rows(sq, sk, sv, wl.w, scale, sample)
    check_close(rows(down(ys).reshape(U, N, wl.d_h)[:, sample]), rows(want), TOL["bf16"], "long sequence swa rows")


def test_prefill_graph_replay(based):
    """A captured segmented prefill (increments and main pass in one launch, ready flags in the
    workspace) gives the eager result on every replay, with eager work and synchronisation between."""
    wl = synth.WORKLOADS["prefill_360m"]
    B, H, N = 1, 2, 1600
    q, k, v = lin_case(wl, B, H, N)
    tq, tk, tv = (up(a, "bf16", (B, H, N, a.shape[-1])) for a in (q, k, v))
    ws = based.alloc_prefill_workspace(B, H, N, wl.d_feat, wl.d_v, based.BF16)
    y_eager = based.prefill(tq, tk, tv, workspace=ws)
    torch.cuda.synchronize()
    want = oracle.linattn_quadratic(q, k, v)
    check_close(rows(down(y_eager).reshape(B * H, N, wl.d_v)), rows(want), TOL["bf16"], "eager segmented prefill")
    y_graph = torch.empty_like(y_eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        based.prefill(tq, tk, tv, y=y_graph, workspace=ws)   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        based.prefill(tq, tk, tv, y=y_graph, workspace=ws)
    for rep in range(3):
        y_graph.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {rep} differs from the eager result"
        # eager work on the same workspace between replays
        y2 = based.prefill(tq, tk, tv, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(y2, y_eager)


def test_prefill_bounded_wait_reports_failure(based):
    """The single-launch segmented prefill: a workgroup that gives up waiting for a segment's increment sets
    the sticky status word and based_prefill_status reports the call as failed.  The condition is forced
    from the host (poll limit 0: a waiting workgroup gives up at its first look), so every workgroup still
    exits normally.  After the query the same workspace serves a correct call again, replays included."""
    wl = synth.WORKLOADS["prefill_360m"]
    B, H, N = 1, 2, 2048   # four segments
    q, k, v = lin_case(wl, B, H, N)
    tq, tk, tv = (up(a, "bf16", (B, H, N, a.shape[-1])) for a in (q, k, v))
    ws = based.alloc_prefill_workspace(B, H, N, wl.d_feat, wl.d_v, based.BF16)
    sizes = (B, H, N, wl.d_feat, wl.d_v, based.BF16)
    want = oracle.linattn_quadratic(q, k, v)
    y_ok = based.prefill(tq, tk, tv, workspace=ws)
    assert based.prefill_status(ws, *sizes) == based.OK
    check_close(rows(down(y_ok).reshape(B * H, N, wl.d_v)), rows(want), TOL["bf16"], "before the forced failure")
    based.debug_set_poll_limit(0)
    try:
        based.prefill(tq, tk, tv, workspace=ws)
        assert based.prefill_status(ws, *sizes) == based.ERR_LAUNCH
        assert based.prefill_status(ws, *sizes) == based.OK   # reported once, then cleared
    finally:
        based.debug_set_poll_limit(-1)
    y2 = based.prefill(tq, tk, tv, workspace=ws)
    assert based.prefill_status(ws, *sizes) == based.OK
    assert torch.equal(y2, y_ok)
    # configurations without waiting workgroups always report OK
    assert based.prefill_status(ws, 1, 2, 100, 32, 64, based.BF16) == based.OK


@pytest.mark.parametrize("dp", [16, 32])
def test_whole_step_graph_replay(based, dp):
    """Linear-attention prefill (with final state), window prefill (with ring fill) and the fused decode
    step of the next token captured as one graph: every replay reproduces the eager results bit for bit.
    (d' = 32: three prefill launches handing data through the workspace.)"""
    wl = make_wl("prefill_360m", d_feat=dp)
    B, H, N = 1, 2, 1300
    dv, dh, w = wl.d_v, wl.d_h, wl.w
    scale = 1.0 / math.sqrt(dh)
    q, k, v = lin_case(wl, B, H, N)
    sq, sk, sv = synth.swa_inputs(wl, units=B * H, N=N)
    dec = synth.decode_inputs(wl, 1, units=B * H)
    tq, tk, tv = (up(a, "bf16", (B, H, N, a.shape[-1])) for a in (q, k, v))
    tsq, tsk, tsv = (up(a, "bf16", (B, H, N, dh)) for a in (sq, sk, sv))
    tok = [up(dec[n][0], "bf16", (B, H, -1)) for n in ("q", "k", "v", "swa_q", "swa_k", "swa_v")]
    ws = based.alloc_prefill_workspace(B, H, N, dp, dv, based.BF16)

    def step(bufs):
        y, sy, state, ring, yl, ys = bufs
        state.zero_()
        based.prefill(tq, tk, tv, y=y, state=state, workspace=ws)
        based.swa_prefill(tsq, tsk, tsv, w, scale, y=sy, ring=ring)
        based.decode_fused(*tok[:3], state, *tok[3:], ring, N + 1, w, scale, y_lin=yl, y_swa=ys)

    def bufs():
        return (torch.empty((B, H, N, dv), dtype=torch.bfloat16, device="cuda"),
                torch.empty((B, H, N, dh), dtype=torch.bfloat16, device="cuda"),
                based.alloc_state(B, H, dp, dv), based.alloc_swa_ring(B, H, w, dh, torch.bfloat16),
                torch.empty((B, H, dv), dtype=torch.bfloat16, device="cuda"),
                torch.empty((B, H, dh), dtype=torch.bfloat16, device="cuda"))

    eager = bufs()
    step(eager)
    torch.cuda.synchronize()
    check_close(rows(down(eager[0]).reshape(B * H, N, dv)), rows(oracle.linattn_quadratic(q, k, v)), TOL["bf16"],
                "eager prefill of the captured step")
    g = bufs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(g)
    for rep in range(3):
        for t in g:
            t.fill_(1) if t.dtype == torch.float32 else t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("y", "swa y", "state", "ring", "decode y_lin", "decode y_swa"), g, eager):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager result"
        step(bufs())   # eager work on the same workspace between replays
        torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------
# packed state (one row per unordered feature pair)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,dp,dv", [("f32", 16, 64), ("bf16", 16, 128), ("bf16", 32, 64), ("f32", 32, 128),
                                         ("bf16", 8, 64), ("f32", 24, 128)])
def test_decode_steps_packed_state(based, dtype, dp, dv):
    """Decode on the packed state gives the oracle's rows; unpacking it gives the oracle's state."""
    wl = make_wl("decode_1p3b", d_feat=dp, d_v=dv, dtype=dtype)
    B, H, N0, T = 2, 3, 40, 12
    U = B * H
    q, k, v = lin_case(wl, B, H, N0)
    dec = synth.decode_inputs(wl, T, units=U)
    S, z = oracle.linattn_state(k, v)
    state = based.alloc_state(B, H, dp, dv)
    based.state_import(state, up(S, "f32", (B, H, S.shape[1], dv)), up(z, "f32", (B, H, z.shape[1])), dp)
    packed = based.alloc_packed_state(B, H, dp, dv)
    based.state_pack(state, packed, B, H, dp, dv)
    # round trip through the packed layout is exact for a state of the recurrence
    back = based.alloc_state(B, H, dp, dv)
    based.state_unpack(packed, back, B, H, dp, dv)
    torch.cuda.synchronize()
    assert torch.equal(back, state)
    Sd, zd = S.astype(np.float32).astype(np.float64), z.astype(np.float32).astype(np.float64)
    for t in range(T):
        qt, kt, vt = dec["q"][t], dec["k"][t], dec["v"][t]
        y = based.decode_step(up(qt, dtype, (B, H, dp)), up(kt, dtype, (B, H, dp)), up(vt, dtype, (B, H, dv)),
                              packed, packed=True)
        yw, Sd, zd = oracle.linattn_recurrent(qt[:, None], kt[:, None], vt[:, None], Sd, zd)
        check_close(down(y).reshape(U, dv), yw[:, 0], TOL[dtype], f"packed decode step {t}")
    based.state_unpack(packed, back, B, H, dp, dv)
    Sg, zg = based.state_export(back, B, H, dp, dv)
    check_close(down(Sg).reshape(Sd.shape), Sd, TOL["f32"], "packed decode final S")
    check_close(down(zg).reshape(zd.shape), zd, TOL["f32"], "packed decode final z")


@pytest.mark.parametrize("dp,dv,N,N1", [(16, 64, 300, 130), (16, 128, 1400, 1100), (32, 64, 300, 130),
                                        (32, 128, 1700, 600)])
def test_prefill_packed_state(based, dp, dv, N, N1):
    """based_prefill_packed: the same y as the oracle over a split sequence (second part starting from
    the packed state of the first), the packed state equals pack(state of based_prefill) bit for bit,
    and packed decode continues from it."""
    dtype = "bf16"
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv, dtype=dtype)
    B, H, T = 1, 3, 3
    U = B * H
    q, k, v = lin_case(wl, B, H, N + T)
    want = oracle.linattn_quadratic(q, k, v)

    def part(a, lo, hi, d):
        return up(a[:, lo:hi], dtype, (B, H, hi - lo, d))

    packed = based.alloc_packed_state(B, H, dp, dv)
    y1 = based.prefill(part(q, 0, N1, dp), part(k, 0, N1, dp), part(v, 0, N1, dv), state=packed, packed=True)
    # the unpacked call on the same tokens, then packed: identical buffers
    state = based.alloc_state(B, H, dp, dv)
    based.prefill(part(q, 0, N1, dp), part(k, 0, N1, dp), part(v, 0, N1, dv), state=state)
    ref = based.alloc_packed_state(B, H, dp, dv)
    based.state_pack(state, ref, B, H, dp, dv)
    torch.cuda.synchronize()
    assert torch.equal(packed, ref)
    y2 = based.prefill(part(q, N1, N, dp), part(k, N1, N, dp), part(v, N1, N, dv), state=packed, has_init=True,
                       packed=True)
    torch.cuda.synchronize()
    check_close(rows(down(y1).reshape(U, N1, dv)), rows(want[:, :N1]), TOL[dtype], "packed prefill part 1")
    check_close(rows(down(y2).reshape(U, N - N1, dv)), rows(want[:, N1:N]), TOL[dtype], "packed prefill part 2")
    for t in range(N, N + T):
        y = based.decode_step(up(q[:, t], dtype, (B, H, dp)), up(k[:, t], dtype, (B, H, dp)),
                              up(v[:, t], dtype, (B, H, dv)), packed, packed=True)
        check_close(down(y).reshape(U, dv), want[:, t], TOL[dtype], f"decode after packed prefill, token {t}")
    back = based.alloc_state(B, H, dp, dv)
    based.state_unpack(packed, back, B, H, dp, dv)
    Sg, zg = based.state_export(back, B, H, dp, dv)
    Sw, zw = oracle.linattn_state(k, v)
    check_close(down(Sg).reshape(Sw.shape), Sw, TOL[dtype], "state after packed prefill + decode")
    check_close(down(zg).reshape(zw.shape), zw, TOL[dtype], "K-state after packed prefill + decode")


def test_decode_fused_packed_equals_separate(based):
    wl = make_wl("decode_1p3b", dtype="bf16")
    B, H, N0, T = 2, 2, 70, 4
    dp, dv, dh, w = wl.d_feat, wl.d_v, wl.d_h, wl.w
    U = B * H
    q, k, v = lin_case(wl, B, H, N0)
    sq, sk, sv = synth.swa_inputs(wl, units=U, N=N0)
    dec = synth.decode_inputs(wl, T, units=U)
    scale = 1.0 / math.sqrt(dh)

    def fresh():
        state = based.alloc_state(B, H, dp, dv)
        run_prefill(based, wl, B, H, N0, q, k, v, state=state)
        packed = based.alloc_packed_state(B, H, dp, dv)
        based.state_pack(state, packed, B, H, dp, dv)
        ring = based.alloc_swa_ring(B, H, w, dh, torch.bfloat16)
        based.swa_prefill(up(sq, "bf16", (B, H, N0, dh)), up(sk, "bf16", (B, H, N0, dh)),
                          up(sv, "bf16", (B, H, N0, dh)), w, scale, ring=ring)
        return packed, ring

    pa, ra = fresh()
    pb, rb = fresh()
    cat = lambda a, b: np.concatenate([a, b.transpose(1, 0, 2)], axis=1)
    want_lin = oracle.linattn_rows(cat(q, dec["q"]), cat(k, dec["k"]), cat(v, dec["v"]), np.arange(N0, N0 + T))
    for t in range(T):
        args = [up(dec[n][t], "bf16", (B, H, -1)) for n in ("q", "k", "v", "swa_q", "swa_k", "swa_v")]
        y1 = based.decode_step(args[0], args[1], args[2], pa, packed=True)
        y2 = based.swa_decode(args[3], args[4], args[5], ra, N0 + t + 1, w, scale)
        f1, f2 = based.decode_fused(args[0], args[1], args[2], pb, args[3], args[4], args[5], rb,
                                    N0 + t + 1, w, scale, packed=True)
        torch.cuda.synchronize()
        assert torch.equal(y1, f1) and torch.equal(y2, f2)
        check_close(down(f1).reshape(U, dv), want_lin[:, t], TOL["bf16"], f"fused packed lin step {t}")
    assert torch.equal(pa, pb) and torch.equal(ra, rb)


# ------------------------------------------------------------------------------------------------
# ragged batches: per-sequence positions in device memory
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("packed", [False, True])
def test_decode_fused_ragged_positions(based, packed):
    """Sequences that start at different steps: every sequence, on its own token stream, matches the
    oracle; a sequence whose position is < 1 is left untouched and gets zero rows."""
    # 70 > w: the ring wraps for the early starters
    _ragged_decode_case(based, "bf16", 16, 128, 128, 64, packed, B=4, H=2, T=70, start=np.array([0, 3, 40, 69]))


def _ragged_decode_case(based, dtype, dp, dv, dh, w, packed, B, H, T, start):
    wl = make_wl("decode_1p3b", dtype=dtype, d_feat=dp, d_v=dv, d_h=dh, w=w)
    U = B * H
    dec = synth.decode_inputs(wl, T, units=U)
    scale = 1.0 / math.sqrt(dh)
    state = (based.alloc_packed_state if packed else based.alloc_state)(B, H, dp, dv)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    ylin = np.zeros((T, U, dv)); yswa = np.zeros((T, U, dh))
    for t in range(T):
        pos = torch.tensor(np.maximum(t - start + 1, 0), dtype=torch.int32, device="cuda")
        args = [up(dec[n][t], dtype, (B, H, -1)) for n in ("q", "k", "v", "swa_q", "swa_k", "swa_v")]
        f1, f2 = based.decode_fused(args[0], args[1], args[2], state, args[3], args[4], args[5], ring,
                                    pos, w, scale, packed=packed)
        torch.cuda.synchronize()
        ylin[t] = down(f1).reshape(U, dv); yswa[t] = down(f2).reshape(U, dh)
    for b in range(B):
        units = np.arange(b * H, (b + 1) * H)
        s0 = int(start[b])
        assert not ylin[:s0, units].any() and not yswa[:s0, units].any()
        if s0 >= T:
            continue
        seq = lambda name: dec[name][s0:, units].transpose(1, 0, 2)
        want_lin = oracle.linattn_quadratic(seq("q"), seq("k"), seq("v"))
        want_swa = oracle.swa(seq("swa_q"), seq("swa_k"), seq("swa_v"), w, scale)
        check_close(rows(ylin[s0:, units].transpose(1, 0, 2)), rows(want_lin), TOL[dtype], f"ragged lin seq {b}")
        check_close(rows(yswa[s0:, units].transpose(1, 0, 2)), rows(want_swa), TOL[dtype], f"ragged swa seq {b}")


def _random_decode_cases():
    g = np.random.Generator(np.random.Philox(key=31))
    cases = []
    for _ in range(8):
        B = int(g.integers(1, 5)); T = int(g.integers(3, 40))
        cases.append((str(g.choice(["bf16", "f32"])), int(g.choice([16, 32])), int(g.choice([64, 128])),
                      int(g.choice([64, 128])), int(g.choice([16, 32, 64, 128])), bool(g.integers(0, 2)), B,
                      int(g.integers(1, 4)), T, tuple(int(x) for x in g.integers(0, T + 1, size=B))))
    return cases


@pytest.mark.parametrize("dtype,dp,dv,dh,w,packed,B,H,T,start", _random_decode_cases())
def test_decode_fused_random_cases(based, dtype, dp, dv, dh, w, packed, B, H, T, start):
    """Fused decode from empty state and ring at random sizes, dtypes, windows and state layouts, with
    sequences joining at random steps (a start of T: the sequence never takes part)."""
    _ragged_decode_case(based, dtype, dp, dv, dh, w, packed, B, H, T, np.array(start))


def test_decode_step_graph_replay_with_device_positions(based):
    """One captured fused decode step, replayed token after token while a device tensor holds the
    positions: every replay equals the eager step (eager work and synchronisation in between)."""
    wl = make_wl("decode_1p3b", dtype="bf16")
    B, H, T = 2, 2, 6
    dp, dv, dh, w = wl.d_feat, wl.d_v, wl.d_h, wl.w
    dec = synth.decode_inputs(wl, T, units=B * H)
    scale = 1.0 / math.sqrt(dh)
    names = ("q", "k", "v", "swa_q", "swa_k", "swa_v")
    toks = [[up(dec[n][t], "bf16", (B, H, -1)) for n in names] for t in range(T)]

    def eager():
        state = based.alloc_state(B, H, dp, dv)
        ring = based.alloc_swa_ring(B, H, w, dh, torch.bfloat16)
        outs = []
        for t in range(T):
            pos = torch.full((B,), t + 1, dtype=torch.int32, device="cuda")
            outs.append(based.decode_fused(*toks[t][:3], state, *toks[t][3:], ring, pos, w, scale))
        torch.cuda.synchronize()
        return outs, state, ring

    want, state_w, ring_w = eager()
    state = based.alloc_state(B, H, dp, dv)
    ring = based.alloc_swa_ring(B, H, w, dh, torch.bfloat16)
    inputs = [torch.empty_like(x) for x in toks[0]]
    y_lin = torch.empty((B, H, dv), dtype=torch.bfloat16, device="cuda")
    y_swa = torch.empty((B, H, dh), dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros((B,), dtype=torch.int32, device="cuda")   # every sequence inactive: warm-up touches nothing
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        based.decode_fused(*inputs[:3], state, *inputs[3:], ring, pos, w, scale, y_lin=y_lin, y_swa=y_swa)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        based.decode_fused(*inputs[:3], state, *inputs[3:], ring, pos, w, scale, y_lin=y_lin, y_swa=y_swa)
    for t in range(T):
        for dst, src in zip(inputs, toks[t]):
            dst.copy_(src)
        pos.add_(1)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_lin, want[t][0]) and torch.equal(y_swa, want[t][1]), f"replay {t}"
    assert torch.equal(state, state_w) and torch.equal(ring, ring_w)


def test_decode_loop_captured_whole(based):
    """A whole decode loop in one graph: [fused step on token slot t, positions_advance] for T tokens,
    captured once, replayed for two batches of T tokens; ragged start positions, one sequence sitting out.
    State, ring and every output equal the eager loop's."""
    wl = synth.WORKLOADS["prefill_360m"]
    B, H, dp, dv, dh, w, T = 4, 2, wl.d_feat, wl.d_v, wl.d_h, wl.w, 6
    dec = synth.decode_inputs(wl, 2 * T, units=B * H)
    scale = 1.0 / math.sqrt(dh)
    names = ("q", "k", "v", "swa_q", "swa_k", "swa_v")
    toks = [[up(dec[n][t], "bf16", (B, H, -1)) for n in names] for t in range(2 * T)]
    start = [1, 60, 0, 7]   # sequence 2 takes no part

    state_w = based.alloc_state(B, H, dp, dv)
    ring_w = based.alloc_swa_ring(B, H, w, dh, torch.bfloat16)
    pos_w = torch.tensor(start, dtype=torch.int32, device="cuda")
    want = []
    for t in range(2 * T):
        want.append(based.decode_fused(*toks[t][:3], state_w, *toks[t][3:], ring_w, pos_w, w, scale))
        based.positions_advance(pos_w)
    torch.cuda.synchronize()
    assert pos_w.tolist() == [1 + 2 * T, 60 + 2 * T, 0, 7 + 2 * T]

    state = based.alloc_state(B, H, dp, dv)
    ring = based.alloc_swa_ring(B, H, w, dh, torch.bfloat16)
    slots = [[torch.empty_like(x) for x in toks[0]] for _ in range(T)]
    y_lin = [torch.empty((B, H, dv), dtype=torch.bfloat16, device="cuda") for _ in range(T)]
    y_swa = [torch.empty((B, H, dh), dtype=torch.bfloat16, device="cuda") for _ in range(T)]
    pos = torch.zeros((B,), dtype=torch.int32, device="cuda")   # warm-up: nobody takes part

    def loop():
        for t in range(T):
            based.decode_fused(*slots[t][:3], state, *slots[t][3:], ring, pos, w, scale, y_lin=y_lin[t], y_swa=y_swa[t])
            based.positions_advance(pos)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        loop()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        loop()
    pos.copy_(torch.tensor(start, dtype=torch.int32, device="cuda"))
    for half in range(2):
        for t in range(T):
            for dst, src in zip(slots[t], toks[half * T + t]):
                dst.copy_(src)
        graph.replay()
        torch.cuda.synchronize()
        for t in range(T):
            assert torch.equal(y_lin[t], want[half * T + t][0]), f"y_lin replay {half} token {t}"
            assert torch.equal(y_swa[t], want[half * T + t][1]), f"y_swa replay {half} token {t}"
    assert torch.equal(state, state_w) and torch.equal(ring, ring_w) and torch.equal(pos, pos_w)


def test_full_size_long_config_sampled_rows(based):
    """The long-sequence / larger-state workload at full size (B2 H16 N16384, d' = 32: the segmented
    matrix-core path with the K-state kept as moments; window 128): sampled rows of sampled units against the oracle."""
    wl = synth.WORKLOADS["prefill_long"]
    B, H, N, U = wl.B, wl.H, wl.N, wl.units
    q, k, v = synth.linattn_inputs(wl)
    y = run_prefill(based, wl, B, H, N, q, k, v)
    units = np.array([0, 1, U // 2, U - 1])
    sample = np.array([0, 1, 255, 256, 511, 512, 513, 4095, 4096, 8192, 12345, N - 2, N - 1])
    want = oracle.linattn_rows(q[units], k[units], v[units], sample)
    check_close(rows(y[units][:, sample]), rows(want), TOL[wl.dtype], "prefill_long sampled rows")
    sq, sk, sv = synth.swa_inputs(wl)
    scale = 1.0 / math.sqrt(wl.d_h)
    ys = based.swa_prefill(up(sq, wl.dtype, (B, H, N, wl.d_h)), up(sk, wl.dtype, (B, H, N, wl.d_h)),
                           up(sv, wl.dtype, (B, H, N, wl.d_h)), wl.w, scale)
    torch.cuda.synchronize()
    want = oracle.swa_rows(sq[units], sk[units], sv[units], wl.w, scale, sample)
    check_close(rows(down(ys).reshape(U, N, wl.d_h)[units][:, sample]), rows(want), TOL[wl.dtype],
                "prefill_long swa sampled rows")


# ------------------------------------------------------------------------------------------------
# projections around the mixers
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N", [(300, 128, 128), (128, 64, 256), (1, 192, 128), (129, 1024, 384), (1000, 256, 1536)])
def test_linear_projection(based, M, K, N):
    """y = x W^T against the fp64 oracle: several tiles, ragged M (rows past the end of a tile), one row."""
    x, W = synth.linear_inputs(7, M, K, N)
    y = based.linear(up(x, "bf16"), up(W, "bf16"))
    torch.cuda.synchronize()
    check_close(down(y), oracle.linear(x, W), TOL["bf16"], f"linear {M}x{K}x{N}")


def test_linear_projection_full_size_sampled(based):
    """The fused q / k / v projection of the 360M-shaped layer (16384 tokens, d_model 1024 -> 16 heads x
    (16 + 16 + 64)) at full size: sampled rows against the oracle, every output feature."""
    M, K, N = 8 * 2048, 1024, 16 * (16 + 16 + 64)
    x, W = synth.linear_inputs(8, M, K, N)
    y = based.linear(up(x, "bf16"), up(W, "bf16"))
    torch.cuda.synchronize()
    sample = np.array([0, 1, 127, 128, 129, 4095, 8192, 12345, M - 2, M - 1])
    check_close(down(y)[sample], oracle.linear(x[sample], W), TOL["bf16"], "qkv projection, sampled rows")


# ------------------------------------------------------------------------------------------------
# seeded random shapes (segment boundaries, ragged chunks, splits at arbitrary tokens)
# ------------------------------------------------------------------------------------------------
# ------------------------------------------------------------------------------------------------
# projections in the mixers' layout
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,N,dm,H,dp,dv", [(2, 300, 256, 4, 16, 64), (1, 129, 128, 16, 16, 128), (3, 50, 192, 2, 32, 64),
                                            (1, 1, 64, 8, 8, 16)])
def test_project_qkv_and_out(based, B, N, dm, H, dp, dv):
    """based_project_qkv / based_project_out against the oracle's head-major projections (several tiles of
    tokens and features, ragged token tile, chunks of 8 features that end on head boundaries)."""
    Ntot = H * (2 * dp + dv)
    x, W = synth.linear_inputs(21, B * N, dm, Ntot)
    x = x.reshape(B, N, dm)
    q, k, v = based.project_qkv(up(x, "bf16"), up(W, "bf16"), H, dp, dv)
    torch.cuda.synchronize()
    Wq, Wk, Wv = W[:H * dp], W[H * dp:2 * H * dp], W[2 * H * dp:]
    for name, got, Wp in (("q", q, Wq), ("k", k, Wk), ("v", v, Wv)):
        want = oracle.project_heads(x, Wp, H)
        check_close(rows(down(got).reshape(B * H, N, -1)), rows(want.reshape(B * H, N, -1)), TOL["bf16"], f"project {name}")
    if dv % 64 == 0:
        dmo = 256
        yh, Wo = synth.linear_inputs(22, B * H * N, dv, 8)[0].reshape(B, H, N, dv), synth.linear_inputs(23, 8, H * dv, dmo)[1]
        out = based.project_out(up(yh, "bf16"), up(Wo, "bf16"))
        check_close(rows(down(out)), rows(oracle.project_out(yh, Wo)), TOL["bf16"], "project out")


@pytest.mark.parametrize("K", [64, 128, 192, 1024])
def test_linear_wide_tiles_sampled(based, K):
    """The 256 x 256 tiling of the projections (taken when N is a multiple of 256 and the tiles fill whole
    rounds of the chip well): a ragged last band of rows, one, two, three and many K steps (its loads run two
    steps ahead).  Sampled rows against the oracle, every output feature."""
    M, N = 127 * 256 + 232, 1024          # 128 x 4 = 512 tiles
    x, W = synth.linear_inputs(31, M, K, N)
    y = based.linear(up(x, "bf16"), up(W, "bf16"))
    torch.cuda.synchronize()
    sample = np.array([0, 1, 31, 32, 127, 128, 255, 256, 257, 12345, 127 * 256 - 1, 127 * 256, M - 2, M - 1])
    check_close(down(y)[sample], oracle.linear(x[sample], W), TOL["bf16"], f"wide tiles, K = {K}")


def test_project_qkv_and_out_wide_tiles_sampled(based):
    """based_project_qkv / based_project_out on the 256 x 256 tiling: the 1.3B-shaped head layout (16 heads,
    d' 16, d_v 128) over 17 sequences of 2000 tokens (sequence ends inside tiles, a ragged last band), a short
    d_model for the q / k / v projection.  Sampled (sequence, token) rows, every head and feature."""
    B, N, dm, H, dp, dv = 17, 2000, 128, 16, 16, 128
    Ntot = H * (2 * dp + dv)
    x, W = synth.linear_inputs(32, B * N, dm, Ntot)
    x = x.reshape(B, N, dm)
    q, k, v = based.project_qkv(up(x, "bf16"), up(W, "bf16"), H, dp, dv)
    torch.cuda.synchronize()
    bs = np.array([0, 0, 0, 1, 7, 16, 16])
    ts = np.array([0, 255, 1999, 0, 1234, 1998, 1999])
    xs = x[bs, ts][:, None, :]                      # [samples, 1, d_model]: one-token sequences for the oracle
    Wq, Wk, Wv = W[:H * dp], W[H * dp:2 * H * dp], W[2 * H * dp:]
    for name, got, Wp in (("q", q, Wq), ("k", k, Wk), ("v", v, Wv)):
        want = oracle.project_heads(xs, Wp, H)[:, :, 0, :]          # [samples, H, d]
        check_close(rows(down(got)[bs, :, ts, :]), rows(want), TOL["bf16"], f"wide project {name}")
    # the output projection reads the head-major mixer output: K = H d_v = 2048, N = 1792 (7 tiles wide)
    dmo = 1792
    yh = synth.linear_inputs(33, B * H * N, dv, 8)[0].reshape(B, H, N, dv)
    Wo = synth.linear_inputs(34, 8, H * dv, dmo)[1]
    out = based.project_out(up(yh, "bf16"), up(Wo, "bf16"))
    torch.cuda.synchronize()
    ys = np.stack([yh[b_, :, t_, :] for b_, t_ in zip(bs, ts)])[:, :, None, :]     # [samples, H, 1, d_v]
    want = oracle.project_out(ys, Wo)[:, 0, :]
    check_close(rows(down(out)[bs, ts]), rows(want), TOL["bf16"], "wide project out")


def test_linear_attention_layer_chain(based):
    """A linear-attention layer end to end in the library's own layouts (project q, k, v -> prefill -> project
    out, no transposing pass in between) against the same chain in the oracle, each stage fed the GPU's
    rounded output of the stage before so that the comparison stays stage by stage."""
    B, N, dm, H, dp, dv = 2, 200, 256, 4, 16, 64
    x, W = synth.linear_inputs(24, B * N, dm, H * (2 * dp + dv))
    W = W * 0.5
    W = synth.round_to(W, "bf16")
    x = x.reshape(B, N, dm)
    q, k, v = based.project_qkv(up(x, "bf16"), up(W, "bf16"), H, dp, dv)
    y = based.prefill(q, k, v)
    Wo = synth.linear_inputs(25, 8, H * dv, dm)[1]
    out = based.project_out(y, up(Wo, "bf16"))
    torch.cuda.synchronize()
    qd, kd, vd = (down(t).reshape(B * H, N, -1) for t in (q, k, v))
    check_close(rows(qd), rows(oracle.project_heads(x, W[:H * dp], H).reshape(B * H, N, dp)), TOL["bf16"], "chain q")
    yw = oracle.linattn_quadratic(qd, kd, vd)
    check_close(rows(down(y).reshape(B * H, N, dv)), rows(yw), TOL["bf16"], "chain mixer")
    check_close(rows(down(out)), rows(oracle.project_out(down(y), Wo)), TOL["bf16"], "chain out")


# ------------------------------------------------------------------------------------------------
# rotary encoding in the window-attention staging
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dh,pos0,N", [(64, 0, 300), (128, 1000, 77), (64, 16000, 400)])
def test_rotary_table(based, dh, pos0, N):
    """The table against cos / sin of the fp64 angles: correct to fp32 rounding."""
    t = down(based.rotary_table(N, dh, pos0=pos0))
    theta = 10000.0 ** (-2.0 * np.arange(dh // 2) / dh)
    ang = (pos0 + np.arange(N))[:, None] * theta[None, :]
    assert np.abs(t[..., 0] - np.cos(ang)).max() <= 2.0 ** -24 and np.abs(t[..., 1] - np.sin(ang)).max() <= 2.0 ** -24


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dh,w,B,H,N,pos0", [(64, 64, 2, 2, 300, 0), (128, 64, 1, 2, 150, 37), (64, 128, 1, 2, 333, 0),
                                             (128, 16, 1, 1, 1300, 5000), (64, 32, 1, 2, 1, 9), (128, 128, 1, 1, 1500, 0),
                                             (64, 64, 1, 1, 2100, 14000)])
def test_swa_prefill_rotary(based, dtype, dh, w, B, H, N, pos0):
    """based_swa_prefill_rotary against the oracle (rotation, then window attention), several steps and
    segments, a ragged tail, and a sequence that starts far from position 0; the ring holds rotated keys."""
    wl = make_wl("prefill_360m", d_h=dh, w=w, dtype=dtype)
    U = B * H
    q, k, v = synth.swa_inputs(wl, units=U, N=N)
    scale = 1.0 / math.sqrt(dh)
    want = oracle.swa_rotary(q, k, v, w, scale, pos0=pos0)
    table = based.rotary_table(N, dh, pos0=pos0)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    y = based.swa_prefill(up(q, dtype, (B, H, N, dh)), up(k, dtype, (B, H, N, dh)), up(v, dtype, (B, H, N, dh)),
                          w, scale, ring=ring, rotary=table)
    torch.cuda.synchronize()
    check_close(rows(down(y).reshape(U, N, dh)), rows(want), TOL[dtype], f"rotary window attention {dtype}")
    rk = oracle.rotary(k, pos0 + np.arange(N))
    r = down(ring).reshape(U, 2, w, dh)
    for j in range(max(0, N - w), N):
        check_close(r[:, 0, j % w], rk[:, j], TOL[dtype] / 4, f"ring key {j}")
        assert np.array_equal(r[:, 1, j % w], v[:, j].astype(np.float64))


def test_swa_prefill_rotary_non_positive_scale(based):
    """bf16 with a scale the matrix-core kernel does not take: the vector kernel rotates too."""
    wl = make_wl("prefill_360m", d_h=64, w=64)
    B, H, N = 1, 2, 200
    q, k, v = synth.swa_inputs(wl, units=B * H, N=N)
    table = based.rotary_table(N, 64)
    y = based.swa_prefill(up(q, "bf16", (B, H, N, 64)), up(k, "bf16", (B, H, N, 64)), up(v, "bf16", (B, H, N, 64)),
                          64, -0.11, rotary=table)
    check_close(rows(down(y).reshape(B * H, N, 64)), rows(oracle.swa_rotary(q, k, v, 64, -0.11)), TOL["bf16"],
                "rotary, negative scale")


@pytest.mark.parametrize("dtype,dh,w", [("bf16", 128, 64), ("f32", 64, 64), ("bf16", 64, 16), ("f32", 128, 128)])
@pytest.mark.parametrize("ragged", [False, True])
def test_swa_rotary_prefill_then_decode(based, dtype, dh, w, ragged):
    """Rotary prefill fills the ring with rotated keys; rotary decode steps continue from it, with one
    position for all sequences or one per sequence in device memory: every step is the oracle's row of the
    whole sequence."""
    wl = make_wl("decode_1p3b", d_h=dh, w=w, dtype=dtype)
    B, H, N, T = 2, 2, 100, 6
    U = B * H
    q, k, v = synth.swa_inputs(wl, units=U, N=N + T)
    scale = 1.0 / math.sqrt(dh)
    want = oracle.swa_rotary(q, k, v, w, scale)
    table = based.rotary_table(N + T, dh)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    based.swa_prefill(up(q[:, :N], dtype, (B, H, N, dh)), up(k[:, :N], dtype, (B, H, N, dh)),
                      up(v[:, :N], dtype, (B, H, N, dh)), w, scale, ring=ring, rotary=table[:N].contiguous())
    pos = torch.full((B,), N + 1, dtype=torch.int32, device="cuda")
    for t in range(N, N + T):
        y = based.swa_decode(up(q[:, t], dtype, (B, H, dh)), up(k[:, t], dtype, (B, H, dh)),
                             up(v[:, t], dtype, (B, H, dh)), ring, pos if ragged else t + 1, w, scale, rotary=table)
        check_close(down(y).reshape(U, dh), want[:, t], TOL[dtype], f"rotary decode token {t}")
        if ragged:
            based.positions_advance(pos)


@pytest.mark.parametrize("dtype,packed,ragged", [("bf16", False, False), ("f32", False, True), ("bf16", True, True)])
def test_decode_fused_rotary(based, dtype, packed, ragged):
    """The fused step with a rotary window half: bit-equal to the two separate calls (linear-attention step,
    rotary window step) on copies of the same state and ring, over several steps through the ring's wrap."""
    wl = make_wl("decode_1p3b", d_v=64, d_h=64, w=16, dtype=dtype)
    B, H, T, dp, dv, dh, w = 2, 3, 20, wl.d_feat, 64, 64, 16
    dec = synth.decode_inputs(wl, T, units=B * H)
    scale = 1.0 / math.sqrt(dh)
    table = based.rotary_table(T, dh)
    alloc = based.alloc_packed_state if packed else based.alloc_state
    st_a, st_b = alloc(B, H, dp, dv), alloc(B, H, dp, dv)
    ring_a = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    ring_b = torch.zeros_like(ring_a)
    pos = torch.ones((B,), dtype=torch.int32, device="cuda")
    for t in range(T):
        a = [up(dec[n][t], dtype, (B, H, d)) for n, d in (("q", dp), ("k", dp), ("v", dv), ("swa_q", dh), ("swa_k", dh), ("swa_v", dh))]
        p_arg = pos if ragged else t + 1
        yl, ys = based.decode_fused(a[0], a[1], a[2], st_a, a[3], a[4], a[5], ring_a, p_arg, w, scale, packed=packed,
                                    rotary=table)
        yl2 = based.decode_step(a[0], a[1], a[2], st_b, packed=packed)
        ys2 = based.swa_decode(a[3], a[4], a[5], ring_b, p_arg, w, scale, rotary=table)
        torch.cuda.synchronize()
        assert torch.equal(yl, yl2) and torch.equal(ys, ys2), t
        if ragged:
            based.positions_advance(pos)
    assert torch.equal(st_a, st_b) and torch.equal(ring_a, ring_b)


# ------------------------------------------------------------------------------------------------
# BaseConv gate
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,N,Dc", [(2, 100, 256), (1, 1, 8), (3, 33, 1032), (1, 2, 64), (2, 65, 4096)])
def test_short_conv_gate(based, dtype, B, N, Dc):
    """based_short_conv_gate against the oracle: whole sequences (several runs of tokens, ragged last run,
    channel counts that leave a workgroup partly idle), and the state rows it hands on."""
    a, c, h, b1, b2 = synth.baseconv_gate_inputs(7, B, N, Dc, dtype)
    want = oracle.short_conv_gate(a, c, h, b1, b2)
    th, tb1, tb2 = up(h, "f32"), up(b1, "f32"), up(b2, "f32")
    last = torch.full((B, 2, Dc), 7.0, dtype=TORCH_DTYPE[dtype], device="cuda")
    got = based.short_conv_gate(up(a, dtype), up(c, dtype), th, tb1, tb2, c_last=last)
    torch.cuda.synchronize()
    check_close(rows(down(got)), rows(want), TOL[dtype], f"conv gate {dtype} N={N} Dc={Dc}")
    ext = np.concatenate([np.zeros((B, 2, Dc)), c], axis=1)
    assert np.array_equal(down(last), ext[:, -2:])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_short_conv_gate_continuation_and_steps(based, dtype):
    """A sequence in two parts (the second from the state rows of the first), then token by token with the
    state updated in place: every row equals the oracle's row of the whole sequence."""
    B, N, Dc, N1, T = 2, 150, 512, 77, 5
    a, c, h, b1, b2 = synth.baseconv_gate_inputs(8, B, N + T, Dc, dtype)
    want = oracle.short_conv_gate(a, c, h, b1, b2)
    th, tb1, tb2 = up(h, "f32"), up(b1, "f32"), up(b2, "f32")
    state = torch.zeros((B, 2, Dc), dtype=TORCH_DTYPE[dtype], device="cuda")
    g1 = based.short_conv_gate(up(a[:, :N1], dtype), up(c[:, :N1], dtype), th, tb1, tb2, c_last=state)
    state2 = torch.empty_like(state)
    g2 = based.short_conv_gate(up(a[:, N1:N], dtype), up(c[:, N1:N], dtype), th, tb1, tb2, c_prev=state, c_last=state2)
    torch.cuda.synchronize()
    check_close(rows(down(g1)), rows(want[:, :N1]), TOL[dtype], "conv gate part 1")
    check_close(rows(down(g2)), rows(want[:, N1:N]), TOL[dtype], "conv gate part 2")
    for t in range(N, N + T):
        g = based.short_conv_gate(up(a[:, t:t + 1], dtype), up(c[:, t:t + 1], dtype), th, tb1, tb2,
                                  c_prev=state2, c_last=state2)
        check_close(rows(down(g)), rows(want[:, t:t + 1]), TOL[dtype], f"conv gate step {t}")
    assert np.array_equal(down(state2), c[:, N + T - 2:N + T].astype(np.float64))
    # in place is refused where the reader and the writer of the state are different threads
    with pytest.raises(based.BasedError):
        based.short_conv_gate(up(a[:, :40], dtype), up(c[:, :40], dtype), th, tb1, tb2, c_prev=state2, c_last=state2)


def _random_prefill_cases():
    g = np.random.Generator(np.random.Philox(key=2402))
    cases = []
    for _ in range(14):
        dp = int(g.choice([16, 32])); dv = int(g.choice([64, 128]))
        B = int(g.integers(1, 3)); H = int(g.integers(1, 4))
        N = int(g.integers(2, 4200)); N1 = int(g.integers(1, N))
        cases.append((dp, dv, B, H, N, N1))
    return cases


@pytest.mark.parametrize("dp,dv,B,H,N,N1", _random_prefill_cases())
def test_prefill_random_shapes(based, dp, dv, B, H, N, N1):
    """bf16 prefill of N tokens as one call and as two calls split at token N1 (state handed over), both
    against the oracle; final states agree with the oracle's."""
    wl = make_wl("prefill_360m", d_feat=dp, d_v=dv)
    q, k, v = lin_case(wl, B, H, N)
    want = oracle.linattn_quadratic(q, k, v)
    state = based.alloc_state(B, H, dp, dv)
    y = run_prefill(based, wl, B, H, N, q, k, v, state=state)
    check_close(rows(y), rows(want), TOL["bf16"], f"random shape one call d'={dp} dv={dv} U={B * H} N={N}")
    state2 = based.alloc_state(B, H, dp, dv)
    y1 = run_prefill(based, wl, B, H, N1, q[:, :N1], k[:, :N1], v[:, :N1], state=state2)
    y2 = run_prefill(based, wl, B, H, N - N1, q[:, N1:], k[:, N1:], v[:, N1:], state=state2, has_init=True)
    check_close(rows(y1), rows(want[:, :N1]), TOL["bf16"], f"random shape part 1 (N1={N1})")
    check_close(rows(y2), rows(want[:, N1:]), TOL["bf16"], f"random shape part 2 (N1={N1})")
    Sw, zw = oracle.linattn_state(k, v)
    for st, what in ((state, "one call"), (state2, "two calls")):
        S, z = based.state_export(st, B, H, dp, dv)
        check_close(down(S).reshape(Sw.shape), Sw, TOL["bf16"], f"random shape final S, {what}")
        check_close(down(z).reshape(zw.shape), zw, TOL["bf16"], f"random shape final z, {what}")


def _random_swa_cases():
    g = np.random.Generator(np.random.Philox(key=18668))
    cases = []
    for _ in range(12):
        cases.append((str(g.choice(["bf16", "bf16", "f32"])), int(g.choice([64, 128])), int(g.choice([16, 32, 64, 128])),
                      int(g.integers(1, 3)), int(g.integers(1, 4)), int(g.integers(1, 3000))))
    return cases


@pytest.mark.parametrize("dtype,dh,w,B,H,N", _random_swa_cases())
def test_swa_random_shapes(based, dtype, dh, w, B, H, N):
    """Window attention prefill at random sizes, then one decode step from the ring it leaves."""
    wl = make_wl("prefill_360m", d_h=dh, w=w, dtype=dtype)
    U = B * H
    q, k, v = synth.swa_inputs(wl, units=U, N=N + 1)
    scale = 1.0 / math.sqrt(dh)
    want = oracle.swa(q, k, v, w, scale)
    ring = based.alloc_swa_ring(B, H, w, dh, TORCH_DTYPE[dtype])
    y = based.swa_prefill(up(q[:, :N], dtype, (B, H, N, dh)), up(k[:, :N], dtype, (B, H, N, dh)),
                          up(v[:, :N], dtype, (B, H, N, dh)), w, scale, ring=ring)
    torch.cuda.synchronize()
    check_close(down(y).reshape(U * N, dh), rows(want[:, :N]), TOL[dtype], f"random swa {dtype} dh={dh} w={w} N={N}")
    yd = based.swa_decode(up(q[:, N], dtype, (B, H, dh)), up(k[:, N], dtype, (B, H, dh)), up(v[:, N], dtype, (B, H, dh)),
                          ring, N + 1, w, scale)
    check_close(down(yd).reshape(U, dh), want[:, N], TOL[dtype], f"random swa decode after N={N}")

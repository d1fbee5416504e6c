"""Pins for the CPU oracle: everything here checks ``oracle/`` against something other than itself
(closed forms, equivalent forms written independently in numpy, a pure-Python brute force,
textbook special cases, a library attention routine, and the dimension facts the paper prints).
CPU only."""
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------------------------
# pure-Python brute force (independent authoring path; tiny sizes only)
# --------------------------------------------------------------------------------------------
def brute_linattn(q, k, v):
    U, N, dp = len(q), len(q[0]), len(q[0][0])
    dv = len(v[0][0])
    out = [[[0.0] * dv for _ in range(N)] for _ in range(U)]
    for u in range(U):
        for i in range(N):
            den = 0.0
            num = [0.0] * dv
            for j in range(i + 1):
                x = 0.0
                for a in range(dp):
                    x += q[u][i][a] * k[u][j][a]
                w = 1.0 + x + x * x / 2.0
                den += w
                for c in range(dv):
                    num[c] += w * v[u][j][c]
            out[u][i] = [n / den for n in num]
    return out


def brute_swa(q, k, v, w, scale):
    U, N, dh = len(q), len(q[0]), len(q[0][0])
    out = [[[0.0] * dh for _ in range(N)] for _ in range(U)]
    for u in range(U):
        for i in range(N):
            js = [j for j in range(N) if j <= i and j > i - w]
            logits = [scale * sum(q[u][i][a] * k[u][j][a] for a in range(dh)) for j in js]
            m = max(logits)
            e = [math.exp(l - m) for l in logits]
            s = sum(e)
            for c in range(dh):
                out[u][i][c] = sum(e[t] * v[u][j][c] for t, j in enumerate(js)) / s
    return out


# --------------------------------------------------------------------------------------------
# dimension facts printed in the paper
# --------------------------------------------------------------------------------------------
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "state_sizes.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, a, b = line.split()
            rows.append((key, int(a), int(b)))
    return rows


def test_dimension_facts_from_the_paper():
    rows = _golden_rows()
    assert len(rows) >= 5
    for key, arg, expected in rows:
        if key == "D":
            assert oracle.feature_dim(arg) == expected
        elif key == "SYM":
            # per-column count: (d + 1) * (...) with d = 0
            assert oracle.state_size_symmetric(arg, 0) == expected
        else:
            raise AssertionError(f"unknown golden key {key}")
    # the full formula with its (d + 1) factor, d = 64, d' = 16
    assert oracle.state_size_symmetric(16, 64) == 65 * 153
    assert oracle.feature_dim(32) == 1057


# --------------------------------------------------------------------------------------------
# Eq. 4: phi(q).phi(k) = 1 + q.k + (q.k)^2 / 2, and the feature order
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dp", [1, 2, 4, 16, 32])
def test_feature_map_closed_form(dp):
    g = rng(dp)
    for scale in (1e-3, 1.0, 30.0):
        q = g.standard_normal((64, dp)) * scale
        k = g.standard_normal((64, dp)) * scale
        pq, pk = oracle.feature_map(q), oracle.feature_map(k)
        assert pq.shape == (64, 1 + dp + dp * dp)
        lhs = (pq * pk).sum(-1)
        x = (q * k).sum(-1)
        rhs = 1.0 + x + 0.5 * x * x
        assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12 * max(1.0, scale ** 4))


def test_feature_map_order_and_scaling():
    x = np.array([2.0, 3.0, 5.0])
    phi = oracle.feature_map(x)
    assert phi[0] == 1.0
    assert list(phi[1:4]) == [2.0, 3.0, 5.0]
    # row-major (a, b) block: index 1 + d' + a d' + b holds x_a x_b / sqrt(2)
    blk = phi[4:].reshape(3, 3)
    assert np.allclose(blk, np.outer(x, x) / math.sqrt(2.0), rtol=0, atol=1e-15)
    assert blk[0, 2] == blk[2, 0]
    # adversarial: orthogonal q, k => kernel is exactly 1
    q = np.array([1.0, 0.0, 0.0]); k = np.array([0.0, 7.0, 0.0])
    assert (oracle.feature_map(q) * oracle.feature_map(k)).sum() == 1.0


# --------------------------------------------------------------------------------------------
# brute force
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("U,N,dp,dv", [(1, 1, 1, 1), (2, 7, 3, 2), (1, 32, 4, 4), (3, 13, 2, 5)])
def test_linattn_vs_pure_python(U, N, dp, dv):
    g = rng(100 + N)
    q = g.standard_normal((U, N, dp)); k = g.standard_normal((U, N, dp)); v = g.standard_normal((U, N, dv))
    want = np.array(brute_linattn(q.tolist(), k.tolist(), v.tolist()))
    assert np.allclose(oracle.linattn_quadratic(q, k, v), want, rtol=1e-12, atol=1e-13)
    rows = np.array(sorted({0, N // 2, N - 1}))
    assert np.allclose(oracle.linattn_rows(q, k, v, rows), want[:, rows], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("U,N,dh,w", [(1, 1, 1, 1), (2, 9, 3, 4), (1, 20, 4, 64), (2, 17, 2, 1), (1, 12, 3, 12)])
def test_swa_vs_pure_python(U, N, dh, w):
    g = rng(200 + N)
    q = g.standard_normal((U, N, dh)); k = g.standard_normal((U, N, dh)); v = g.standard_normal((U, N, dh))
    want = np.array(brute_swa(q.tolist(), k.tolist(), v.tolist(), w, 0.7))
    assert np.allclose(oracle.swa(q, k, v, w, 0.7), want, rtol=1e-12, atol=1e-13)
    rows = np.array(sorted({0, N // 3, N - 1}))
    assert np.allclose(oracle.swa_rows(q, k, v, w, 0.7, rows), want[:, rows], rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------------------------
# equality of forms: parallel (Eq. 2) == recurrent (Eq. 3) == tile split (Sec. 4) == cumsum form
# --------------------------------------------------------------------------------------------
def np_phi(x):
    """numpy feature map written separately from the oracle (explicit outer product)."""
    dp = x.shape[-1]
    second = (x[..., :, None] * x[..., None, :]).reshape(x.shape[:-1] + (dp * dp,)) / np.sqrt(2.0)
    return np.concatenate([np.ones(x.shape[:-1] + (1,)), x, second], axis=-1)


def np_cumsum_form(q, k, v):
    """Materialised-feature cumsum form of the appendix listing (no epsilon)."""
    pq, pk = np_phi(q), np_phi(k)
    kv = np.cumsum(pk[..., :, None] * v[..., None, :], axis=1)      # [U, N, D, dv]
    num = np.einsum("unf,unfc->unc", pq, kv)
    den = np.einsum("unf,unf->un", pq, np.cumsum(pk, axis=1))
    return num / den[..., None]


def np_chunked(q, k, v, C):
    """Tile split of Sec. 4: on-diagonal quadratic block + off-diagonal readout of the running state."""
    U, N, dp = q.shape
    dv = v.shape[-1]
    D = 1 + dp + dp * dp
    S = np.zeros((U, D, dv)); z = np.zeros((U, D))
    y = np.empty((U, N, dv))
    for c0 in range(0, N, C):
        c1 = min(N, c0 + C)
        qc, kc, vc = q[:, c0:c1], k[:, c0:c1], v[:, c0:c1]
        A = np.einsum("uia,uja->uij", qc, kc)
        P = np.tril(np.ones((c1 - c0, c1 - c0)))[None] * (1.0 + A + 0.5 * A * A)
        pq, pk = np_phi(qc), np_phi(kc)
        num = np.einsum("uij,ujc->uic", P, vc) + np.einsum("uif,ufc->uic", pq, S)
        den = P.sum(-1) + np.einsum("uif,uf->ui", pq, z)
        y[:, c0:c1] = num / den[..., None]
        S += np.einsum("ujf,ujc->ufc", pk, vc)
        z += pk.sum(1)
    return y, S, z


@pytest.mark.parametrize("U,N,dp,dv", [(2, 50, 4, 6), (1, 100, 16, 8), (1, 37, 8, 3)])
def test_forms_agree(U, N, dp, dv):
    g = rng(300 + N)
    q = g.standard_normal((U, N, dp)) * 0.7; k = g.standard_normal((U, N, dp)) * 0.7
    v = g.standard_normal((U, N, dv))
    yq = oracle.linattn_quadratic(q, k, v)
    yr, Sr, zr = oracle.linattn_recurrent(q, k, v)
    assert np.allclose(yq, yr, rtol=1e-10, atol=1e-12)
    assert np.allclose(yq, np_cumsum_form(q, k, v), rtol=1e-10, atol=1e-12)
    for C in (1, 16, 7, N, N + 5):
        yc, Sc, zc = np_chunked(q, k, v, C)
        assert np.allclose(yq, yc, rtol=1e-10, atol=1e-12), C
        assert np.allclose(Sr, Sc, rtol=1e-10, atol=1e-12)
        assert np.allclose(zr, zc, rtol=1e-10, atol=1e-12)
    S, z = oracle.linattn_state(k, v)
    assert np.allclose(S, Sr, rtol=1e-12, atol=1e-12) and np.allclose(z, zr, rtol=1e-12, atol=1e-12)
    # state against the independent numpy feature map
    assert np.allclose(S, np.einsum("ujf,ujc->ufc", np_phi(k), v), rtol=1e-12, atol=1e-12)
    assert np.allclose(z, np_phi(k).sum(1), rtol=1e-12, atol=1e-12)


def test_recurrent_continuation_equals_one_pass():
    """Split prefill: running the recurrent view on a suffix from the prefix's state gives the
    quadratic view's rows for that suffix; a single decode step is the N = 1 case."""
    g = rng(7)
    U, N, dp, dv, N1 = 2, 60, 4, 5, 23
    q = g.standard_normal((U, N, dp)); k = g.standard_normal((U, N, dp)); v = g.standard_normal((U, N, dv))
    yq = oracle.linattn_quadratic(q, k, v)
    S1, z1 = oracle.linattn_state(k[:, :N1], v[:, :N1])
    y2, S2, z2 = oracle.linattn_recurrent(q[:, N1:], k[:, N1:], v[:, N1:], S1, z1)
    assert np.allclose(y2, yq[:, N1:], rtol=1e-10, atol=1e-12)
    Sf, zf = oracle.linattn_state(k, v)
    assert np.allclose(S2, Sf, rtol=1e-12, atol=1e-12) and np.allclose(z2, zf, rtol=1e-12, atol=1e-12)
    # adding to a given state
    S3, z3 = oracle.linattn_state(k[:, N1:], v[:, N1:], S1, z1)
    assert np.allclose(S3, Sf, rtol=1e-12, atol=1e-12) and np.allclose(z3, zf, rtol=1e-12, atol=1e-12)
    # one token at a time
    S, z = S1, z1
    for t in range(N1, N1 + 4):
        yt, S, z = oracle.linattn_recurrent(q[:, t:t + 1], k[:, t:t + 1], v[:, t:t + 1], S, z)
        assert np.allclose(yt[:, 0], yq[:, t], rtol=1e-10, atol=1e-12)


def test_numerator_only_pins():
    """The undivided output: against a pure-Python sum, against numerator = y * denominator with both
    factors from other routes, against the state route phi(q_i) S_i, and on closed forms."""
    g = rng(77)
    U, N, dp, dv = 2, 23, 3, 4
    q = g.standard_normal((U, N, dp)); k = g.standard_normal((U, N, dp)); v = g.standard_normal((U, N, dv))
    got = oracle.linattn_numerator(q, k, v)
    ql, kl, vl = q.tolist(), k.tolist(), v.tolist()
    den = np.zeros((U, N))
    for u in range(U):
        for i in range(N):
            num = [0.0] * dv
            for j in range(i + 1):
                x = sum(ql[u][i][a] * kl[u][j][a] for a in range(dp))
                wgt = 1.0 + x + x * x / 2.0
                den[u, i] += wgt
                for c in range(dv):
                    num[c] += wgt * vl[u][j][c]
            assert np.allclose(got[u, i], num, rtol=1e-12, atol=1e-13)
    # Eq. 2 is numerator / denominator: the C oracle's normalised rows times the denominators above
    assert np.allclose(got, oracle.linattn_quadratic(q, k, v) * den[:, :, None], rtol=1e-11, atol=1e-12)
    # Eq. 3: the same row from the running KV-state (the C oracle's state of the prefix, token included)
    for i in (0, 5, N - 1):
        S, _ = oracle.linattn_state(k[:, :i + 1], v[:, :i + 1])
        assert np.allclose(got[:, i], np.einsum("uf,ufc->uc", np_phi(q[:, i]), S), rtol=1e-11, atol=1e-12)
    # continuation from a state: rows N1.. of the whole sequence
    N1 = 9
    S1, _ = oracle.linattn_state(k[:, :N1], v[:, :N1])
    assert np.allclose(oracle.linattn_numerator(q[:, N1:], k[:, N1:], v[:, N1:], S1), got[:, N1:], rtol=1e-11, atol=1e-12)
    # q = 0: every weight is 1, the numerator is the running sum of v; first row is v_0 (1 + x + x^2/2 at j = i = 0)
    assert np.allclose(oracle.linattn_numerator(np.zeros_like(q), k, v), np.cumsum(v, axis=1), rtol=1e-13, atol=1e-13)
    x0 = np.einsum("ua,ua->u", q[:, 0], k[:, 0])
    assert np.allclose(got[:, 0], (1 + x0 + x0 * x0 / 2)[:, None] * v[:, 0], rtol=1e-13, atol=1e-13)


def test_decay_pins():
    """The decayed recurrence against the weighted quadratic form written with pure-Python loops, against the
    undecayed oracle at gamma = 1, an exponential moving average at q = 0, and continuation from a state."""
    g = rng(12)
    U, N, dp, dv = 2, 17, 3, 4
    q = g.standard_normal((U, N, dp)); k = g.standard_normal((U, N, dp)); v = g.standard_normal((U, N, dv))
    gamma = np.array([0.9, 0.5])
    y, S, z = oracle.linattn_decay(q, k, v, gamma)
    for u in range(U):
        for i in range(N):
            num = np.zeros(dv); den = 0.0
            for j in range(i + 1):
                x = float(q[u, i] @ k[u, j])
                wgt = gamma[u] ** (i - j) * (1.0 + x + x * x / 2.0)
                num += wgt * v[u, j]; den += wgt
            assert np.allclose(y[u, i], num / den, rtol=1e-11, atol=1e-12)
    # final state: decayed sums of phi(k) v^T and phi(k)
    wts = gamma[:, None] ** (N - 1 - np.arange(N))[None, :]
    assert np.allclose(S, np.einsum("uj,ujf,ujc->ufc", wts, np_phi(k), v), rtol=1e-11, atol=1e-12)
    assert np.allclose(z, np.einsum("uj,ujf->uf", wts, np_phi(k)), rtol=1e-11, atol=1e-12)
    # gamma = 1: the plain method (C oracle)
    y1, S1, z1 = oracle.linattn_decay(q, k, v, np.ones(U))
    yr, Sr, zr = oracle.linattn_recurrent(q, k, v)
    assert np.allclose(y1, yr, rtol=1e-11, atol=1e-12) and np.allclose(S1, Sr, rtol=1e-11) and np.allclose(z1, zr, rtol=1e-11)
    # q = 0: every weight is gamma^(i - j), an exponential moving average of v
    y0, _, _ = oracle.linattn_decay(np.zeros_like(q), k, v, gamma)
    for u in range(U):
        acc = np.zeros(dv); cnt = 0.0
        for i in range(N):
            acc = gamma[u] * acc + v[u, i]; cnt = gamma[u] * cnt + 1.0
            assert np.allclose(y0[u, i], acc / cnt, rtol=1e-12, atol=1e-13)
    # continuation from the state of a prefix, and the gate
    N1 = 6
    _, Sa, za = oracle.linattn_decay(q[:, :N1], k[:, :N1], v[:, :N1], gamma)
    gt = g.standard_normal((U, N - N1))
    yb, Sb, zb = oracle.linattn_decay(q[:, N1:], k[:, N1:], v[:, N1:], gamma, Sa, za, gate=gt)
    assert np.allclose(yb, y[:, N1:] * gt[:, :, None], rtol=1e-11, atol=1e-12)
    assert np.allclose(Sb, S, rtol=1e-12) and np.allclose(zb, z, rtol=1e-12)


@pytest.mark.parametrize("dp", [8, 24])
def test_ablation_feature_dimensions(dp):
    """d' = 8 and 24 (the feature-dimension rows of the ablation table): the sizes the table prints in
    parentheses (45 and 325, the count of distinct monomials of degree <= 2), D = 1 + d' + d'^2, and the
    three views agreeing at those sizes."""
    printed = {8: 45, 24: 325}
    assert oracle.state_size_symmetric(dp, 0) == printed[dp]
    assert oracle.feature_dim(dp) == 1 + dp + dp * dp
    # distinct rows of the expanded state: the (a, b) and (b, a) rows coincide, leaving the printed count
    x = rng(1000 + dp).standard_normal(dp)
    assert len(np.unique(np.round(oracle.feature_map(x), 12))) == printed[dp]
    g = rng(dp)
    U, N, dv = 2, 40, 5
    q = g.standard_normal((U, N, dp)) * 0.5; k = g.standard_normal((U, N, dp)) * 0.5
    v = g.standard_normal((U, N, dv))
    yq = oracle.linattn_quadratic(q, k, v)
    yr, Sr, zr = oracle.linattn_recurrent(q, k, v)
    assert np.allclose(yq, yr, rtol=1e-10, atol=1e-12)
    assert np.allclose(yq, np_cumsum_form(q, k, v), rtol=1e-10, atol=1e-12)
    assert np.allclose(Sr, np.einsum("ujf,ujc->ufc", np_phi(k), v), rtol=1e-12, atol=1e-12)
    assert np.allclose(zr, np_phi(k).sum(1), rtol=1e-12, atol=1e-12)
    want = np.array(brute_linattn(q[:, :9].tolist(), k[:, :9].tolist(), v[:, :9].tolist()))
    assert np.allclose(yq[:, :9], want, rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------------------------
# special cases with known answers
# --------------------------------------------------------------------------------------------
def test_linattn_special_cases():
    g = rng(11)
    U, N, dp, dv = 2, 40, 4, 3
    q = g.standard_normal((U, N, dp)); k = g.standard_normal((U, N, dp)); v = g.standard_normal((U, N, dv))
    running_mean = np.cumsum(v, axis=1) / np.arange(1, N + 1)[None, :, None]
    # q == 0 or k == 0: kernel is 1, output is the running mean of v (0th-order term)
    assert np.allclose(oracle.linattn_quadratic(np.zeros_like(q), k, v), running_mean, rtol=1e-12, atol=1e-13)
    assert np.allclose(oracle.linattn_quadratic(q, np.zeros_like(k), v), running_mean, rtol=1e-12, atol=1e-13)
    assert np.allclose(oracle.linattn_recurrent(np.zeros_like(q), k, v)[0], running_mean, rtol=1e-12, atol=1e-13)
    # first row is v_0
    y = oracle.linattn_quadratic(q, k, v)
    assert np.allclose(y[:, 0], v[:, 0], rtol=1e-14, atol=0)
    # constant v passes through; outputs are convex combinations (kernel is positive)
    c = np.broadcast_to(np.array([1.5, -2.0, 0.25]), v.shape).copy()
    assert np.allclose(oracle.linattn_quadratic(q, k, c), c, rtol=1e-12, atol=1e-13)
    lo = np.minimum.accumulate(v, axis=1); hi = np.maximum.accumulate(v, axis=1)
    assert (y >= lo - 1e-12).all() and (y <= hi + 1e-12).all()
    # state: row 0 is sum of v, z[0] counts tokens, (a,b) and (b,a) rows are identical
    S, z = oracle.linattn_state(k, v)
    assert np.allclose(S[:, 0], v.sum(1), rtol=1e-13, atol=1e-13)
    assert np.allclose(z[:, 0], N)
    assert np.allclose(S[:, 1:1 + dp], np.einsum("uja,ujc->uac", k, v), rtol=1e-12, atol=1e-13)
    blk = S[:, 1 + dp:].reshape(U, dp, dp, dv)
    assert np.array_equal(blk, blk.transpose(0, 2, 1, 3))
    zb = z[:, 1 + dp:].reshape(U, dp, dp)
    assert np.allclose(zb, np.einsum("uja,ujb->uab", k, k) / np.sqrt(2.0), rtol=1e-12, atol=1e-13)


def test_linattn_tracks_softmax_for_small_logits():
    """For |q.k| <= 0.1 the Taylor kernel is within |x|^3 e^|x| / 6 of exp(x), so the output agrees
    with unscaled causal softmax attention to that order (library routine, fp64)."""
    g = rng(13)
    U, N, dp, dv = 2, 48, 8, 4
    q = g.standard_normal((U, N, dp)); k = g.standard_normal((U, N, dp))
    q *= 0.3 / np.abs(q).max() / np.sqrt(dp); k *= 0.3 / np.abs(k).max() / np.sqrt(dp)
    v = g.standard_normal((U, N, dv))
    x = np.abs(np.einsum("uia,uja->uij", q, k)).max()
    assert x <= 0.1
    tq, tk, tv = (torch.from_numpy(a)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=1.0)[0].numpy()
    bound = 2.5 * (x ** 3 * math.exp(x) / 6.0) * np.abs(v).max()
    assert np.abs(oracle.linattn_quadratic(q, k, v) - ref).max() <= bound
    # sign/term check: dropping the quadratic term would exceed this bound
    first_order_gap = 0.25 * x * x * np.abs(v).max()
    assert bound < first_order_gap


# --------------------------------------------------------------------------------------------
# sliding-window attention
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,dh,w", [(33, 8, 33), (40, 16, 64), (17, 4, 1000)])
def test_swa_full_window_equals_library_causal_attention(N, dh, w):
    g = rng(400 + N)
    U = 3
    q = g.standard_normal((U, N, dh)); k = g.standard_normal((U, N, dh)); v = g.standard_normal((U, N, dh))
    scale = 1.0 / math.sqrt(dh)
    tq, tk, tv = (torch.from_numpy(a)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)[0].numpy()
    assert np.allclose(oracle.swa(q, k, v, w, scale), ref, rtol=1e-11, atol=1e-12)


def test_swa_banded_equals_library_attention_with_band_mask():
    g = rng(17)
    U, N, dh, w = 2, 50, 8, 7
    q = g.standard_normal((U, N, dh)); k = g.standard_normal((U, N, dh)); v = g.standard_normal((U, N, dh))
    i = np.arange(N)[:, None]; j = np.arange(N)[None, :]
    mask = torch.from_numpy((j <= i) & (j > i - w))
    tq, tk, tv = (torch.from_numpy(a)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.5)[0].numpy()
    assert np.allclose(oracle.swa(q, k, v, w, 0.5), ref, rtol=1e-11, atol=1e-12)


def test_swa_special_cases():
    g = rng(19)
    U, N, dh, w = 2, 30, 4, 5
    q = g.standard_normal((U, N, dh)); k = g.standard_normal((U, N, dh)); v = g.standard_normal((U, N, dh))
    # w = 1: every token sees only itself
    assert np.allclose(oracle.swa(q, k, v, 1, 0.5), v, rtol=1e-14, atol=0)
    # q = 0: mean of the last min(i + 1, w) values
    want = np.stack([v[:, max(0, i - w + 1):i + 1].mean(1) for i in range(N)], axis=1)
    assert np.allclose(oracle.swa(np.zeros_like(q), k, v, w, 0.5), want, rtol=1e-12, atol=1e-13)
    # adding a constant to every logit of a row changes nothing: shift k by a vector c with q.c constant
    # is not available in general, so use scale = 0 against q = 0 instead, and the shift via an extra
    # coordinate that is 1 in q and constant in k
    q1 = np.concatenate([q, np.ones((U, N, 1))], -1)
    k1 = np.concatenate([k, np.full((U, N, 1), 3.7)], -1)
    v1 = np.concatenate([v, np.zeros((U, N, 1))], -1)
    assert np.allclose(oracle.swa(q1, k1, v1, w, 0.5)[..., :dh], oracle.swa(q, k, v, w, 0.5), rtol=1e-11, atol=1e-12)
    # large logits do not overflow
    big = oracle.swa(q * 1e3, k * 1e3, v, w, 1.0)
    assert np.isfinite(big).all()
    # a decode step (one query against the last min(pos, w) cached rows, any cache order) is the prefill row
    y = oracle.swa(q, k, v, w, 0.5)
    for pos in (1, 3, w, w + 1, N):
        lo = max(0, pos - w)
        perm = g.permutation(pos - lo)
        kc, vc = k[:, lo:pos][:, perm], v[:, lo:pos][:, perm]
        # put the query last in a fresh sequence whose other rows are the permuted cache; window covers all
        qs = np.zeros((U, pos - lo, dh)); qs[:, -1] = q[:, pos - 1]
        row = oracle.swa_rows(qs, kc, vc, w, 0.5, np.array([pos - lo - 1]))[:, 0]
        assert np.allclose(row, y[:, pos - 1], rtol=1e-12, atol=1e-13)


def test_head_projection_pins():
    """Head-major projections against einsum written per head and torch's linear + view + transpose."""
    g = rng(9)
    B, N, dm, H, d = 2, 7, 12, 3, 4
    x = g.standard_normal((B, N, dm)); W = g.standard_normal((H * d, dm))
    got = oracle.project_heads(x, W, H)
    assert got.shape == (B, H, N, d)
    assert np.allclose(got, np.einsum("bnk,hjk->bhnj", x, W.reshape(H, d, dm)), rtol=1e-12, atol=1e-13)
    t = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(W)).view(B, N, H, d).transpose(1, 2)
    assert np.allclose(got, t.numpy(), rtol=1e-12, atol=1e-13)
    # one-hot weight: head h, feature j picks input column h d + j
    E = np.zeros((H * d, dm)); E[np.arange(H * d), np.arange(H * d)] = 1.0
    assert np.array_equal(oracle.project_heads(x, E, H)[:, 2, :, 1], x[:, :, 2 * d + 1])
    y = g.standard_normal((B, H, N, d)); Wo = g.standard_normal((dm, H * d))
    out = oracle.project_out(y, Wo)
    assert np.allclose(out, np.einsum("bhnj,mhj->bnm", y, Wo.reshape(dm, H, d)), rtol=1e-12, atol=1e-13)
    to = torch.nn.functional.linear(torch.from_numpy(y).transpose(1, 2).reshape(B, N, H * d), torch.from_numpy(Wo))
    assert np.allclose(out, to.numpy(), rtol=1e-12, atol=1e-13)


def test_rotary_pins():
    """The rotary encoding against its complex-number form, the 2x2 rotation matrix, and the properties
    that define it: norms kept, position 0 the identity, angles add, and q.k depending on the positions
    only through their difference."""
    g = rng(5)
    N, dh, base = 37, 8, 10000.0
    x = g.standard_normal((2, N, dh))
    pos = np.arange(N) * 3 + 11
    got = oracle.rotary(x, pos, base)
    # complex form: (x_2i + j x_2i+1) e^{j p theta_i}
    theta = np.array([base ** (-2.0 * i / dh) for i in range(dh // 2)])
    zc = (x[..., 0::2] + 1j * x[..., 1::2]) * np.exp(1j * pos[:, None] * theta[None, :])
    assert np.allclose(got[..., 0::2], zc.real, rtol=1e-12, atol=1e-13)
    assert np.allclose(got[..., 1::2], zc.imag, rtol=1e-12, atol=1e-13)
    # d_h = 2: one textbook rotation by p radians (theta_0 = 1)
    v2 = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -1.0]])
    p2 = np.array([0, 1, 2])
    r = oracle.rotary(v2, p2)
    for t in range(3):
        c, s_ = math.cos(p2[t]), math.sin(p2[t])
        assert np.allclose(r[t], [v2[t, 0] * c - v2[t, 1] * s_, v2[t, 0] * s_ + v2[t, 1] * c], rtol=1e-14, atol=1e-15)
    assert np.array_equal(oracle.rotary(x, np.zeros(N, dtype=np.int64)), x)
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    # pairwise norms too (each pair is rotated on its own)
    assert np.allclose(got[..., 0::2] ** 2 + got[..., 1::2] ** 2, x[..., 0::2] ** 2 + x[..., 1::2] ** 2, rtol=1e-12)
    # angles add: rotating by p then by p' is rotating by p + p'
    again = oracle.rotary(got, pos[::-1].copy(), base)
    assert np.allclose(again, oracle.rotary(x, pos + pos[::-1], base), rtol=1e-11, atol=1e-12)
    # relative positions: <R_m q, R_n k> = <R_{m-n} q, k>
    q = g.standard_normal((1, N, dh)); k = g.standard_normal((1, N, dh))
    rq, rk = oracle.rotary(q, pos, base), oracle.rotary(k, pos, base)
    for (m, n) in [(5, 2), (20, 20), (36, 0), (7, 30)]:
        lhs = rq[0, m] @ rk[0, n]
        rel = oracle.rotary(q[:, m:m + 1], np.array([pos[m] - pos[n]]), base)[0, 0] @ k[0, n]
        assert abs(lhs - rel) < 1e-11
    # the slowest pair: theta_{d/2 - 1} = base^(-(d-2)/d)
    one = np.zeros((1, 1, dh)); one[0, 0, dh - 2] = 1.0
    out = oracle.rotary(one, np.array([1000]), base)
    ang = 1000 * base ** (-(dh - 2) / dh)
    assert np.allclose(out[0, 0, dh - 2:], [math.cos(ang), math.sin(ang)], rtol=1e-13)


def test_swa_rotary_pins():
    """Window attention on rotary-encoded q, k: shifting every position by the same amount changes
    nothing (scores depend on position differences), and it equals library attention on separately
    rotated inputs with a band mask."""
    g = rng(6)
    U, N, dh, w, scale = 2, 50, 8, 16, 0.3
    q = g.standard_normal((U, N, dh)); k = g.standard_normal((U, N, dh)); v = g.standard_normal((U, N, dh))
    y0 = oracle.swa_rotary(q, k, v, w, scale, pos0=0)
    assert np.allclose(y0, oracle.swa_rotary(q, k, v, w, scale, pos0=1234), rtol=1e-9, atol=1e-10)
    assert not np.allclose(y0, oracle.swa(q, k, v, w, scale), rtol=1e-3, atol=1e-3)
    # library route: complex-form rotation, torch attention with an explicit band mask
    theta = 10000.0 ** (-2.0 * np.arange(dh // 2) / dh)
    ph = np.exp(1j * np.arange(N)[:, None] * theta[None, :])
    def rot(a):
        zc = (a[..., 0::2] + 1j * a[..., 1::2]) * ph
        out = np.empty_like(a); out[..., 0::2] = zc.real; out[..., 1::2] = zc.imag
        return out
    i = np.arange(N)[:, None]; j = np.arange(N)[None, :]
    mask = torch.from_numpy((j <= i) & (j > i - w))
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(rot(q)), torch.from_numpy(rot(k)), torch.from_numpy(v), attn_mask=mask, scale=scale).numpy()
    assert np.allclose(y0, want, rtol=1e-10, atol=1e-11)


def test_short_conv_gate_pins():
    """The BaseConv gate against library convolutions (numpy per channel, torch depthwise conv1d with left
    padding), SiLU values, causality, the identity filter, and continuation from the previous rows."""
    g = rng(8)
    B, N, Dc, K = 2, 29, 6, 3
    a = g.standard_normal((B, N, Dc)); c = g.standard_normal((B, N, Dc))
    h = g.standard_normal((K, Dc)); b1 = g.standard_normal(Dc); b2 = g.standard_normal(Dc)
    got = oracle.short_conv_gate(a, c, h, b1, b2)
    silu = lambda x: x / (1.0 + np.exp(-x))
    # numpy's full convolution per channel, truncated to the first N outputs
    for b in range(B):
        for ch in range(Dc):
            conv = np.convolve(c[b, :, ch], h[:, ch])[:N]
            assert np.allclose(got[b, :, ch], (a[b, :, ch] + b1[ch]) * silu(conv + b2[ch]), rtol=1e-12, atol=1e-13)
    # torch: depthwise conv1d (cross-correlation, so the filter is flipped) after K - 1 zeros on the left
    x = torch.from_numpy(c).transpose(1, 2)
    wt = torch.from_numpy(h[::-1].copy().T).unsqueeze(1)     # [Dc, 1, K], tap K - 1 is the current token
    conv_t = torch.nn.functional.conv1d(torch.nn.functional.pad(x, (K - 1, 0)), wt, groups=Dc).transpose(1, 2).numpy()
    assert np.allclose(got, (a + b1) * torch.nn.functional.silu(torch.from_numpy(conv_t + b2)).numpy(), rtol=1e-12, atol=1e-13)
    # SiLU: 0 at 0, x sigmoid(x) elsewhere; with h = [1, 0, 0], b2 = 0 the gate is (a + b1) silu(c)
    e0 = np.zeros((K, Dc)); e0[0] = 1.0
    assert np.allclose(oracle.short_conv_gate(a, c, e0, b1, np.zeros(Dc)), (a + b1) * c / (1 + np.exp(-c)), rtol=1e-13)
    assert np.array_equal(oracle.short_conv_gate(a, np.zeros_like(c), h, b1, np.zeros(Dc)), np.zeros_like(a))
    one = oracle.short_conv_gate(np.ones((1, 1, 1)), np.ones((1, 1, 1)), np.array([[1.0], [5.0], [7.0]]), np.zeros(1), np.zeros(1))
    assert abs(one[0, 0, 0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    # a pure delay: h = [0, 0, 1] reads the token two back
    e2 = np.zeros((K, Dc)); e2[2] = 1.0
    d2 = oracle.short_conv_gate(np.ones_like(a), c, e2, np.zeros(Dc), np.zeros(Dc))
    assert np.allclose(d2[:, 2:], silu(c[:, :-2]), rtol=1e-13) and np.array_equal(d2[:, :2], np.zeros((B, 2, Dc)))
    # causal: changing the future leaves the past alone
    c2 = c.copy(); c2[:, 17:] += 1.0
    assert np.array_equal(oracle.short_conv_gate(a, c2, h, b1, b2)[:, :17], got[:, :17])
    # continuation: the second part with the last two rows of the first equals the whole
    N1 = 11
    part2 = oracle.short_conv_gate(a[:, N1:], c[:, N1:], h, b1, b2, c_prev=c[:, N1 - 2:N1])
    assert np.allclose(part2, got[:, N1:], rtol=1e-13, atol=1e-14)
    # the whole layer: the same three steps through torch's linear layers
    d = 4
    u = g.standard_normal((B, N, d)); W1 = g.standard_normal((Dc, d)); W2 = g.standard_normal((Dc, d))
    W3 = g.standard_normal((d, Dc)); b3 = g.standard_normal(d)
    tl = torch.nn.functional.linear
    ut = torch.from_numpy(u)
    at = tl(ut, torch.from_numpy(W1), torch.from_numpy(b1))
    ct = tl(ut, torch.from_numpy(W2)).transpose(1, 2)
    cv = torch.nn.functional.conv1d(torch.nn.functional.pad(ct, (K - 1, 0)), wt, groups=Dc).transpose(1, 2) + torch.from_numpy(b2)
    want = tl(at * torch.nn.functional.silu(cv), torch.from_numpy(W3), torch.from_numpy(b3)).numpy()
    assert np.allclose(oracle.baseconv(u, W1, b1, W2, b2, h, W3, b3), want, rtol=1e-11, atol=1e-12)


def test_linear_projection_pins():
    """y = x W^T against what fixes it: brute-force loops, the identity and a one-hot weight (picks a
    column of x), a closed form with constant rows, and linearity in each argument (a transposed operand
    or a swapped index fails the brute-force and the one-hot case)."""
    g = rng(23)
    M, K, N = 5, 7, 3
    x = g.standard_normal((M, K)); W = g.standard_normal((N, K))
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            for kk in range(K):
                want[m, n] += x[m, kk] * W[n, kk]
    assert np.allclose(oracle.linear(x, W), want, rtol=1e-13, atol=1e-14)
    assert np.array_equal(oracle.linear(x, np.eye(K)), x)
    onehot = np.zeros((2, K)); onehot[0, 4] = 1.0; onehot[1, 1] = -2.0
    assert np.array_equal(oracle.linear(x, onehot), np.stack([x[:, 4], -2.0 * x[:, 1]], axis=1))
    # x row m constant c_m, W row n constant d_n: y[m, n] = K c_m d_n
    c = g.standard_normal(M); d = g.standard_normal(N)
    y = oracle.linear(np.repeat(c[:, None], K, 1), np.repeat(d[:, None], K, 1))
    assert np.allclose(y, K * np.outer(c, d), rtol=1e-13, atol=0)
    x2 = g.standard_normal((M, K)); W2 = g.standard_normal((N, K))
    assert np.allclose(oracle.linear(2 * x + x2, W), 2 * oracle.linear(x, W) + oracle.linear(x2, W), rtol=1e-12, atol=1e-13)
    assert np.allclose(oracle.linear(x, W - 3 * W2), oracle.linear(x, W) - 3 * oracle.linear(x, W2), rtol=1e-12, atol=1e-13)
    with pytest.raises(ValueError):
        oracle.linear(x, g.standard_normal((N, K + 1)))


def test_oracle_threads_reported():
    assert oracle.threads() >= 1

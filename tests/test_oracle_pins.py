"""Pins for the fp64 oracle: each test checks it against something other than itself.

What fixes the expected values: closed forms of the Hard-Concrete sampler
(Section 3), the agreement the paper asserts between that sampler and Eq.(3)
(checked by Monte-Carlo), identities of Section 4.1 evaluated with numpy's
matmul (all gates open, rank-1 sum, input-feature pruning, absorbing G),
closing-equals-deleting (Sections 4.1/4.4), central finite differences for
every gradient, brute-force compaction and the one-hot form of Section 4.2.
Golden constants in ``tests/golden/hard_concrete_points.txt`` are closed-form
values worked out by hand from those displays.
"""
import math
import os

import numpy as np
import pytest

import oracle
from paper_1910_04732_amd import synth

BETA, L, R = 2.0 / 3.0, -0.1, 1.1
GOLD = os.path.join(os.path.dirname(__file__), "golden", "hard_concrete_points.txt")


def _rng(seed):
    return np.random.default_rng(seed)


def _tiny(seed, n=3, d=4, r=5, dout=2):
    g = _rng(seed)
    return (g.standard_normal((n, d)), g.standard_normal((r, d)), g.standard_normal((dout, r)),
            g.standard_normal((n, dout)), g.standard_normal(r), g.uniform(0.05, 0.95, r))


# ----------------------------------------------------------------- sampler ---
def test_golden_points():
    """Hand-derived points of the sampler and of Eq.(3) (see the fixture's header)."""
    rows = [ln.split() for ln in open(GOLD) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 8
    for kind, *vals in rows:
        vals = [float(v) for v in vals]
        if kind == "gate":
            beta, l, r, alpha, u, z_exp = vals
            z, _ = oracle.gate_sample([alpha], [u], beta, l, r)
            assert z[0] == pytest.approx(z_exp, abs=1e-6)
        elif kind == "gate_det":
            l, r, alpha, z_exp = vals
            z, _ = oracle.gate_sample([alpha], None, 1.0, l, r, deterministic=True)
            assert z[0] == pytest.approx(z_exp, abs=1e-6)
        elif kind == "gate_det_grad":
            beta, l, r, alpha, d_exp = vals
            _, dzda = oracle.gate_sample([alpha], None, beta, l, r, deterministic=True)
            assert dzda[0] == pytest.approx(d_exp, abs=1e-12)
        elif kind == "l0":
            beta, l, r, alpha, count, s_exp = vals
            s, _ = oracle.expected_l0(np.full(int(count), alpha), beta, l, r)
            assert s == pytest.approx(s_exp, rel=2e-6)
        else:
            raise AssertionError(kind)


@pytest.mark.parametrize("beta", [1.0, 2.0 / 3.0, 0.5])
def test_gate_midpoint_and_range(beta):
    # u = 1/2 and alpha = 0 give s = 1/2 whatever the temperature: z = (l + r) / 2.
    z, dzda = oracle.gate_sample([0.0], [0.5], beta, L, R)
    assert z[0] == pytest.approx(0.5, abs=1e-15)
    assert dzda[0] == pytest.approx((R - L) * 0.25 / beta, rel=1e-14)
    g = _rng(1)
    a = g.normal(0, 3, 4000)
    u = g.uniform(1e-6, 1 - 1e-6, 4000)
    z, dzda = oracle.gate_sample(a, u, beta, L, R)
    assert z.min() >= 0.0 and z.max() <= 1.0
    assert (z == 0).any() and (z == 1).any() and ((z > 0) & (z < 1)).any()
    assert np.all(dzda[(z == 0) | (z == 1)] == 0.0)
    assert np.all(dzda[(z > 0) & (z < 1)] > 0.0)


def test_gate_thresholds_and_monotone():
    # z = 0  <=>  logit(u) + alpha <= beta log(-l/r);  z = 1  <=>  >= beta log((1-l)/(r-1)).
    lo = BETA * math.log(-L / R)
    hi = BETA * math.log((1 - L) / (R - 1))
    assert lo == pytest.approx(-1.598597, abs=1e-6) and hi == pytest.approx(1.598597, abs=1e-6)
    for eps, z_is_zero, z_is_one in ((-1e-9, True, False), (1e-9, False, False)):
        z, _ = oracle.gate_sample([lo + eps], [0.5], BETA, L, R)
        assert (z[0] == 0.0) == z_is_zero
    z, _ = oracle.gate_sample([hi + 1e-9, hi - 1e-9], [0.5, 0.5], BETA, L, R)
    assert z[0] == 1.0 and z[1] < 1.0
    t = np.linspace(-6, 6, 801)
    z_a, _ = oracle.gate_sample(t, np.full_like(t, 0.3), BETA, L, R)
    assert np.all(np.diff(z_a) >= 0)
    uu = np.linspace(1e-4, 1 - 1e-4, 801)
    z_u, _ = oracle.gate_sample(np.full_like(uu, 0.2), uu, BETA, L, R)
    assert np.all(np.diff(z_u) >= 0)
    # logit(u) shifts alpha: G(u; alpha) depends on logit(u) + alpha only.
    z1, _ = oracle.gate_sample([0.7], [0.25], BETA, L, R)
    z2, _ = oracle.gate_sample([0.7 + math.log(0.25 / 0.75)], [0.5], BETA, L, R)
    assert z1[0] == pytest.approx(z2[0], abs=1e-14)


def test_deterministic_gate():
    # closed  <=>  alpha <= log(-l/r), whatever beta; alpha = 0 gives (l + r)/2.
    thr = math.log(-L / R)
    z, _ = oracle.gate_sample([thr - 1e-9, thr + 1e-9, 0.0, 30.0], None, BETA, L, R, deterministic=True)
    assert z[0] == 0.0 and z[1] > 0.0 and z[2] == pytest.approx(0.5) and z[3] == 1.0


def test_deterministic_gate_gradient():
    """dz/dalpha of the deterministic gate z = clamp(sigmoid(alpha)(r - l) + l): no temperature in it, so it is
    (r - l) s (1 - s) whatever beta is, zero outside the clamp, and the slope of z itself."""
    a = np.array([-2.0, -1.0, -0.3, 0.0, 0.4, 1.0986122886681098, 2.0])       # all strictly inside the clamp
    for beta in (1.0, 2.0 / 3.0, 0.25):
        z, dzda = oracle.gate_sample(a, None, beta, L, R, deterministic=True)
        assert np.all((z > 0) & (z < 1))
        s = 1.0 / (1.0 + np.exp(-a))
        np.testing.assert_allclose(dzda, (R - L) * s * (1 - s), rtol=1e-13)
        h = 1e-6
        zp, _ = oracle.gate_sample(a + h, None, beta, L, R, deterministic=True)
        zm, _ = oracle.gate_sample(a - h, None, beta, L, R, deterministic=True)
        np.testing.assert_allclose(dzda, (zp - zm) / (2 * h), rtol=1e-8)
    # beta does enter the training mode: the two modes differ by exactly 1/beta at u = 1/2
    _, d_train = oracle.gate_sample([0.0], [0.5], 0.25, L, R)
    _, d_det = oracle.gate_sample([0.0], None, 0.25, L, R, deterministic=True)
    assert d_train[0] == pytest.approx(4.0 * d_det[0], rel=1e-14)
    # closed and saturated gates pass no gradient
    _, dz = oracle.gate_sample([math.log(-L / R) - 0.5, math.log((1 - L) / (R - 1)) + 0.5], None, BETA, L, R,
                               deterministic=True)
    assert dz[0] == 0.0 and dz[1] == 0.0


def test_noise_at_the_ends_of_its_range():
    """u = 0 and u = 1 (outside the open interval the workloads draw from): log u - log(1 - u) is -inf / +inf,
    so the gate is closed / saturated whatever alpha is, with zero slope and no NaN."""
    z, dzda = oracle.gate_sample([-3.0, 0.0, 25.0, -25.0, 0.0, 3.0], [0.0, 0.0, 0.0, 1.0, 1.0, 1.0], BETA, L, R)
    assert z.tolist() == [0.0, 0.0, 0.0, 1.0, 1.0, 1.0] and dzda.tolist() == [0.0] * 6


@pytest.mark.parametrize("beta,alpha", [(1.0, 0.0), (2.0 / 3.0, 0.0), (2.0 / 3.0, -1.3), (0.5, 0.8)])
def test_eq3_matches_sampler_monte_carlo(beta, alpha):
    """Eq.(3) says P[z > 0] = sigmoid(alpha - beta log(-l/r)): count it."""
    N = 2_000_000
    u = _rng(7).uniform(0.0, 1.0, N)
    u = np.clip(u, 1e-300, 1 - 1e-16)
    z, _ = oracle.gate_sample(np.full(N, alpha), u, beta, L, R)
    freq = np.count_nonzero(z > 0) / N
    s, _ = oracle.expected_l0(np.full(1, alpha), beta, L, R)
    assert abs(freq - s) < 4.0 * math.sqrt(s * (1 - s) / N)
    # symmetric stretch (l = 1 - r): P[z = 0 | alpha] = P[z = 1 | -alpha]
    z_neg, _ = oracle.gate_sample(np.full(N, -alpha), u, beta, L, R)
    p0 = np.count_nonzero(z == 0) / N
    p1 = np.count_nonzero(z_neg == 1) / N
    assert abs(p0 - p1) < 6.0 * math.sqrt(max(p0, 1e-4) / N)


def test_expected_l0_limits_weights_grad():
    s, _ = oracle.expected_l0(np.full(10, 50.0), BETA, L, R)
    assert s == pytest.approx(10.0)
    s, _ = oracle.expected_l0(np.full(10, -50.0), BETA, L, R)
    assert s == pytest.approx(0.0, abs=1e-12)
    # beta = 1 is the paper's sigmoid(alpha + 2.397895)
    s, _ = oracle.expected_l0([0.3], 1.0, L, R)
    assert s == pytest.approx(1 / (1 + math.exp(-(0.3 + 2.3978952728)))), s
    g = _rng(3)
    a = g.normal(0, 2, 37)
    w = g.uniform(1, 9, 37)
    s_w, grad = oracle.expected_l0(a, BETA, L, R, w)
    per = np.array([oracle.expected_l0(a[k:k + 1], BETA, L, R)[0] for k in range(37)])
    assert s_w == pytest.approx(float(np.dot(w, per)), rel=1e-13)
    h = 1e-6
    for k in (0, 11, 36):
        ap, am = a.copy(), a.copy()
        ap[k] += h
        am[k] -= h
        fd = (oracle.expected_l0(ap, BETA, L, R, w)[0] - oracle.expected_l0(am, BETA, L, R, w)[0]) / (2 * h)
        assert grad[k] == pytest.approx(fd, rel=1e-6)


# ----------------------------------------------------------------- forward ---
def test_all_gates_open_is_dense_product():
    g = _rng(11)
    n, d, r, dout = 17, 13, 9, 21
    x, Q, P = g.standard_normal((n, d)), g.standard_normal((r, d)), g.standard_normal((dout, r))
    h, gg, y = oracle.fwd(x, Q, P, np.ones(r))
    W = P @ Q
    np.testing.assert_allclose(y, x @ W.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(h, x @ Q.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gg, h, rtol=0, atol=0)


def test_rank1_sum_absorb_and_feature_pruning():
    g = _rng(12)
    n, d, r, dout = 10, 7, 6, 5
    x, Q, P = g.standard_normal((n, d)), g.standard_normal((r, d)), g.standard_normal((dout, r))
    z = g.uniform(0, 1, r)
    z[2] = 0.0
    _, gg, y = oracle.fwd(x, Q, P, z)
    W_eff, y1 = oracle.fwd_rank1(x, Q, P, z)
    W_np = sum(z[k] * np.outer(P[:, k], Q[k, :]) for k in range(r))
    np.testing.assert_allclose(W_eff, W_np, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y, x @ W_np.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(y1, y, rtol=1e-12, atol=1e-12)
    # G absorbed into Q or into P
    np.testing.assert_allclose(y, x @ (z[:, None] * Q).T @ P.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(y, (x @ Q.T) @ (P * z[None, :]).T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gg, (x @ Q.T) * z[None, :], rtol=1e-12, atol=1e-13)
    # input-feature pruning: P = W, Q = I gives (x .* z) W^T
    W = g.standard_normal((dout, d))
    zz = g.uniform(0, 1, d)
    _, _, yf = oracle.fwd(x, np.eye(d), W, zz)
    np.testing.assert_allclose(yf, (x * zz[None, :]) @ W.T, rtol=1e-12, atol=1e-12)


def test_closing_a_gate_deletes_the_component():
    g = _rng(13)
    n, d, r, dout = 8, 6, 7, 5
    x, Q, P = g.standard_normal((n, d)), g.standard_normal((r, d)), g.standard_normal((dout, r))
    z = g.uniform(0.1, 1, r)
    z[[1, 4]] = 0.0
    _, _, y = oracle.fwd(x, Q, P, z)
    keep = [0, 2, 3, 5, 6]
    _, _, y_del = oracle.fwd(x, Q[keep], P[:, keep], z[keep])
    np.testing.assert_allclose(y, y_del, rtol=1e-13, atol=1e-13)
    idx, Qc, Pc, zc = oracle.compact(z, Q, P)
    assert idx.tolist() == keep
    _, _, y_c = oracle.fwd(x, Qc, Pc, zc)
    np.testing.assert_array_equal(y_c, y_del)


# ---------------------------------------------------------------- backward ---
def _loss(x, Q, P, alpha, u, dy):
    z, _ = oracle.gate_sample(alpha, u, BETA, L, R)
    return float(np.sum(oracle.fwd(x, Q, P, z)[2] * dy))


def test_finite_differences_all_gradients():
    x, Q, P, dy, alpha, u = _tiny(21)
    # keep every gate strictly inside (0, 1) except one closed and one saturated
    alpha[:] = [0.2, -0.4, 0.6, -9.0, 9.0]
    u[:] = [0.4, 0.55, 0.5, 0.5, 0.5]
    z, dzda = oracle.gate_sample(alpha, u, BETA, L, R)
    assert z[3] == 0 and z[4] == 1 and np.all((z[:3] > 0.05) & (z[:3] < 0.95))
    out = oracle.bwd(dy, x, Q, P, z, dzda)
    h = 1e-6

    def fd(arr, idx):
        orig = arr[idx]
        arr[idx] = orig + h
        fp = _loss(x, Q, P, alpha, u, dy)
        arr[idx] = orig - h
        fm = _loss(x, Q, P, alpha, u, dy)
        arr[idx] = orig
        return (fp - fm) / (2 * h)

    for name, arr in (("dx", x), ("dQ", Q), ("dP", P), ("dalpha", alpha)):
        num = np.empty_like(arr)
        for idx in np.ndindex(*arr.shape):
            num[idx] = fd(arr, idx)
        np.testing.assert_allclose(out[name], num, rtol=2e-6, atol=2e-7, err_msg=name)
    assert out["dalpha"][3] == 0.0 and out["dalpha"][4] == 0.0
    # dz is the derivative w.r.t. the gate value itself
    for k in range(5):
        zp, zm = z.copy(), z.copy()
        zp[k] += h
        zm[k] -= h
        num = (np.sum(oracle.fwd(x, Q, P, zp)[2] * dy) - np.sum(oracle.fwd(x, Q, P, zm)[2] * dy)) / (2 * h)
        assert out["dz"][k] == pytest.approx(num, rel=1e-6, abs=1e-7)


def test_backward_matches_numpy_matmul_and_adjoint():
    g = _rng(22)
    n, d, r, dout = 19, 11, 8, 14
    x, Q, P = g.standard_normal((n, d)), g.standard_normal((r, d)), g.standard_normal((dout, r))
    dy = g.standard_normal((n, dout))
    z = g.uniform(0, 1, r)
    dzda = g.uniform(0, 2, r)
    out = oracle.bwd(dy, x, Q, P, z, dzda)
    W_eff = (P * z[None, :]) @ Q
    np.testing.assert_allclose(out["dx"], dy @ W_eff, rtol=1e-12, atol=1e-12)
    hh = x @ Q.T
    dg = dy @ P
    np.testing.assert_allclose(out["dP"], dy.T @ (hh * z), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dQ"], (dg * z).T @ x, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dz"], np.sum(dg * hh, axis=0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dalpha"], out["dz"] * dzda, rtol=1e-14, atol=0)
    # adjoint identity <dy, y(x)> = <dx, x>
    _, _, y = oracle.fwd(x, Q, P, z)
    assert float(np.sum(dy * y)) == pytest.approx(float(np.sum(out["dx"] * x)), rel=1e-12)


def test_closed_ranks_get_zero_gradient_and_compacted_backward_agrees():
    g = _rng(23)
    n, d, r, dout = 9, 6, 7, 5
    x, Q, P = g.standard_normal((n, d)), g.standard_normal((r, d)), g.standard_normal((dout, r))
    dy = g.standard_normal((n, dout))
    alpha = g.normal(0, 1, r)
    alpha[[0, 5]] = -20.0
    u = g.uniform(0.2, 0.8, r)
    z, dzda = oracle.gate_sample(alpha, u, BETA, L, R)
    full = oracle.bwd(dy, x, Q, P, z, dzda)
    assert np.all(full["dP"][:, [0, 5]] == 0) and np.all(full["dQ"][[0, 5]] == 0)
    assert np.all(full["dalpha"][[0, 5]] == 0)
    idx, Qc, Pc, zc = oracle.compact(z, Q, P)
    small = oracle.bwd(dy, x, Qc, Pc, zc, dzda[idx])
    np.testing.assert_allclose(small["dx"], full["dx"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(small["dP"], full["dP"][:, idx], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(small["dQ"], full["dQ"][idx], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(small["dalpha"], full["dalpha"][idx], rtol=1e-13, atol=1e-13)


# -------------------------------------------------------------- compaction ---
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_compaction_brute_force(seed):
    g = _rng(30 + seed)
    d, r, dout = 5, 23, 4
    Q, P = g.standard_normal((r, d)), g.standard_normal((dout, r))
    z = g.uniform(-1, 1, r).clip(0, 1)
    if seed == 1:
        z[:] = 0.0
    if seed == 2:
        z[:] = 0.5
    idx, Qc, Pc, zc = oracle.compact(z, Q, P)
    mask = z > 0
    assert idx.tolist() == np.flatnonzero(mask).tolist()
    np.testing.assert_array_equal(Qc, Q[mask])
    np.testing.assert_array_equal(Pc, P[:, mask])
    np.testing.assert_array_equal(zc, z[mask])
    _, Qa, Pa, _ = oracle.compact(z, Q, P, absorb=True)
    np.testing.assert_array_equal(Qa, z[mask][:, None] * Q[mask])
    np.testing.assert_array_equal(Pa, P[:, mask])


# --------------------------------------------------------------- embedding ---
def test_embedding_equals_one_hot_layer():
    """E_i G_i O_i looked up by id is the gated layer applied to one-hot rows."""
    g = _rng(40)
    offsets = (0, 6, 15, 19)
    dims = (5, 3, 2)
    d = 7
    ids = np.array([0, 5, 6, 14, 15, 18, 5, 5, 7, 0, 16, 6], dtype=np.int64)
    E = [g.standard_normal((offsets[c + 1] - offsets[c], dims[c])) for c in range(3)]
    O = [g.standard_normal((dims[c], d)) for c in range(3)]
    alpha = [g.normal(0.5, 1, dims[c]) for c in range(3)]
    u = [g.uniform(0.1, 0.9, dims[c]) for c in range(3)]
    zd = [oracle.gate_sample(alpha[c], u[c], BETA, L, R) for c in range(3)]
    z = [a for a, _ in zd]
    dzda = [b for _, b in zd]
    dy = g.standard_normal((len(ids), d))
    y = oracle.embed_fwd(ids, offsets, E, O, z)
    grads = oracle.embed_bwd(ids, offsets, dy, E, O, z, dzda)
    y_ref = np.zeros_like(y)
    for c in range(3):
        rows = offsets[c + 1] - offsets[c]
        sel = np.flatnonzero((ids >= offsets[c]) & (ids < offsets[c + 1]))
        onehot = np.zeros((len(sel), rows))
        onehot[np.arange(len(sel)), ids[sel] - offsets[c]] = 1.0
        # x = one-hot, Q = E^T (r x rows), P = O^T (d x r)
        _, _, yc = oracle.fwd(onehot, E[c].T, O[c].T, z[c])
        y_ref[sel] = yc
        np.testing.assert_allclose(yc, (E[c][ids[sel] - offsets[c]] * z[c]) @ O[c], rtol=1e-12, atol=1e-12)
        b = oracle.bwd(dy[sel], onehot, E[c].T, O[c].T, z[c], dzda[c])
        np.testing.assert_allclose(grads[c]["dE"], b["dQ"].T, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(grads[c]["dO"], b["dP"].T, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(grads[c]["dalpha"], b["dalpha"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(y, y_ref, rtol=1e-12, atol=1e-12)


# ------------------------------------------- Section 4.4: the paper's own inference mask ---
def test_topk_mask_against_sorting_and_threshold_form():
    g = np.random.default_rng(41)
    alpha = np.round(g.standard_normal(300) * 1.5, 1)   # one decimal: plenty of ties
    shift = BETA * math.log(-L / R)
    p = 1.0 / (1.0 + np.exp(-(alpha - shift)))
    for keep in (0, 1, 17, 150, 299, 300, 400, -3):
        z, kept = oracle.topk_mask(alpha, keep, BETA, L, R)
        want = min(max(keep, 0), 300)
        assert kept == want == np.count_nonzero(z)
        # library sort as the independent definition: descending alpha, stable in the index
        order = np.argsort(-alpha, kind="stable")[:want]
        ref = np.zeros(300)
        ref[order] = p[order]
        np.testing.assert_allclose(z, ref, rtol=1e-15, atol=0)
        if 0 < want < 300:
            kept_idx, dropped = np.flatnonzero(z), np.flatnonzero(z == 0)
            assert alpha[kept_idx].min() >= alpha[dropped].max()
            # among gates equal to the smallest kept alpha, the kept ones come first
            edge = alpha[kept_idx].min()
            tied_kept, tied_dropped = kept_idx[alpha[kept_idx] == edge], dropped[alpha[dropped] == edge]
            if tied_dropped.size:
                assert tied_kept.max() < tied_dropped.min()
    # keeping as many gates as the threshold form leaves open selects the same components
    alpha = g.standard_normal(500) * 2.0
    z_thr, _ = oracle.gate_sample(alpha, None, BETA, L, R, deterministic=True)
    z_top, kept = oracle.topk_mask(alpha, int(np.count_nonzero(z_thr)), BETA, L, R)
    np.testing.assert_array_equal(z_top > 0, z_thr > 0)
    # the kept values are the per-gate terms of Eq.(3): all gates kept -> they add up to the expected L0
    z_all, _ = oracle.topk_mask(alpha, 500, BETA, L, R)
    s, _ = oracle.expected_l0(alpha, BETA, L, R)
    assert abs(z_all.sum() - s) < 1e-10


# ------------------------------------------- Section 4.3: augmented-Lagrangian penalty ---
def test_lagrangian_penalty_values_and_gradients():
    g = np.random.default_rng(43)
    alpha = g.standard_normal(60)
    w = g.integers(100, 4000, 60).astype(np.float64)
    total = w.sum()
    s, ds = oracle.expected_l0(alpha, BETA, L, R, w)
    for (t, l1, l2) in ((0.3, 0.7, 2.5), (0.9, -0.4, 0.0), (s / total, 1.3, 5.0)):
        val, d1, d2, da = oracle.lagrangian(alpha, BETA, L, R, 1.0 / total, t, l1, l2, w)
        viol = s / total - t
        assert abs(val - (l1 * viol + l2 * viol ** 2)) < 1e-13
        assert abs(d1 - viol) < 1e-13 and abs(d2 - viol ** 2) < 1e-13
        np.testing.assert_allclose(da, (l1 + 2 * l2 * viol) * ds / total, rtol=1e-12, atol=1e-18)
        # central differences of the penalty itself
        for k in (0, 17, 59):
            e = np.zeros(60); e[k] = 1e-6
            vp = oracle.lagrangian(alpha + e, BETA, L, R, 1.0 / total, t, l1, l2, w)[0]
            vm = oracle.lagrangian(alpha - e, BETA, L, R, 1.0 / total, t, l1, l2, w)[0]
            assert abs((vp - vm) / 2e-6 - da[k]) < 1e-8 * max(1.0, abs(da[k]))
    # constraint met: the penalty vanishes, the multipliers get no push, alpha only feels lambda1
    val, d1, d2, da = oracle.lagrangian(alpha, BETA, L, R, 1.0 / total, s / total, 1.3, 5.0, w)
    assert abs(val) < 1e-13 and abs(d1) < 1e-13 and d2 < 1e-26
    np.testing.assert_allclose(da, 1.3 * ds / total, rtol=1e-10)
    # unweighted, unscaled form against the closed form for equal gates: s = R * p
    val, d1, _, da = oracle.lagrangian(np.full(8, 0.25), 1.0, L, R, 1.0, 3.0, 2.0, 0.5)
    pp = 1.0 / (1.0 + math.exp(-(0.25 - math.log(-L / R))))
    assert abs(d1 - (8 * pp - 3.0)) < 1e-13
    assert abs(val - (2.0 * d1 + 0.5 * d1 * d1)) < 1e-13
    np.testing.assert_allclose(da, np.full(8, (2.0 + d1) * pp * (1 - pp)), rtol=1e-12)


# ------------------------------------------------------------ input recipe ---
def test_synth_is_seeded_and_storage_rounded():
    a = synth.normal(5, (64, 33), 0.0, 1.0, "bf16")
    b = synth.normal(5, (64, 33), 0.0, 1.0, "bf16")
    np.testing.assert_array_equal(a, b)
    # bf16 values survive a float32 round trip and have at most 8 significant bits
    f = a.astype(np.float32)
    assert np.all((f.view(np.uint32) & 0xFFFF) == 0)
    big = synth.normal(6, (200000,), 1.0, 2.0, "f32")
    assert abs(big.mean() - 1.0) < 0.02 and abs(big.var() - 2.0) < 0.03
    uu = synth.uniform(7, (100000,), 1e-6, 1 - 1e-6, "f32")
    assert uu.min() >= 1e-6 * 0.999 and uu.max() < 1.0 and abs(uu.mean() - 0.5) < 0.01
    ids = synth.zipf_ids(8, 8192, synth.C5_VOCAB, 1.1)
    assert ids.min() >= 0 and ids.max() < synth.C5_VOCAB
    assert np.count_nonzero(ids < 20000) > 6500  # Zipf head dominates
    c4 = synth.config_c4(0.2, n=4, d=8, r=200, dout=8)
    thr = math.log(-L / R)
    assert np.count_nonzero(c4["log_alpha"] > thr) == 40
    assert np.min(np.abs(c4["log_alpha"] - thr)) >= 0.049

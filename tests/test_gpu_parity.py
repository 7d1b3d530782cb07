"""GPU parity: every C-ABI entry point against the fp64 oracle on the same seeded inputs.

Tolerances (written here, per the stated targets): max-abs and Frobenius
relative error <= 1e-5 for float32 and <= 2e-2 for bfloat16 tensors against
the fp64 oracle; gate values, Eq.(3) sums <= 1e-5; compaction indices and
copied entries bit-exact.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_1910_04732_amd import flop, synth
from _util import TOL, TORCH_DT, assert_close, dev, hc_struct, padded, to_dev, to_np

pytestmark = pytest.mark.gpu

BETA, L, R = synth.BETA, synth.L, synth.R


# ---------------------------------------------------------------------------
def run_layer(c, beta=BETA, pad=0, grads=("dx", "dQ", "dP", "dalpha"), accumulate=False, align=0):
    """gate -> fwd -> bwd on the GPU for the synth layer ``c``; returns dict of numpy results.

    ``pad`` extra elements per row, or (``align``) rows padded to a multiple of ``align`` elements;
    the padding of the inputs holds junk.
    """
    dt = c["dtype"]
    n, d, r, dout = c["n"], c["d"], c["r"], c["dout"]
    hc = hc_struct(beta)
    ld = (lambda cols: -(-cols // align) * align) if align else (lambda cols: cols + pad)
    mk = (lambda a, cols: padded(to_dev(a, dt), ld(cols))) if (pad or align) else (lambda a, cols: to_dev(a, dt))
    x, Q, P, dy = mk(c["x"], d), mk(c["Q"], d), mk(c["P"], r), mk(c["dy"], dout)
    la, u = to_dev(c["log_alpha"]), to_dev(c["u"])
    z, dzda = torch.empty_like(la), torch.empty_like(la)
    flop.flop_gate_sample(la, u, hc, flop.FLOP_GATE_TRAIN, z, dzda)
    tdt = TORCH_DT[dt]
    out_buf = lambda rows, cols: torch.full((rows, ld(cols)), 5.0, dtype=tdt, device=dev())[:, :cols]
    g, y = out_buf(n, r), out_buf(n, dout)
    flop.flop_fwd(x, Q, P, z, g, y)
    dx = out_buf(n, d) if "dx" in grads else None
    dQ = out_buf(r, d) if "dQ" in grads else None
    dP = out_buf(dout, r) if "dP" in grads else None
    da = torch.full((r,), 3.0 if accumulate else float("nan"), dtype=torch.float32, device=dev()) \
        if "dalpha" in grads else None
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(x), n, d, r, dout), dev())
    flop.flop_bwd(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da, ws, accumulate=accumulate)
    torch.cuda.synchronize()
    out = dict(z=z, dzda=dzda, g=g, y=y, dx=dx, dQ=dQ, dP=dP, dalpha=da)
    return {k: (None if v is None else to_np(v)) for k, v in out.items()}


def oracle_layer(c, beta=BETA):
    z, dzda = oracle.gate_sample(c["log_alpha"], c["u"], beta, L, R)
    _, g, y = oracle.fwd(c["x"], c["Q"], c["P"], z)
    b = oracle.bwd(c["dy"], c["x"], c["Q"], c["P"], z, dzda)
    return dict(z=z, dzda=dzda, g=g, y=y, **b)


def check_layer(c, beta=BETA, pad=0, align=0):
    got = run_layer(c, beta, pad, align=align)
    want = oracle_layer(c, beta)
    tol = TOL[c["dtype"]]
    assert_close(got["z"], want["z"], 1e-5, "z")
    assert_close(got["dzda"], want["dzda"], 1e-5, "dzda")
    for k in ("g", "y", "dx", "dQ", "dP", "dalpha"):
        assert_close(got[k], want[k], tol, k)
    check_per_rank(c, got, tol)
    return got, want


def check_per_rank(c, got, tol):
    """The gradients of component k scale with its gate z_k, so an error in a nearly closed component
    is invisible in a whole-tensor measure.  Every open component on its own scale: column k of dP and row k of
    dQ relative to the oracle's own column / row (Frobenius), dlog_alpha_k against the bound that the arithmetic
    gives for a sum of n rounded products, |dzda_k| * ||dg[:, k]|| * ||h[:, k]|| (a plain ratio to the oracle's
    dlog_alpha_k would be meaningless where that sum cancels).  Closed components: exactly zero.
    The gates themselves are held to an absolute 1e-5 (float32 cancels in s (r - l) + l near the threshold), which
    is a large relative error of a gate of 1e-3 and would hide the products' own error here: the oracle is therefore
    evaluated again on the float32 gate values the device computed, so that both sides scale by the same z."""
    z, dzda = got["z"], got["dzda"]
    want = oracle.bwd(c["dy"], c["x"], c["Q"], c["P"], z, dzda)
    open_k = np.flatnonzero(z > 0)
    closed_k = np.flatnonzero(z == 0)
    assert np.all(got["dP"][:, closed_k] == 0) and np.all(got["dQ"][closed_k] == 0) and np.all(got["dalpha"][closed_k] == 0)
    if open_k.size == 0 or c["n"] == 0:
        return
    eps = 1e-300
    ep = np.linalg.norm(got["dP"][:, open_k] - want["dP"][:, open_k], axis=0) / np.maximum(np.linalg.norm(want["dP"][:, open_k], axis=0), eps)
    eq = np.linalg.norm(got["dQ"][open_k] - want["dQ"][open_k], axis=1) / np.maximum(np.linalg.norm(want["dQ"][open_k], axis=1), eps)
    h = c["x"] @ c["Q"][open_k].T
    dg = c["dy"] @ c["P"][:, open_k]
    scale = np.abs(dzda[open_k]) * np.linalg.norm(dg, axis=0) * np.linalg.norm(h, axis=0)
    ea = np.abs(got["dalpha"][open_k] - want["dalpha"][open_k]) / np.maximum(scale, eps)
    ea[scale == 0] = np.abs(got["dalpha"][open_k][scale == 0])
    for name, e in (("dP column", ep), ("dQ row", eq), ("dlog_alpha", ea)):
        worst = int(np.argmax(e))
        assert e[worst] <= tol, f"{name} of component {open_k[worst]} (z = {z[open_k[worst]]:.3e}): {e[worst]:.3e} > {tol:g}"
    small = (z[open_k] < 0.05)
    return int(np.count_nonzero(small))


SHAPES = [
    # n, d, r, dout: tiny; ragged; several tiles + ragged tail; odd leading dimensions; k = 16 cluster-like
    (1, 1, 1, 1),
    (3, 4, 5, 2),
    (200, 96, 80, 136),
    (300, 200, 130, 260),
    (333, 50, 41, 123),
    (129, 16, 16, 1024),
    (520, 264, 136, 72),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_layer_shapes(dtype, shape):
    n, d, r, dout = shape
    c = synth.layer_inputs(100 + n + d, n, d, r, dout, dtype)
    check_layer(c)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_padded_leading_dimensions(dtype):
    c = synth.layer_inputs(321, 150, 72, 40, 88, dtype)
    check_layer(c, pad=8)    # keeps 16-byte alignment: vector path with ld > cols
    check_layer(c, pad=3)    # odd leading dimensions: element-wise path


@pytest.mark.parametrize("shape", [(333, 50, 41, 123), (300, 203, 131, 262), (70, 9, 3, 5), (5, 67, 66, 65)],
                         ids=lambda s: "x".join(map(str, s)))
def test_layer_rows_padded_to_16_bytes(shape):
    # odd extents inside 16-byte aligned rows: asynchronous-transfer kernel with a partial last chunk
    n, d, r, dout = shape
    check_layer(synth.layer_inputs(700 + n + d, n, d, r, dout, "bf16"), align=8)


@pytest.mark.parametrize("dtype,shape,pad", [("f32", (260, 300, 258, 270), 0), ("f32", (257, 1030, 264, 291), 1),
                                             ("f32", (600, 300, 520, 260), 0), ("bf16", (520, 530, 515, 540), 3),
                                             ("bf16", (200, 530, 515, 190), 3)],
                         ids=lambda v: v if isinstance(v, str) else ("x".join(map(str, v)) if isinstance(v, tuple) else f"pad{v}"))
def test_generic_kernel_k_groups(dtype, shape, pad):
    """Few tiles and long contractions on the register-staged kernel (float32; bfloat16 with odd leading
    dimensions): blocks of four k groups on 32x32 tiles whose k steps are split over the wavefronts (launches of up
    to 128 tiles of 64x64), with a ragged last round of the groups."""
    n, d, r, dout = shape
    check_layer(synth.layer_inputs(5200 + n + d, n, d, r, dout, dtype), pad=pad)


@pytest.mark.parametrize("beta", [1.0, 0.5])
def test_layer_other_temperatures(beta):
    c = synth.layer_inputs(55, 70, 48, 64, 40, "f32")
    check_layer(c, beta=beta)


@pytest.mark.parametrize("dtype,shape", [("bf16", (1100, 264, 392, 520)), ("bf16", (300, 75, 130, 41)), ("f32", (260, 96, 200, 72))],
                         ids=lambda v: v if isinstance(v, str) else "x".join(map(str, v)))
def test_nearly_closed_components_on_their_own_scale(dtype, shape):
    """Half of the gates are placed just above the closing threshold (0 < z < 0.05) by choosing log_alpha from
    the drawn noise; their columns of dP, rows of dQ and entries of dlog_alpha are 20 to 1000 times smaller than
    those of open components and are compared on their own scale by check_per_rank."""
    n, d, r, dout = shape
    c = synth.layer_inputs(4300 + n, n, d, r, dout, dtype, 1.0, 2.0)
    t = synth.uniform(4390, (r,), -2.39, -1.96)          # sigmoid(t) * 1.2 - 0.1 lies in (0.0002, 0.048)
    near = np.arange(r) % 2 == 0
    logit_u = np.log(c["u"]) - np.log1p(-c["u"])
    c["log_alpha"] = np.where(near, synth.round_storage(BETA * t - logit_u, "f32"), c["log_alpha"])
    got, want = check_layer(c)
    small = (want["z"] > 0) & (want["z"] < 0.05)
    assert np.count_nonzero(small) >= 0.45 * r
    assert np.max(np.abs(want["dP"][:, small])) < 0.1 * np.max(np.abs(want["dP"]))


def test_config_c1_fp32():
    got, want = check_layer(synth.config_c1())
    closed = float(np.mean(want["z"] == 0))
    assert 0.1 < closed < 0.35
    # closed ranks get exactly zero gradient on the GPU as well
    kz = np.flatnonzero(want["z"] == 0)
    assert np.all(got["dalpha"][kz] == 0) and np.all(got["dP"][:, kz] == 0) and np.all(got["dQ"][kz] == 0)


@pytest.mark.parametrize("layer", [0, 1])
def test_config_c2_bf16_full_size(layer):
    check_layer(synth.config_c2(layer))


def test_config_c2_half_closed_variant():
    c = synth.config_c2(0, closed_half=True)
    got, want = check_layer(c)
    assert 0.4 < float(np.mean(want["z"] == 0)) < 0.6


@pytest.mark.parametrize("matrix", [0, 1, 2, 3])
def test_config_c3_matrices_unpadded(matrix):
    # full token count, unpadded 410-wide rows (820-byte rows are only 4-byte aligned: 4-byte transfers)
    check_layer(synth.config_c3(0, matrix))


@pytest.mark.parametrize("matrix", [0, 1, 2, 3])
def test_config_c3_matrices_padded_rows(matrix):
    # the same matrices in rows padded to 416 / 1232 / 2104 elements (timing layout of this config)
    check_layer(synth.config_c3(1, matrix), align=8)


def test_partial_outputs_and_accumulate():
    c = synth.layer_inputs(9, 90, 40, 56, 72, "f32")
    want = oracle_layer(c)
    got = run_layer(c, grads=("dP",))
    assert_close(got["dP"], want["dP"], 1e-5, "dP only")
    got = run_layer(c, grads=("dx", "dalpha"), accumulate=True)
    assert_close(got["dx"], want["dx"], 1e-5, "dx")
    assert_close(got["dalpha"] - 3.0, want["dalpha"], 2e-5, "dalpha accumulate")


def test_backward_is_deterministic():
    c = synth.config_c2(1)
    a = run_layer(c)
    b = run_layer(c)
    for k in ("y", "dx", "dQ", "dP", "dalpha"):
        assert np.array_equal(a[k], b[k]), k


def test_zero_tokens():
    c = synth.layer_inputs(4, 0, 24, 16, 40, "bf16")
    got = run_layer(c)
    assert got["y"].shape == (0, 40)
    assert np.all(got["dQ"] == 0) and np.all(got["dP"] == 0) and np.all(got["dalpha"] == 0)


# ------------------------------------------------------------------- gates ---
@pytest.mark.parametrize("n", [1, 7, 512, 4099, 26240])
@pytest.mark.parametrize("beta", [1.0, 2.0 / 3.0])
def test_gate_sample_train(n, beta):
    la = synth.normal(11, (n,), 0.0, 4.0)
    u = synth.uniform(12, (n,), 1e-6, 1 - 1e-6)
    z, dzda = torch.empty(n, device=dev()), torch.empty(n, device=dev())
    flop.flop_gate_sample(to_dev(la), to_dev(u), hc_struct(beta), flop.FLOP_GATE_TRAIN, z, dzda)
    zo, dzo = oracle.gate_sample(la, u, beta, L, R)
    zg, dg = to_np(z), to_np(dzda)
    assert np.max(np.abs(zg - zo)) <= 1e-5 and np.max(np.abs(dg - dzo)) <= 1e-5 * max(1.0, dzo.max())
    # away from the clamp points both sides agree on which gates are closed / saturated
    sure = np.abs(np.log(u) - np.log1p(-u) + la - beta * math.log(-L / R)) > 1e-3
    assert np.array_equal((zg == 0)[sure], (zo == 0)[sure])
    assert zg.min() >= 0 and zg.max() <= 1


def test_gate_sample_unaligned_views_and_no_dzda():
    n = 1001
    la = synth.normal(13, (n + 1,), 0.0, 2.0)
    u = synth.uniform(14, (n + 1,), 1e-6, 1 - 1e-6)
    la_d, u_d = to_dev(la)[1:], to_dev(u)[1:]
    z = torch.empty(n + 1, device=dev())[1:]
    flop.flop_gate_sample(la_d, u_d, hc_struct(), flop.FLOP_GATE_TRAIN, z, None)
    zo, _ = oracle.gate_sample(la[1:], u[1:], BETA, L, R)
    assert np.max(np.abs(to_np(z) - zo)) <= 1e-5


def test_gate_sample_deterministic():
    c = synth.config_c4(0.2, n=1, d=8, r=3056, dout=8)
    la = c["log_alpha"]
    z = torch.empty(3056, device=dev())
    flop.flop_gate_sample(to_dev(la), None, hc_struct(), flop.FLOP_GATE_DETERMINISTIC, z, None)
    zo, _ = oracle.gate_sample(la, None, BETA, L, R, deterministic=True)
    zg = to_np(z)
    assert np.max(np.abs(zg - zo)) <= 1e-5
    assert np.array_equal(zg > 0, zo > 0) and int(np.count_nonzero(zg > 0)) == c["keep"] == 611


@pytest.mark.parametrize("beta", [1.0, 2.0 / 3.0])
@pytest.mark.parametrize("n", [5, 3056, 4099])
def test_gate_sample_deterministic_with_slope(n, beta):
    """Deterministic mode with dz/dalpha requested: (r - l) s (1 - s), no temperature, zero outside the clamp."""
    la = synth.normal(15, (n,), 0.0, 6.0)
    z, dzda = torch.full((n,), 9.0, device=dev()), torch.full((n,), 9.0, device=dev())
    flop.flop_gate_sample(to_dev(la), None, hc_struct(beta), flop.FLOP_GATE_DETERMINISTIC, z, dzda)
    zo, dzo = oracle.gate_sample(la, None, beta, L, R, deterministic=True)
    zg, dg = to_np(z), to_np(dzda)
    assert np.max(np.abs(zg - zo)) <= 1e-5 and np.max(np.abs(dg - dzo)) <= 1e-5
    sure = np.minimum(np.abs(la - math.log(-L / R)), np.abs(la - math.log((1 - L) / (R - 1)))) > 1e-3
    assert np.array_equal((dg == 0)[sure], (dzo == 0)[sure])
    if n > 100:
        assert (dzo == 0).any() and (dzo > 0.29).any()
    # exact points: alpha = 0 -> 0.3, alpha = ln 3 -> 0.225, saturated and closed -> 0
    pts = to_dev(np.array([0.0, math.log(3.0), 30.0, -5.0]))
    zz, dd = torch.empty(4, device=dev()), torch.empty(4, device=dev())
    flop.flop_gate_sample(pts, None, hc_struct(beta), flop.FLOP_GATE_DETERMINISTIC, zz, dd)
    assert np.max(np.abs(to_np(dd) - np.array([0.3, 0.225, 0.0, 0.0]))) <= 1e-5
    assert np.max(np.abs(to_np(zz) - np.array([0.5, 0.8, 1.0, 0.0]))) <= 1e-5


def test_gate_sample_noise_at_range_ends():
    """u = 0 and u = 1: closed and saturated gates with zero slope on both sides, no NaN."""
    la = np.array([-3.0, 0.0, 25.0, -25.0, 0.0, 3.0, 0.5, 0.5])
    u = np.array([0.0, 0.0, 0.0, 1.0, 1.0, 1.0, 0.0, 1.0])
    z, dzda = torch.empty(8, device=dev()), torch.empty(8, device=dev())
    flop.flop_gate_sample(to_dev(la), to_dev(u), hc_struct(), flop.FLOP_GATE_TRAIN, z, dzda)
    zo, dzo = oracle.gate_sample(la, u, BETA, L, R)
    assert np.array_equal(to_np(z), zo) and np.array_equal(to_np(dzda), dzo)
    assert zo.tolist() == [0, 0, 0, 1, 1, 1, 0, 1]


# ------------------------------------------------------------- expected L0 ---
@pytest.mark.parametrize("n", [1, 512, 1536, 26240, 300001])
@pytest.mark.parametrize("weighted", [False, True])
def test_expected_l0(n, weighted):
    la = synth.normal(21, (n,), 0.0, 1.5)
    w = synth.uniform(22, (n,), 800.0, 4200.0) if weighted else None
    out = torch.empty(1, device=dev())
    grad = torch.empty(n, device=dev())
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, n, 0, 0, 0), dev())
    flop.flop_expected_l0(to_dev(la), hc_struct(), out, None if w is None else to_dev(w), grad, ws)
    so, go = oracle.expected_l0(la, BETA, L, R, w)
    assert abs(float(out.item()) - so) / so <= 1e-5
    assert_close(grad, go, 1e-5, "l0 grad")


@pytest.mark.parametrize("n", [1, 1536, 4096, 26240])
def test_gates_and_expected_l0_in_one_call(n):
    la = synth.normal(31, (n,), 1.0, 2.0)
    u = synth.uniform(32, (n,), 1e-6, 1.0 - 1e-6)
    w = np.floor(synth.uniform(33, (n,), 800.0, 4200.0))
    z, dzda, grad = (torch.full((n,), 7.0, device=dev()) for _ in range(3))
    out = torch.empty(1, device=dev())
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, n, 0, 0, 0), dev())
    flop.flop_gate_sample_l0(to_dev(la), to_dev(u), hc_struct(), z, dzda, out, to_dev(w), grad, ws)
    zo, dzo = oracle.gate_sample(la, u, BETA, L, R)
    so, go = oracle.expected_l0(la, BETA, L, R, w)
    assert_close(z, zo, 1e-5, "z")
    assert_close(dzda, dzo, 1e-5, "dzda")
    assert abs(float(out.item()) - so) / so <= 1e-5
    assert_close(grad, go, 1e-5, "l0 grad")


def test_expected_l0_c1_value_and_empty():
    out = torch.empty(1, device=dev())
    flop.flop_expected_l0(torch.zeros(512, device=dev()), hc_struct(), out)
    assert abs(float(out.item()) - 425.8929582) / 425.8929582 <= 1e-5
    flop.flop_expected_l0(torch.zeros(0, device=dev()), hc_struct(), out)
    assert float(out.item()) == 0.0


# -------------------------------------------------------------- compaction ---
def run_compact(z64, Q64, P64, dtype, absorb=False, pad=0):
    r, d = Q64.shape
    dout = P64.shape[0]
    z = to_dev(z64)
    Q, P = to_dev(Q64, dtype), to_dev(P64, dtype)
    tdt = TORCH_DT[dtype]
    r_out = torch.full((1,), -1, dtype=torch.int32, device=dev())
    idx = torch.full((max(r, 1),), -1, dtype=torch.int32, device=dev())[:r]
    Qc = torch.full((r, d + pad), 9.0, dtype=tdt, device=dev())[:, :d]
    Pc = torch.full((dout, r + pad), 9.0, dtype=tdt, device=dev())[:, :r]
    zc = torch.full((max(r, 1),), 9.0, dtype=torch.float32, device=dev())[:r]
    flop.flop_compact(z, Q, P, r_out, idx, Qc, Pc, zc, absorb_z_into_Q=absorb)
    torch.cuda.synchronize()
    return int(r_out.item()), to_np(idx).astype(np.int64), to_np(Qc), to_np(Pc), to_np(zc)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", ["random", "none", "all", "one", "big"])
def test_compact_bit_exact(dtype, case):
    r, d, dout = (3056, 72, 40) if case == "big" else (203, 50, 37)
    Q = synth.normal(31, (r, d), 0, 1, dtype)
    P = synth.normal(32, (dout, r), 0, 1, dtype)
    z = np.clip(synth.uniform(33, (r,), -1.0, 1.0), 0.0, 1.0)
    if case == "none":
        z[:] = 0.0
    elif case == "all":
        z[:] = 0.25
    elif case == "one":
        z[:] = 0.0
        z[r - 1] = 1.0
    rp, idx, Qc, Pc, zc = run_compact(z, Q, P, dtype)
    idx_o, Qo, Po, zo = oracle.compact(z, Q, P)
    assert rp == len(idx_o)
    assert np.array_equal(idx[:rp], idx_o)
    assert np.array_equal(Qc[:rp], Qo) and np.array_equal(Pc[:, :rp], Po) and np.array_equal(zc[:rp], zo)
    pad = min(r, (rp + 31) // 32 * 32)
    assert np.all(Qc[rp:pad] == 0) and np.all(Pc[:, rp:pad] == 0) and np.all(zc[rp:pad] == 0)
    # beyond the pad nothing is written
    assert np.all(Qc[pad:] == 9.0) and np.all(Pc[:, pad:] == 9.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compact_absorb_and_unaligned(dtype):
    r, d, dout = 130, 43, 21
    Q = synth.normal(34, (r, d), 0, 1, dtype)
    P = synth.normal(35, (dout, r), 0, 1, dtype)
    z = np.clip(synth.uniform(36, (r,), -0.5, 1.0), 0.0, 1.0)
    rp, idx, Qc, Pc, zc = run_compact(z, Q, P, dtype, absorb=True, pad=5)
    idx_o, Qo, Po, zo = oracle.compact(z, Q, P, absorb=True)
    assert np.array_equal(idx[:rp], idx_o) and np.array_equal(Pc[:, :rp], Po) and np.array_equal(zc[:rp], zo)
    assert_close(Qc[:rp], Qo, 1e-6 if dtype == "f32" else 2.0 ** -8, "absorbed Q")


def test_compact_threshold_self_consistency():
    # log_alpha exactly at, and one float32 step either side of, log(-l/r): whatever z the
    # library computes, its own keep decision must be z > 0 on that stored value.
    thr = np.float32(math.log(-L / R))
    la = np.array([thr, np.nextafter(thr, np.float32(1)), np.nextafter(thr, np.float32(-10)), 0.0, -30.0],
                  dtype=np.float32)
    z = torch.empty(5, device=dev())
    flop.flop_gate_sample(to_dev(la), None, hc_struct(), flop.FLOP_GATE_DETERMINISTIC, z, None)
    Q = to_dev(np.ones((5, 8)))
    P = to_dev(np.ones((8, 5)))
    r_out = torch.empty(1, dtype=torch.int32, device=dev())
    idx = torch.empty(5, dtype=torch.int32, device=dev())
    flop.flop_compact(z, Q, P, r_out, idx)
    zg = to_np(z)
    assert to_np(idx)[: int(r_out.item())].astype(int).tolist() == np.flatnonzero(zg > 0).tolist()


@pytest.mark.parametrize("frac", [0.1, 0.2, 0.35])
def test_config_c4_compacted_inference(frac):
    """Full-size recurrent-LM projection: gate -> compact -> forward on P', Q'.

    Indices, P', Q' bit for bit; every row of y against the oracle, in blocks of 1024 token rows (rows of y
    are independent), each block held to the tolerance on its own."""
    c = synth.config_c4(frac)
    n, d, r, dout = c["n"], c["d"], c["r"], c["dout"]
    x, Q, P = to_dev(c["x"], "bf16"), to_dev(c["Q"], "bf16"), to_dev(c["P"], "bf16")
    la = to_dev(c["log_alpha"])
    z = torch.empty(r, device=dev())
    flop.flop_gate_sample(la, None, hc_struct(), flop.FLOP_GATE_DETERMINISTIC, z, None)
    r_out = torch.empty(1, dtype=torch.int32, device=dev())
    idx = torch.empty(r, dtype=torch.int32, device=dev())
    Qc = torch.empty(r, d, dtype=torch.bfloat16, device=dev())
    Pc = torch.empty(dout, r, dtype=torch.bfloat16, device=dev())
    zc = torch.empty(r, device=dev())
    flop.flop_compact(z, Q, P, r_out, idx, Qc, Pc, zc)
    rp = int(r_out.item())
    assert rp == c["keep"] == int(round(frac * r))
    g = torch.empty(n, rp, dtype=torch.bfloat16, device=dev())
    y = torch.empty(n, dout, dtype=torch.bfloat16, device=dev())
    flop.flop_fwd(x, Qc[:rp], Pc[:, :rp], zc[:rp], g, y)
    torch.cuda.synchronize()

    zo, _ = oracle.gate_sample(c["log_alpha"], None, BETA, L, R, deterministic=True)
    idx_o, Qo, Po, zco = oracle.compact(zo, c["Q"], c["P"])
    assert np.array_equal(to_np(idx[:rp]).astype(np.int64), idx_o)
    assert np.array_equal(to_np(Qc[:rp]), Qo) and np.array_equal(to_np(Pc[:, :rp]), Po)
    for r0 in range(0, n, 1024):
        _, go, yo = oracle.fwd(c["x"][r0:r0 + 1024], Qo, Po, zco)
        assert_close(to_np(g[r0:r0 + 1024]), go, 2e-2, f"g (compacted) rows {r0}..")
        assert_close(to_np(y[r0:r0 + 1024]), yo, 2e-2, f"y (compacted) rows {r0}..")
    # closing == deleting: the dense gated layer gives the same rows
    rows = synth.permutation(4099, n)[:48]
    _, _, yo = oracle.fwd(c["x"][rows], Qo, Po, zco)
    _, _, y_dense = oracle.fwd(c["x"][rows], c["Q"], c["P"], zo)
    np.testing.assert_allclose(yo, y_dense, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------ error returns ---
def test_error_statuses_do_not_launch():
    x = torch.zeros(4, 8, device=dev())
    Q = torch.zeros(6, 8, device=dev())
    P = torch.zeros(5, 6, device=dev())
    z = torch.zeros(6, device=dev())
    g = torch.zeros(4, 6, device=dev())
    y = torch.zeros(4, 5, device=dev())
    with pytest.raises(flop.FlopError) as e:
        flop.flop_gate_sample(z, z, flop.flop_hc(0.5, 0.1, 1.1), flop.FLOP_GATE_TRAIN, z)
    assert e.value.status == -5
    with pytest.raises(flop.FlopError) as e:
        flop.flop_gate_sample(z, None, hc_struct(), flop.FLOP_GATE_TRAIN, z)
    assert e.value.status == -1
    with pytest.raises(flop.FlopError) as e:
        flop.flop_bwd(y, x, Q, P, z, z, g, x.clone(), None, None, None, None)
    assert e.value.status == -6
    L_ = flop.lib()
    import ctypes
    rc = L_.flop_fwd(0, 4, 8, 6, 5, x.data_ptr(), 7, Q.data_ptr(), 8, P.data_ptr(), 6, z.data_ptr(),
                     g.data_ptr(), 6, y.data_ptr(), 5, None, 0, None)
    assert rc == -3
    rc = L_.flop_fwd(7, 4, 8, 6, 5, x.data_ptr(), 8, Q.data_ptr(), 8, P.data_ptr(), 6, z.data_ptr(),
                     g.data_ptr(), 6, y.data_ptr(), 5, None, 0, None)
    assert rc == -4
    torch.cuda.synchronize()


# ----------------------------------------------------------- gate gradient ---
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1), (33, 7), (300, 130), (2048, 768)], ids=str)
def test_gate_grad_standalone(dtype, shape):
    """flop_gate_grad on dh = dg*z and g = h*z equals the oracle's dz * dzda."""
    n, r = shape
    c = synth.layer_inputs(700 + n, n, 24, r, 16, dtype)
    z, dzda = oracle.gate_sample(c["log_alpha"], c["u"], BETA, L, R)
    h, g, _ = oracle.fwd(c["x"], c["Q"], c["P"], z)
    want = oracle.bwd(c["dy"], c["x"], c["Q"], c["P"], z, dzda)
    dg = c["dy"] @ c["P"]
    dh64, g64 = synth.round_storage(dg * z, dtype), synth.round_storage(g, dtype)
    da = torch.full((r,), 2.0, device=dev())
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_GATE_GRAD, flop._dt(to_dev(g64, dtype)), n, 0, r, 0), dev())
    flop.flop_gate_grad(to_dev(dh64, dtype), to_dev(g64, dtype), to_dev(z), to_dev(dzda), da, ws, accumulate=True)
    assert_close(to_np(da) - 2.0, want["dalpha"], TOL[dtype] if dtype == "bf16" else 2e-5, "dlog_alpha")


@pytest.mark.parametrize("dtype,n,r,ld", [("bf16", 130, 2056, 2056), ("bf16", 70, 2051, 2056), ("f32", 37, 1030, 1032),
                                          ("f32", 300, 1024, 1024), ("bf16", 16500, 2048, 2048)],
                         ids=lambda v: str(v))
def test_gate_grad_long_rows(dtype, n, r, ld):
    """Long rows in 16-byte aligned storage through the column-sum kernel: many block columns, whole and partial last
    column groups (row length not a multiple of 16 bytes inside padded rows), chunks of 32 and (from 16384 rows) 128
    rows with ragged last chunks."""
    c = synth.layer_inputs(760 + n, n, 24, r, 16, dtype)
    z, dzda = oracle.gate_sample(c["log_alpha"], c["u"], BETA, L, R)
    h, g, _ = oracle.fwd(c["x"], c["Q"], c["P"], z)
    want = oracle.bwd(c["dy"], c["x"], c["Q"], c["P"], z, dzda)
    dg = c["dy"] @ c["P"]
    dh64, g64 = synth.round_storage(dg * z, dtype), synth.round_storage(g, dtype)
    dh_t, g_t = padded(to_dev(dh64, dtype), ld), padded(to_dev(g64, dtype), ld)
    da = torch.full((r,), float("nan"), device=dev())
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_GATE_GRAD, flop._dt(g_t), n, 0, r, 0), dev())
    flop.flop_gate_grad(dh_t, g_t, to_dev(z), to_dev(dzda), da, ws)
    assert_close(to_np(da), want["dalpha"], TOL[dtype] if dtype == "bf16" else 2e-5, "dlog_alpha")


# ------------------------------------------------- tied adaptive softmax side ---
def test_tied_softmax_cluster_shapes():
    """Section 4.2 on the output side: the logits of a vocabulary cluster are a gated
    factorized layer with Q = O_c (rank = cluster width) and P = E_c (one row per word),
    i.e. a very wide, very low-rank layer: 200,000 outputs at rank 64."""
    # forward + backward, all outputs, at a token count the oracle finishes in seconds
    c = synth.layer_inputs(8100, 384, 1024, 64, 200000, "bf16", 0.5, 1.0)
    check_layer(c)
    # forward at the full batch: every row of the logits, in blocks of 256 token rows
    n = 8192
    big = synth.layer_inputs(8200, n, 1024, 64, 1000, "bf16", 0.5, 1.0)   # x, Q, gates; P below
    P = c["P"]
    x, Q, Pd = to_dev(big["x"], "bf16"), to_dev(big["Q"], "bf16"), to_dev(P, "bf16")
    z, _ = oracle.gate_sample(big["log_alpha"], big["u"], BETA, L, R)
    g = torch.empty(n, 64, dtype=torch.bfloat16, device=dev())
    y = torch.empty(n, 200000, dtype=torch.bfloat16, device=dev())
    flop.flop_fwd(x, Q, Pd, to_dev(z), g, y)
    torch.cuda.synchronize()
    for r0 in range(0, n, 256):
        _, _, yo = oracle.fwd(big["x"][r0:r0 + 256], big["Q"], P, z)
        assert_close(to_np(y[r0:r0 + 256]), yo, 2e-2, f"logits rows {r0}..")


def test_operand_beyond_two_gib():
    """Backward pass with a 2.25 GB gradient of the logits (5632 x 200000 bf16): the contraction kernel's
    buffer descriptors span less than 2 GiB, so dy P addresses dy tile by tile and dy^T g is cut along the
    tokens.  Rows of dx and rows of dP are independent of one another: the oracle computes sampled ones
    from the matching sub-problems (sampled tokens; sampled words with every token)."""
    n, d, r, dout = 5632, 1024, 64, 200000
    small = synth.layer_inputs(8400, n, d, r, 8, "bf16", 0.5, 1.0)            # x, Q, gates
    P = synth.normal(8410, (dout, r), 0.0, 1.0 / r, "bf16")
    dy_dev = torch.empty(n, dout, dtype=torch.bfloat16, device=dev())
    rows = sorted(set([0, 5368, 5369, n - 1] + [int(v) for v in synth.permutation(8411, n)[:20]]))
    cols = sorted(set([0, 1, dout - 1] + [int(v) for v in synth.permutation(8412, dout)[:21]]))
    dy_rows, dy_cols = {}, []
    for i, r0 in enumerate(range(0, n, 512)):                                  # 512 rows at a time
        chunk = synth.normal(8420 + i, (512, dout), 0.0, 1.0, "bf16")
        dy_dev[r0:r0 + 512] = to_dev(chunk, "bf16")
        dy_cols.append(chunk[:, cols].copy())
        for rr in rows:
            if r0 <= rr < r0 + 512:
                dy_rows[rr] = chunk[rr - r0].copy()
        del chunk
    dy_cols = np.concatenate(dy_cols, axis=0)
    z, dzda = oracle.gate_sample(small["log_alpha"], small["u"], BETA, L, R)
    x, Q, Pd = to_dev(small["x"], "bf16"), to_dev(small["Q"], "bf16"), to_dev(P, "bf16")
    g = torch.empty(n, r, dtype=torch.bfloat16, device=dev())
    y8 = torch.empty(n, 8, dtype=torch.bfloat16, device=dev())
    flop.flop_fwd(x, Q, Pd[:8], to_dev(z), g, y8)                              # g = (x Q^T) z, saved for the backward
    dx, dQ, dP = torch.empty_like(x), torch.empty_like(Q), torch.empty_like(Pd)
    da = torch.empty(r, device=dev())
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop.FLOP_BF16, n, d, r, dout), dev())
    flop.flop_bwd(dy_dev, x, Q, Pd, to_dev(z), to_dev(dzda), g, dx, dQ, dP, da, ws)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(to_np(dQ))) and np.all(np.isfinite(to_np(da)))
    sub = oracle.bwd(np.stack([dy_rows[rr] for rr in rows]), small["x"][rows], small["Q"], P, z, dzda)
    assert_close(to_np(dx[torch.tensor(rows, device=dev())]), sub["dx"], 2e-2, "dx (sampled tokens)")
    sub = oracle.bwd(dy_cols, small["x"], small["Q"], P[cols], z, dzda)
    assert_close(to_np(dP[torch.tensor(cols, device=dev())]), sub["dP"], 2e-2, "dP (sampled words)")


# ------------------------------------------------ few tiles, long contraction ---
@pytest.mark.parametrize("shape", [(8192, 128, 64, 128), (256, 8200, 64, 4104), (4100, 72, 40, 8192)],
                         ids=lambda s: "x".join(map(str, s)))
def test_k_split_products(shape):
    """Products with a handful of output tiles and thousands of k steps are cut along k and
    added up by a second kernel (weight gradients at large batch, wide inputs at low rank)."""
    n, d, r, dout = shape
    c = synth.layer_inputs(8300 + n, n, d, r, dout, "bf16")
    want = oracle_layer(c)
    x, Q, P, dy = (to_dev(c[k], "bf16") for k in ("x", "Q", "P", "dy"))
    z, dzda = to_dev(want["z"]), to_dev(want["dzda"])
    g = torch.full((n, r), 5.0, dtype=torch.bfloat16, device=dev())
    y = torch.full((n, dout), 5.0, dtype=torch.bfloat16, device=dev())
    fbytes = flop.flop_workspace_bytes(flop.FLOP_OP_FWD, flop.FLOP_BF16, n, d, r, dout)
    bbytes = flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop.FLOP_BF16, n, d, r, dout)
    plain = flop.flop_workspace_bytes(flop.FLOP_OP_GATE_GRAD, flop.FLOP_BF16, n, 0, r, 0)
    assert fbytes > 0 or bbytes > plain + n * r * 2 + 512, "shape does not exercise the split"
    flop.flop_fwd(x, Q, P, z, g, y, flop.workspace(fbytes, dev()))
    dx, dQ, dP = torch.empty_like(x), torch.empty_like(Q), torch.empty_like(P)
    da = torch.empty(r, device=dev())
    flop.flop_bwd(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da, flop.workspace(bbytes, dev()))
    torch.cuda.synchronize()
    for k, t in (("g", g), ("y", y), ("dx", dx), ("dQ", dQ), ("dP", dP), ("dalpha", da)):
        assert_close(to_np(t), want[k], 2e-2, k)
    # same results without the optional forward workspace (single launches)
    g2, y2 = torch.empty_like(g), torch.empty_like(y)
    flop.flop_fwd(x, Q, P, z, g2, y2)
    torch.cuda.synchronize()
    assert_close(to_np(y2), want["y"], 2e-2, "y (no workspace)")


# ---------------------------------------- gate gradients of several layers in one launch ---
def test_deferred_gate_gradient_finish():
    """flop_bwd_deferred leaves the last stage of the gate gradient to flop_gate_grad_finish, which serves many
    layers with one launch: 18 layers of mixed shapes and types (column sums from the product's epilogue, from the
    reduction kernel, float32) - more than one launch holds - against the oracle and, bit for bit, against
    flop_bwd; the third layer accumulates."""
    shapes = [(300, 200, 130, 260, "bf16"), (333, 50, 41, 123, "bf16"), (256, 64, 96, 64, "f32"), (130, 72, 40, 24, "bf16")]
    layers, pend = [], []
    for i in range(18):
        n, d, r, dout, dt = shapes[i % 4]
        c = synth.layer_inputs(8600 + 10 * i, n, d, r, dout, dt)
        want = oracle_layer(c)
        x, Q, P, dy = (to_dev(c[k], dt) for k in ("x", "Q", "P", "dy"))
        z, dzda = to_dev(want["z"]), to_dev(want["dzda"])
        g = torch.empty(n, r, dtype=TORCH_DT[dt], device=dev())
        y = torch.empty(n, dout, dtype=TORCH_DT[dt], device=dev())
        flop.flop_fwd(x, Q, P, z, g, y)
        acc = i == 2
        start = 0.5 if acc else float("nan")
        da_ref = torch.full((r,), start, device=dev())
        da = torch.full((r,), start, device=dev())
        dx, dQ, dP = torch.empty_like(x), torch.empty_like(Q), torch.empty_like(P)
        wbytes = flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(x), n, d, r, dout)
        flop.flop_bwd(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da_ref, flop.workspace(wbytes, dev()), accumulate=acc)
        ws = flop.workspace(wbytes, dev())
        pend.append(flop.flop_bwd_deferred(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da, ws, accumulate=acc))
        layers.append(dict(want=want, da=da, da_ref=da_ref, ws=ws, keep=(x, Q, P, dy, z, dzda, g), dt=dt, acc=acc, dx=dx))
    torch.cuda.synchronize()
    assert all(np.isnan(to_np(l["da"])).all() for l in layers if not l["acc"]), "deferred call must not write dlog_alpha"
    flop.flop_gate_grad_finish(pend)
    torch.cuda.synchronize()
    for l in layers:
        assert np.array_equal(to_np(l["da"]), to_np(l["da_ref"]))
        assert_close(to_np(l["da"]) - (0.5 if l["acc"] else 0.0), l["want"]["dalpha"], TOL[l["dt"]] * (4 if l["acc"] else 1), "dalpha")
        assert_close(l["dx"], l["want"]["dx"], TOL[l["dt"]], "dx")


@pytest.mark.parametrize("layers,n_gates", [(3, 1000), (16, 4096), (18, 700), (2, 5000)])
def test_step_boundary(layers, n_gates):
    """flop_step_boundary = flop_gate_grad_finish for the ending step + flop_gate_sample_l0 for the next one: gate
    gradients bit for bit against flop_bwd, new gates and the Eq.(3) sum against the oracle and against the separate
    call; 18 layers / 5000 gates are beyond what the single launch holds and take the two-launch route. New gates
    written into a buffer the pending layers still read are refused."""
    shapes = [(300, 200, 130, 260, "bf16"), (256, 64, 96, 64, "f32"), (130, 72, 40, 24, "bf16")]
    items, pend = [], []
    for i in range(layers):
        n, d, r, dout, dt = shapes[i % 3]
        c = synth.layer_inputs(8700 + 10 * i, n, d, r, dout, dt)
        want = oracle_layer(c)
        x, Q, P, dy = (to_dev(c[k], dt) for k in ("x", "Q", "P", "dy"))
        z, dzda = to_dev(want["z"]), to_dev(want["dzda"])
        g = torch.empty(n, r, dtype=TORCH_DT[dt], device=dev())
        y = torch.empty(n, dout, dtype=TORCH_DT[dt], device=dev())
        flop.flop_fwd(x, Q, P, z, g, y)
        da_ref, da = torch.full((r,), float("nan"), device=dev()), torch.full((r,), float("nan"), device=dev())
        dx, dQ, dP = torch.empty_like(x), torch.empty_like(Q), torch.empty_like(P)
        wbytes = flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(x), n, d, r, dout)
        flop.flop_bwd(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da_ref, flop.workspace(wbytes, dev()))
        ws = flop.workspace(wbytes, dev())
        pend.append(flop.flop_bwd_deferred(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da, ws))
        items.append(dict(want=want, da=da, da_ref=da_ref, dt=dt, keep=(x, Q, P, dy, z, dzda, g, ws)))
    rng = np.random.default_rng(8800 + n_gates)
    la = rng.normal(0.0, 2.0, n_gates).astype(np.float32)
    u = rng.uniform(1e-6, 1 - 1e-6, n_gates).astype(np.float32)
    w = rng.uniform(1.0, 900.0, n_gates).astype(np.float32)
    la_d, u_d, w_d = to_dev(la), to_dev(u), to_dev(w)
    new = lambda: (torch.full((n_gates,), float("nan"), device=dev()), torch.full((n_gates,), float("nan"), device=dev()),
                   torch.full((1,), float("nan"), device=dev()), torch.full((n_gates,), float("nan"), device=dev()))
    z2, dzda2, l0, l0g = new()
    gws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, n_gates, 0, 0, 0), dev())
    first = items[0]["keep"]
    with pytest.raises(flop.FlopError) as e:                     # z of the next step over the z layer 0 still reads
        flop.flop_step_boundary(pend, la_d[: first[4].numel()], u_d[: first[4].numel()], hc_struct(), first[4],
                                dzda2[: first[4].numel()], l0, w=w_d[: first[4].numel()], ws=gws)
    assert e.value.status == -9
    flop.flop_step_boundary(pend, la_d, u_d, hc_struct(), z2, dzda2, l0, w=w_d, l0_grad=l0g, ws=gws)
    z3, dzda3, l03, l0g3 = new()
    flop.flop_gate_sample_l0(la_d, u_d, hc_struct(), z3, dzda3, l03, w=w_d, l0_grad=l0g3, ws=gws)
    torch.cuda.synchronize()
    for l in items:
        assert np.array_equal(to_np(l["da"]), to_np(l["da_ref"]))
        assert_close(l["da"], l["want"]["dalpha"], TOL[l["dt"]], "dalpha")
    zo, dzo = oracle.gate_sample(la.astype(np.float64), u.astype(np.float64), BETA, L, R)
    assert np.array_equal(to_np(z2), to_np(z3)) and np.array_equal(to_np(dzda2), to_np(dzda3))
    assert np.array_equal(to_np(l0g), to_np(l0g3))
    assert_close(z2, zo, 1e-5, "z")
    want_l0, want_grad = oracle.expected_l0(la.astype(np.float64), BETA, L, R, w.astype(np.float64))
    assert_close(l0g, want_grad, 1e-5, "l0_grad")
    assert abs(float(l0.item()) - want_l0) <= 1e-5 * abs(want_l0)
    assert abs(float(l03.item()) - want_l0) <= 1e-5 * abs(want_l0)


@pytest.mark.parametrize("case", ["fused", "word_rows", "f32", "odd_rows", "many_gates", "no_tokens"])
def test_fwd_sampling(case):
    """flop_fwd_sampling = flop_gate_sample_l0 over the model's gates + flop_fwd of the layer at gate_offset: g and
    y bit for bit against flop_fwd with separately sampled gates, the gates bit for bit against flop_gate_sample,
    Eq.(3) against the oracle.  'fused' and 'word_rows' (rows only 4-byte aligned) compute the gates in the first
    product's epilogue; float32, odd leading dimensions, more than 4096 gates and an empty batch take the
    separate gate launch."""
    dt = "f32" if case == "f32" else "bf16"
    n, d, r, dout = {"fused": (300, 200, 136, 264), "word_rows": (300, 202, 134, 262), "f32": (200, 96, 80, 136),
                     "odd_rows": (300, 203, 131, 263), "many_gates": (300, 200, 136, 264), "no_tokens": (0, 24, 16, 40)}[case]
    off = 40
    n_gates = 5000 if case == "many_gates" else off + r + 25
    c = synth.layer_inputs(9100 + r, n, d, r, dout, dt)
    rng = np.random.default_rng(9100 + n_gates)
    la = rng.normal(0.0, 2.0, n_gates).astype(np.float32)
    u = rng.uniform(1e-6, 1 - 1e-6, n_gates).astype(np.float32)
    w = rng.uniform(1.0, 900.0, n_gates).astype(np.float32)
    la[off:off + r], u[off:off + r] = c["log_alpha"], c["u"]
    x, Q, P = (to_dev(c[k], dt) for k in ("x", "Q", "P"))
    la_d, u_d, w_d = to_dev(la), to_dev(u), to_dev(w)
    nan = lambda k: torch.full((k,), float("nan"), device=dev())
    z_ref, dz_ref = nan(n_gates), nan(n_gates)
    flop.flop_gate_sample(la_d, u_d, hc_struct(), flop.FLOP_GATE_TRAIN, z_ref, dz_ref)
    tdt = TORCH_DT[dt]
    g_ref, y_ref = torch.zeros(n, r, dtype=tdt, device=dev()), torch.zeros(n, dout, dtype=tdt, device=dev())
    flop.flop_fwd(x, Q, P, z_ref[off:off + r], g_ref, y_ref)
    z, dzda, l0, l0g = nan(n_gates), nan(n_gates), nan(1), nan(n_gates)
    g, y = torch.zeros(n, r, dtype=tdt, device=dev()), torch.zeros(n, dout, dtype=tdt, device=dev())
    gws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, n_gates, 0, 0, 0), dev())
    with pytest.raises(flop.FlopError) as e:      # the layer's gates must lie inside the model's
        flop.flop_fwd_sampling(x, Q, P, la_d, u_d, hc_struct(), z, dzda, l0, n_gates - r + 1, g, y)
    assert e.value.status == -2
    flop.flop_trace_begin(8)
    flop.flop_fwd_sampling(x, Q, P, la_d, u_d, hc_struct(), z, dzda, l0, off, g, y, w=w_d, l0_grad=l0g, l0_ws=gws)
    torch.cuda.synchronize()
    launches = flop.flop_trace_end(8)
    assert len(launches) == (0 if n == 0 else 2)
    assert np.array_equal(to_np(z), to_np(z_ref)) and np.array_equal(to_np(dzda), to_np(dz_ref))
    assert np.array_equal(to_np(g), to_np(g_ref)) and np.array_equal(to_np(y), to_np(y_ref))
    want_l0, want_grad = oracle.expected_l0(la.astype(np.float64), BETA, L, R, w.astype(np.float64))
    assert_close(l0g, want_grad, 1e-5, "l0_grad")
    assert abs(float(l0.item()) - want_l0) <= 1e-5 * abs(want_l0)
    if n:
        want = oracle_layer(c)
        assert_close(g, want["g"], TOL[dt], "g")
        assert_close(y, want["y"], TOL[dt], "y")


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_bwd_boundary_finish_only(dt):
    """A job without gates: only the gate gradients of the earlier layer and of this one are finished (on the last
    contraction launch for bfloat16, by a launch of their own for float32); bit for bit against flop_bwd."""
    ls = []
    for i, (n, d, r, dout) in enumerate([(130, 72, 40, 24), (300, 200, 136, 264)]):
        c = synth.layer_inputs(8970 + i, n, d, r, dout, dt)
        want = oracle_layer(c)
        x, Q, P, dy = (to_dev(c[k], dt) for k in ("x", "Q", "P", "dy"))
        z, dzda = to_dev(want["z"]), to_dev(want["dzda"])
        g = torch.empty(n, r, dtype=TORCH_DT[dt], device=dev())
        flop.flop_fwd(x, Q, P, z, g, torch.empty(n, dout, dtype=TORCH_DT[dt], device=dev()))
        wbytes = flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(x), n, d, r, dout)
        da_ref, da = torch.full((r,), float("nan"), device=dev()), torch.full((r,), float("nan"), device=dev())
        ref = (torch.empty_like(x), torch.empty_like(Q), torch.empty_like(P))
        flop.flop_bwd(dy, x, Q, P, z, dzda, g, *ref, da_ref, flop.workspace(wbytes, dev()))
        ls.append(dict(a=(dy, x, Q, P, z, dzda, g), out=(torch.empty_like(x), torch.empty_like(Q), torch.empty_like(P)),
                       da=da, da_ref=da_ref, ref=ref, ws=flop.workspace(wbytes, dev()), want=want))
    first, last = ls
    pend = [flop.flop_bwd_deferred(*first["a"], *first["out"], first["da"], first["ws"])]
    flop.flop_bwd_boundary(*last["a"], *last["out"], last["da"], last["ws"], pend)
    torch.cuda.synchronize()
    for l in ls:
        assert np.array_equal(to_np(l["da"]), to_np(l["da_ref"]))
        assert_close(l["da"], l["want"]["dalpha"], TOL[dt], "dalpha")
        for got, ref in zip(l["out"], l["ref"]):
            assert np.array_equal(to_np(got), to_np(ref))


@pytest.mark.parametrize("case", ["rides", "f32", "odd_rows", "no_dx", "seventeen", "many_gates"])
def test_bwd_boundary(case):
    """flop_bwd_boundary = flop_bwd_deferred of the last layer + flop_step_boundary: gradients of the layer bit for
    bit against flop_bwd, gate gradients of the earlier layers against flop_bwd, new gates and Eq.(3) against the
    oracle.  'rides': bfloat16 with aligned rows, the boundary goes along with the last contraction launch; the
    other cases take the separate launches (float32, rows without 16-byte alignment, no phase-2 product, more than
    sixteen gate vectors, more than 4096 new gates)."""
    dt = "f32" if case == "f32" else "bf16"
    n_prev = 17 if case == "seventeen" else 2
    n_gates = 5000 if case == "many_gates" else 1536
    shapes = [(300, 200, 136, 264), (130, 72, 40, 24)]
    if case == "odd_rows":
        shapes = [(300, 203, 131, 262), (130, 72, 40, 24)]
    prev, pend = [], []
    def make(i, n, d, r, dout):
        c = synth.layer_inputs(8950 + 10 * i, n, d, r, dout, dt)
        want = oracle_layer(c)
        x, Q, P, dy = (to_dev(c[k], dt) for k in ("x", "Q", "P", "dy"))
        z, dzda = to_dev(want["z"]), to_dev(want["dzda"])
        g = torch.empty(n, r, dtype=TORCH_DT[dt], device=dev())
        y = torch.empty(n, dout, dtype=TORCH_DT[dt], device=dev())
        flop.flop_fwd(x, Q, P, z, g, y)
        da_ref, da = torch.full((r,), float("nan"), device=dev()), torch.full((r,), float("nan"), device=dev())
        bufs = lambda: (torch.empty_like(x), torch.empty_like(Q), torch.empty_like(P))
        wbytes = flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(x), n, d, r, dout)
        ref = bufs()
        flop.flop_bwd(dy, x, Q, P, z, dzda, g, *ref, da_ref, flop.workspace(wbytes, dev()))
        return dict(want=want, x=x, Q=Q, P=P, dy=dy, z=z, dzda=dzda, g=g, da=da, da_ref=da_ref, ref=ref, out=bufs(),
                    ws=flop.workspace(wbytes, dev()))
    for i in range(n_prev):
        l = make(i, *shapes[1])
        pend.append(flop.flop_bwd_deferred(l["dy"], l["x"], l["Q"], l["P"], l["z"], l["dzda"], l["g"], *l["out"], l["da"], l["ws"]))
        prev.append(l)
    last = make(99, *shapes[0])
    rng = np.random.default_rng(8990 + n_gates)
    la = rng.normal(0.0, 2.0, n_gates).astype(np.float32)
    u = rng.uniform(1e-6, 1 - 1e-6, n_gates).astype(np.float32)
    w = rng.uniform(1.0, 900.0, n_gates).astype(np.float32)
    nan = lambda k: torch.full((k,), float("nan"), device=dev())
    z2, dzda2, l0, l0g = nan(n_gates), nan(n_gates), nan(1), nan(n_gates)
    gws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, n_gates, 0, 0, 0), dev())
    dx, dQ, dP = last["out"]
    if case == "no_dx":
        dx, dQ = None, None
    with pytest.raises(flop.FlopError) as e:      # the next gates over the gates this layer still reads
        flop.flop_bwd_boundary(last["dy"], last["x"], last["Q"], last["P"], last["z"], last["dzda"], last["g"], dx, dQ, dP,
                               last["da"], last["ws"], pend, to_dev(la)[: last["z"].numel()], to_dev(u)[: last["z"].numel()],
                               hc_struct(), last["z"], dzda2[: last["z"].numel()], l0)
    assert e.value.status == -9
    flop.flop_trace_begin(16)
    flop.flop_bwd_boundary(last["dy"], last["x"], last["Q"], last["P"], last["z"], last["dzda"], last["g"], dx, dQ, dP,
                           last["da"], last["ws"], pend, to_dev(la), to_dev(u), hc_struct(), z2, dzda2, l0, w=to_dev(w),
                           l0_grad=l0g, l0_ws=gws)
    torch.cuda.synchronize()
    flop.flop_trace_end(16)
    for l in prev + [last]:
        assert np.array_equal(to_np(l["da"]), to_np(l["da_ref"]))
        assert_close(l["da"], l["want"]["dalpha"], TOL[dt], "dalpha")
    for got, ref in zip((dx, dQ, dP), last["ref"]):
        if got is not None:
            assert np.array_equal(to_np(got), to_np(ref))
    zo, dzo = oracle.gate_sample(la.astype(np.float64), u.astype(np.float64), BETA, L, R)
    assert_close(z2, zo, 1e-5, "z")
    assert_close(dzda2, dzo, 1e-5, "dzda")
    want_l0, want_grad = oracle.expected_l0(la.astype(np.float64), BETA, L, R, w.astype(np.float64))
    assert_close(l0g, want_grad, 1e-5, "l0_grad")
    assert abs(float(l0.item()) - want_l0) <= 1e-5 * abs(want_l0)


def test_mfma_probe_counts_and_values():
    """The rate probe reports 2*32*32*K flops per instruction, four chains, four waves per block, and leaves
    finite sums in its sink."""
    sink = torch.full((64,), float("nan"), device=dev())
    assert flop.flop_mfma_probe(flop.FLOP_BF16, 100, 3, sink) == 2.0 * 32 * 32 * 16 * 4 * 100 * 4 * 3
    assert flop.flop_mfma_probe(flop.FLOP_F32, 50, 2, sink) == 2.0 * 32 * 32 * 2 * 4 * 50 * 4 * 2
    torch.cuda.synchronize()
    assert np.all(np.isfinite(to_np(sink)))


# ------------------------------------------------------------ long tile lists ---
@pytest.mark.parametrize("shape", [(2048, 40, 72, 8200), (8192, 2048, 64, 2048)], ids=lambda s: "x".join(map(str, s)))
def test_many_short_tiles(shape):
    """Tile lists several times what the chip holds at once, of tiles with one or two k steps: 1040 tiles with
    ragged edges (y of the first shape), and a list that mixes k-split slices of a [k][row] product with one-step
    tiles of a [row][k] product (dQ and dx of the second)."""
    n, d, r, dout = shape
    c = synth.layer_inputs(8500 + n, n, d, r, dout, "bf16")
    check_layer(c)


# ----------------------------------------------------------- ranks up to 256 ---
@pytest.mark.parametrize("shape,align", [((2085, 40, 64, 4232), 0), ((2085, 40, 64, 4203), 8), ((4100, 24, 8, 2120), 0),
                                         ((130, 16, 48, 65544), 0), ((33000, 72, 24, 264), 0),
                                         ((16400, 24, 128, 8200), 0), ((8200, 24, 72, 16411), 8), ((2100, 24, 104, 64008), 0),
                                         ((2100, 40, 61, 4096), 8), ((16500, 24, 122, 8203), 8), ((2100, 40, 3, 4096), 8),
                                         ((8300, 24, 144, 8200), 0), ((8200, 16, 186, 8211), 8), ((4200, 16, 192, 16040), 64),
                                         ((8200, 16, 250, 8211), 8), ((8200, 16, 256, 8200), 0)],
                         ids=lambda s: "x".join(map(str, s)) if isinstance(s, tuple) else "align%d" % s)
def test_low_rank_wide_output(shape, align):
    """y = g P^T with a contraction extent of 256 or less and enough outputs goes to the store-bound kernel:
    ragged last row band, a last column tile of 8 columns, a row that ends inside a 16-byte chunk (padded rows),
    ranks that leave MFMA k-chunks empty, a single row band with 1025 column tiles, 258 row bands; ranks
    72, 104 and 128 take the variant with eight k-chunks per row; ranks 61, 122 and 3 end inside a 16-byte piece
    whose remainder is junk from the row's padding; ranks 144 to 256 take the variants with 32-column tiles
    and twelve or sixteen k-chunks per row."""
    n, d, r, dout = shape
    check_layer(synth.layer_inputs(8900 + r + dout % 100, n, d, r, dout, "bf16"), align=align)


# ------------------------------------------------------- seeded shape sweep ---
def _sweep_shapes():
    """24 seeded layer shapes: every extent drawn from 1..330, so that tile tails, k tails, and all three
    row-alignment classes (16-byte, 4-byte, 2-byte) of every operand turn up in some combination."""
    rng = np.random.default_rng(20240601)
    shapes = []
    for i in range(24):
        n, d, r, dout = (int(v) for v in rng.integers(1, 331, 4))
        if i % 3 == 0:
            d, r, dout = (v + (-v) % 8 for v in (d, r, dout))       # 16-byte aligned rows in bf16
        elif i % 3 == 1:
            d, r, dout = (v + v % 2 for v in (d, r, dout))          # even: 4-byte aligned rows in bf16
        shapes.append((n, d, r, dout))
    return shapes


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", _sweep_shapes(), ids=lambda s: "x".join(map(str, s)))
def test_layer_shape_sweep(dtype, shape):
    n, d, r, dout = shape
    check_layer(synth.layer_inputs(9000 + 7 * n + d, n, d, r, dout, dtype))


def _medium_shapes():
    """16 seeded shapes beyond the small sweep, four of each kind: mid-sized layers, ranks up to 128 under a wide
    output, long batches over small matrices (weight gradients cut along k), long contractions."""
    rng = np.random.default_rng(20240915)
    shapes = []
    for i in range(16):
        kind = i % 4
        if kind == 0:
            n = int(rng.integers(100, 5000)); d, r, dout = (int(v) for v in rng.integers(8, 2600, 3))
        elif kind == 1:
            r = int(rng.integers(1, 129)); n = int(rng.integers(1000, 9000)); d = int(rng.integers(8, 200))
            dout = int(rng.integers(8400000 // n, 3 * 8400000 // n))
        elif kind == 2:
            n = int(rng.integers(8000, 40000)); d, r, dout = (int(v) for v in rng.integers(16, 400, 3))
        else:
            n = int(rng.integers(64, 3000)); d = int(rng.integers(1500, 6000)); r, dout = (int(v) for v in rng.integers(16, 700, 2))
        align = (0, 8, 64, 0)[(i // 4) % 4]
        shapes.append((n, d, r, dout, align))
    return shapes


@pytest.mark.parametrize("shape", _medium_shapes(), ids=lambda s: "x".join(map(str, s[:4])) + "-align%d" % s[4])
def test_layer_shape_sweep_medium(shape):
    n, d, r, dout, align = shape
    check_layer(synth.layer_inputs(9500 + n % 97 + d, n, d, r, dout, "bf16"), align=align)


# ------------------------------------------------------------- graph replay ---
def test_step_replays_from_a_hip_graph_bit_for_bit():
    """The calls only enqueue kernels on the caller's stream, so a step can be captured; every replay
    must reproduce the eager results exactly (the path is deterministic), with eager work in between."""
    c = synth.layer_inputs(8400, 300, 136, 72, 200, "bf16")
    x, Q, P, dy = (to_dev(c[k], "bf16") for k in ("x", "Q", "P", "dy"))
    la, u = to_dev(c["log_alpha"]), to_dev(c["u"])
    n, d, r, dout = c["n"], c["d"], c["r"], c["dout"]
    z, dzda, da, grad = (torch.zeros(r, device=dev()) for _ in range(4))
    l0 = torch.zeros(1, device=dev())
    g = torch.zeros(n, r, dtype=torch.bfloat16, device=dev())
    y = torch.zeros(n, dout, dtype=torch.bfloat16, device=dev())
    dx, dQ, dP = torch.zeros_like(x), torch.zeros_like(Q), torch.zeros_like(P)
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop.FLOP_BF16, n, d, r, dout), dev())
    outs = (z, dzda, l0, grad, g, y, dx, dQ, dP, da)

    def step():
        flop.flop_gate_sample_l0(la, u, hc_struct(), z, dzda, l0, None, grad)
        flop.flop_fwd(x, Q, P, z, g, y)
        flop.flop_bwd(dy, x, Q, P, z, dzda, g, dx, dQ, dP, da, ws)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):          # capture needs a non-default stream
        step()
        side.synchronize()
        ref = [t.clone() for t in outs]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.fill_(3.0)                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs, ref):
            assert torch.equal(a, b), f"replay {rep} differs"


def test_gates_at_sixteen_million_entries():
    n = 1 << 24
    la = synth.normal(41, (n,), 0.0, 1.5)
    u = synth.uniform(42, (n,), 1e-6, 1.0 - 1e-6)
    z, dzda = torch.empty(n, device=dev()), torch.empty(n, device=dev())
    flop.flop_gate_sample(to_dev(la), to_dev(u), hc_struct(), flop.FLOP_GATE_TRAIN, z, dzda)
    zo, dzo = oracle.gate_sample(la, u, BETA, L, R)
    assert_close(z, zo, 1e-5, "z")
    # the derivative jumps where the stretched value crosses 0 or 1; fp32 and fp64 may take that
    # branch differently within rounding of the crossing, so those few entries are checked apart:
    # there the kernel's value must be one of the two branches (0, or the value just inside)
    s = 1.0 / (1.0 + np.exp(-(np.log(u) - np.log1p(-u) + la) / BETA))
    sbar = s * (R - L) + L
    near = (np.abs(sbar) < 1e-5) | (np.abs(sbar - 1.0) < 1e-5)
    assert near.sum() < n * 1e-4
    got = to_np(dzda)
    assert_close(got[~near], dzo[~near], 1e-5, "dzda")
    inside = (R - L) * s[near] * (1.0 - s[near]) / BETA
    g = got[near]
    assert np.all((g == 0.0) | (np.abs(g - inside) <= 1e-5 * np.abs(inside)))
    out = torch.empty(1, device=dev())
    ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, n, 0, 0, 0), dev())
    flop.flop_expected_l0(to_dev(la), hc_struct(), out, None, None, ws)
    so, _ = oracle.expected_l0(la, BETA, L, R)
    assert abs(float(out.item()) - so) / so <= 1e-5

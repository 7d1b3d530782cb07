"""GPU parity of a whole training step issued through the riding entry points (flop_fwd_sampling,
flop_bwd_deferred, flop_bwd_boundary) on the input classes that their randomized comparison covered:
several layers whose gate vectors are slices at arbitrary offsets of one array, rows of every alignment class
(16-byte, 4-byte, 2-byte) stored densely so that a last row ends its tensor, an empty pending list, a boundary
without new gates, and gate counts beyond what one launch samples.  Every tensor is compared with the fp64
oracle at the stated tolerances and, bit for bit, with the plain calls.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1910_04732_amd import flop, synth
from _util import TOL, TORCH_DT, assert_close, dev, hc_struct, to_dev, to_np

pytestmark = pytest.mark.gpu

BETA, L, R = synth.BETA, synth.L, synth.R

CASES = {
    # name: (dtype, [(n, d, r, dout), ...], gates before the first layer, gates after the last)
    "word_rows_dense_g": ("bf16", [(300, 202, 134, 262), (129, 66, 70, 30)], 3, 0),        # r = 6 mod 8: 4-byte rows of g
    "word_rows_last_tile": ("bf16", [(257, 130, 258, 68), (64, 258, 130, 200)], 1, 5),     # r = 2 mod 8, two tiles + 2 columns
    "single_layer_no_pending": ("bf16", [(300, 200, 136, 264)], 0, 0),                     # boundary with an empty list
    "single_word_layer_no_pending": ("bf16", [(190, 30, 66, 132)], 2, 0),
    "offsets_not_multiples_of_four": ("bf16", [(130, 72, 40, 24), (300, 200, 136, 264), (77, 136, 8, 72)], 5, 9),
    "mixed_classes": ("bf16", [(333, 200, 131, 262), (300, 203, 136, 66), (65, 7, 30, 129), (640, 64, 320, 192)], 7, 11),
    "four_aligned_layers": ("bf16", [(1202, 472, 368, 464), (1232, 440, 160, 520), (848, 616, 288, 520), (720, 160, 288, 344)], 0, 3000),
    "many_extra_gates": ("bf16", [(455, 686, 200, 136), (858, 200, 24, 256)], 13, 5000),   # > 4096 gates: separate gate launch
    "float32": ("f32", [(327, 104, 72, 688), (200, 96, 80, 136)], 6, 10),
    "one_token": ("bf16", [(1, 66, 34, 18), (1, 72, 40, 24)], 1, 1),
}


@pytest.mark.parametrize("case", list(CASES), ids=list(CASES))
def test_training_step_through_riders(case):
    dt, shapes, before, after = CASES[case]
    tdt = TORCH_DT[dt]
    seed = 9300 + 17 * list(CASES).index(case)
    G = before + sum(s[2] for s in shapes) + after
    rng = np.random.default_rng(seed)
    la = rng.normal(0.5, 1.5, G).astype(np.float32)
    u = rng.uniform(1e-6, 1 - 1e-6, G).astype(np.float32)
    w = rng.uniform(1.0, 900.0, G).astype(np.float32)
    layers, off = [], before
    for i, (n, d, r, dout) in enumerate(shapes):
        c = synth.layer_inputs(seed + i, n, d, r, dout, dt)
        la[off:off + r], u[off:off + r] = c["log_alpha"], c["u"]
        t = {k: to_dev(c[k], dt) for k in ("x", "Q", "P", "dy")}
        layers.append(dict(c=c, off=off, n=n, d=d, r=r, dout=dout, **t))
        off += r
    la_d, u_d, w_d = to_dev(la), to_dev(u), to_dev(w)
    nan = lambda k: torch.full((k,), float("nan"), device=dev())
    gws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, G, 0, 0, 0), dev())
    outs = lambda t: dict(g=torch.zeros(t["n"], t["r"], dtype=tdt, device=dev()), y=torch.zeros(t["n"], t["dout"], dtype=tdt, device=dev()),
                          dx=torch.zeros_like(t["x"]), dQ=torch.zeros_like(t["Q"]), dP=torch.zeros_like(t["P"]), da=nan(t["r"]))
    bwd_ws = lambda t: flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(t["x"]), t["n"], t["d"], t["r"], t["dout"]), dev())

    # plain calls
    zr, dzr, l0r, l0gr = nan(G), nan(G), nan(1), nan(G)
    flop.flop_gate_sample_l0(la_d, u_d, hc_struct(), zr, dzr, l0r, w=w_d, l0_grad=l0gr, ws=gws)
    ref = []
    for t in layers:
        o, sl = outs(t), slice(t["off"], t["off"] + t["r"])
        flop.flop_fwd(t["x"], t["Q"], t["P"], zr[sl], o["g"], o["y"])
        flop.flop_bwd(t["dy"], t["x"], t["Q"], t["P"], zr[sl], dzr[sl], o["g"], o["dx"], o["dQ"], o["dP"], o["da"], bwd_ws(t))
        ref.append(o)

    # the same step through the riding entry points
    z, dz, l0, l0g = nan(G), nan(G), nan(1), nan(G)
    got = [outs(t) for t in layers]
    for i, t in enumerate(layers):
        o, sl = got[i], slice(t["off"], t["off"] + t["r"])
        if i == 0:
            flop.flop_fwd_sampling(t["x"], t["Q"], t["P"], la_d, u_d, hc_struct(), z, dz, l0, t["off"], o["g"], o["y"],
                                   w=w_d, l0_grad=l0g, l0_ws=gws)
        else:
            flop.flop_fwd(t["x"], t["Q"], t["P"], z[sl], o["g"], o["y"])
    pend, keep = [], []
    for i in reversed(range(len(layers))):
        t, o, sl = layers[i], got[i], slice(layers[i]["off"], layers[i]["off"] + layers[i]["r"])
        ws = bwd_ws(t)
        keep.append(ws)
        args = (t["dy"], t["x"], t["Q"], t["P"], z[sl], dz[sl], o["g"], o["dx"], o["dQ"], o["dP"], o["da"], ws)
        if i > 0:
            pend.append(flop.flop_bwd_deferred(*args))
        else:
            flop.flop_bwd_boundary(*args, pend)
    torch.cuda.synchronize()

    assert torch.equal(z, zr) and torch.equal(dz, dzr) and torch.equal(l0g, l0gr)
    zo, dzo = oracle.gate_sample(la.astype(np.float64), u.astype(np.float64), BETA, L, R)
    assert_close(z, zo, 1e-5, "z")
    want_l0, want_grad = oracle.expected_l0(la.astype(np.float64), BETA, L, R, w.astype(np.float64))
    assert_close(l0g, want_grad, 1e-5, "l0_grad")
    assert abs(float(l0.item()) - want_l0) <= 1e-5 * abs(want_l0)
    assert abs(float(l0r.item()) - want_l0) <= 1e-5 * abs(want_l0)
    for t, o, o_ref in zip(layers, got, ref):
        for k in o:
            assert torch.equal(o[k], o_ref[k]), f"{k} differs from the plain call"
        c = t["c"]
        zl, dzl = oracle.gate_sample(c["log_alpha"], c["u"], BETA, L, R)
        _, g64, y64 = oracle.fwd(c["x"], c["Q"], c["P"], zl)
        b = oracle.bwd(c["dy"], c["x"], c["Q"], c["P"], zl, dzl)
        for k, want in (("g", g64), ("y", y64), ("dx", b["dx"]), ("dQ", b["dQ"]), ("dP", b["dP"]), ("da", b["dalpha"])):
            assert_close(o[k], want, TOL[dt], k)

"""flop_bwd_static - flop_bwd with its scratch in the library's static device array, for callers that cannot
allocate - against flop_bwd (bit for bit: both run the same kernels) and against the fp64 oracle at the stated
tolerances, on two calls in a row, the second with a smaller input that reuses the array's front part while the
rest still holds the first call's contents.  Run last: a failure here must not hide the other GPU tests.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1910_04732_amd import flop, synth
from _util import TOL, TORCH_DT, assert_close, dev, hc_struct, to_dev

pytestmark = pytest.mark.gpu

BETA, L, R = synth.BETA, synth.L, synth.R


def _layer(seed, n, d, r, dout, dt):
    c = synth.layer_inputs(seed, n, d, r, dout, dt)
    z64, dz64 = oracle.gate_sample(c["log_alpha"], c["u"], BETA, L, R)
    t = {k: to_dev(c[k], dt) for k in ("x", "Q", "P", "dy")}
    z, dzda = to_dev(z64), to_dev(dz64)
    g = torch.empty(n, r, dtype=TORCH_DT[dt], device=dev())
    y = torch.empty(n, dout, dtype=TORCH_DT[dt], device=dev())
    flop.flop_fwd(t["x"], t["Q"], t["P"], z, g, y)
    want = oracle.bwd(c["dy"], c["x"], c["Q"], c["P"], z64, dz64)
    return c, t, z, dzda, g, want


def _outs(t, r, fill):
    return (torch.full_like(t["x"], fill), torch.full_like(t["Q"], fill), torch.full_like(t["P"], fill),
            torch.full((r,), fill, device=dev()))


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_static_scratch_backward_two_calls_in_a_row(dt):
    shapes = [(2048, 768, 768, 3072), (300, 202, 134, 262)] if dt == "bf16" else [(700, 264, 200, 136), (129, 66, 40, 24)]
    for i, (n, d, r, dout) in enumerate(shapes):          # the second input is smaller than the first
        c, t, z, dzda, g, want = _layer(9700 + i, n, d, r, dout, dt)
        ref = _outs(t, r, 3.0)
        ws = flop.workspace(flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop._dt(t["x"]), n, d, r, dout), dev())
        flop.flop_bwd(t["dy"], t["x"], t["Q"], t["P"], z, dzda, g, *ref, ws)
        got = _outs(t, r, 5.0)
        flop.flop_bwd_static(t["dy"], t["x"], t["Q"], t["P"], z, dzda, g, *got)
        torch.cuda.synchronize()
        for name, a, b, w in zip(("dx", "dQ", "dP", "dalpha"), got, ref, (want["dx"], want["dQ"], want["dP"], want["dalpha"])):
            assert torch.equal(a, b), f"call {i}: {name} differs from flop_bwd"
            assert_close(a, w, TOL[dt], name)


def test_static_scratch_refuses_what_does_not_fit():
    n, d, r, dout = 8192, 3056, 3056, 9168          # dh alone is 50 MB
    assert flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop.FLOP_BF16, n, d, r, dout) > flop.FLOP_STATIC_SCRATCH_BYTES
    e = lambda *s: torch.empty(*s, dtype=torch.bfloat16, device=dev())
    zz = torch.ones(r, device=dev())
    with pytest.raises(flop.FlopError) as err:
        flop.flop_bwd_static(e(n, dout), e(n, d), e(r, d), e(dout, r), zz, zz, e(n, r), e(n, d), e(r, d), e(dout, r), torch.empty(r, device=dev()))
    assert err.value.status == -10

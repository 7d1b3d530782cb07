"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
function the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_1910_04732_amd import flop

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in ("flop.h", "flop_bench.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(flop_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(flop.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return flop.lib()


def test_header_symbols_are_exported(lib):
    names = _declared()
    assert {"flop_gate_sample", "flop_fwd", "flop_bwd", "flop_expected_l0", "flop_compact",
            "flop_workspace_bytes", "flop_status_string", "flop_bwd_static", "flop_bench_force_tile_shape"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/*.h but not exported"


def test_every_entry_point_has_declared_argument_types(lib):
    """A foreign function without argtypes gets Python ints as 32-bit C ints: a 64-bit size or leading dimension
    that travels on the stack then arrives with an undefined upper half (a wild row pitch inside a kernel)."""
    for name in _declared():
        fn = getattr(lib, name)
        if name in ("flop_bench_tile_shapes",):   # no parameters
            continue
        assert fn.argtypes is not None, f"flop.py declares no argtypes for {name}"


def test_oversized_leading_dimensions_are_rejected(lib):
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    big = (1 << 32) + 4                    # what a 32-bit 4 with a garbage upper half looks like
    L = lib
    assert L.flop_fwd(0, 2, 4, 4, 4, p, big, p, 4, p, 4, p, p, 4, p, 4, None, 0, None) == -3
    assert L.flop_fwd(0, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, p, 4, p, big, None, 0, None) == -3
    assert L.flop_bwd(1, 2, 4, 4, 4, p, 4, p, 4, p, big, p, 4, p, p, p, 4, p, 4, p, 4, p, 4, p, 0, p, 1 << 20, None) == -3
    assert L.flop_fwd_active_indexed(0, 2, 4, 4, 4, p, 4, p, 4, p, big, p, p, p, p, 4, p, 4, None) == -3
    assert L.flop_bwd_active_indexed(1, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, 4, p, p, p, p, p, 4,
                                     p, big, p, 4, p, 4, p, 0, p, 1 << 20, None) == -3


def test_pending_weight_gradients_are_validated_before_any_launch(lib):
    """flop_weight_grad_finish checks every item first; a malformed one anywhere in the list rejects the call."""
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p).value
    W = flop.flop_weight_grad_pending

    def item(**kw):
        f = dict(dtype=flop.FLOP_BF16, n=2, d=4, r=4, dout=4, dy=p, lddy=4, g=p, ldg=4, dh=p, ldh=4, x=p, ldx=4,
                 dP=p, lddp=4, dQ=p, lddq=4, split_ws=None, split_bytes=0)
        f.update(kw)
        return W(**f)
    L = lib
    for bad, status in ((item(dtype=9), -4), (item(n=-1), -2), (item(dout=0), -2), (item(lddy=3), -3), (item(ldh=3), -3),
                        (item(lddq=(1 << 32) + 4), -3), (item(g=None), -1), (item(x=None), -1)):
        arr = (W * 2)(item(dP=None, dQ=None), bad)
        assert L.flop_weight_grad_finish(arr, 2, None) == status
    assert L.flop_weight_grad_finish(None, 0, None) == 0
    assert L.flop_weight_grad_finish(None, 3, None) == -1
    assert L.flop_weight_grad_finish((W * 1)(item()), -1, None) == -2
    # an item that wants neither product is skipped: nothing to launch, no device needed
    assert L.flop_weight_grad_finish((W * 1)(item(dP=None, dQ=None)), 1, None) == 0
    # the deferring call needs somewhere to put the item
    assert L.flop_bwd_defer_weights(1, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, 4, p, p, p, 4, p, 4, p, 4, p, 4, None, 0, p, 1 << 20,
                                    None, None, None) == -1


def test_phase_stamps_exist_only_in_the_measurement_build(lib):
    """The product library has no stamps compiled into its kernels and says so."""
    buf = (ctypes.c_ulonglong * 10)()
    assert lib.flop_bench_phases_begin() == -5
    assert lib.flop_bench_phases_read(0, ctypes.cast(buf, ctypes.c_void_p), 2) == -5


def test_status_strings(lib):
    seen = {flop.status_string(s) for s in range(0, -10, -1)}
    assert len(seen) == 10 and flop.status_string(0) == "ok"
    assert flop.status_string(-99) == "unknown status"


def test_workspace_sizes(lib):
    wb = flop.flop_workspace_bytes
    assert wb(flop.FLOP_OP_FWD, flop.FLOP_BF16, 2048, 768, 768, 3072) == 0
    b = wb(flop.FLOP_OP_BWD, flop.FLOP_BF16, 2048, 768, 768, 3072)
    assert b >= 2048 * 768 * 2 + 32 * 768 * 4 and b % 256 == 0
    assert wb(flop.FLOP_OP_BWD, flop.FLOP_F32, 256, 512, 512, 512) >= 256 * 512 * 4
    assert wb(flop.FLOP_OP_EXPECTED_L0, flop.FLOP_F32, 26240, 0, 0, 0) > 0
    assert wb(flop.FLOP_OP_BWD, 9, 1, 1, 1, 1) == 0


def test_argument_validation_without_device(lib):
    """Every rejected call returns before any HIP call, so this runs without a GPU."""
    hc = flop.flop_hc(2 / 3, -0.1, 1.1)
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    L = lib
    assert L.flop_gate_sample(p, p, 8, flop.flop_hc(0.0, -0.1, 1.1), 0, p, None, None) == -5
    assert L.flop_gate_sample(p, p, 8, flop.flop_hc(1.0, 0.1, 1.1), 0, p, None, None) == -5
    assert L.flop_gate_sample(p, p, 8, flop.flop_hc(1.0, -0.1, 1.0), 0, p, None, None) == -5
    assert L.flop_gate_sample(p, None, 8, hc, 0, p, None, None) == -1
    assert L.flop_gate_sample(p, p, -1, hc, 0, p, None, None) == -2
    assert L.flop_gate_sample(p, p, 8, hc, 5, p, None, None) == -4
    assert L.flop_gate_sample(p, p, 0, hc, 0, p, None, None) == 0
    fwd = lambda dt, n, d, r, do, ldx, ldq, ldp, ldg, ldy, x=p: L.flop_fwd(
        dt, n, d, r, do, x, ldx, p, ldq, p, ldp, p, p, ldg, p, ldy, None, 0, None)
    assert fwd(3, 2, 4, 4, 4, 4, 4, 4, 4, 4) == -4
    assert fwd(0, 2, 0, 4, 4, 4, 4, 4, 4, 4) == -2
    assert fwd(0, -2, 4, 4, 4, 4, 4, 4, 4, 4) == -2
    assert fwd(0, 2, 4, 4, 4, 3, 4, 4, 4, 4) == -3
    assert fwd(0, 2, 4, 4, 4, 4, 4, 4, 4, 3) == -3
    assert fwd(0, 2, 4, 4, 4, 4, 4, 4, 4, 4, x=None) == -1
    assert fwd(0, 0, 4, 4, 4, 4, 4, 4, 4, 4) == 0
    bwd = lambda ws, nbytes: L.flop_bwd(1, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, 4, p, p, p, 4,
                                         p, 4, p, 4, p, 4, p, 0, ws, nbytes, None)
    assert bwd(None, 0) == -6
    assert bwd(p, 16) == -6
    mis = ctypes.c_void_p(ctypes.addressof(buf) | 0x10)
    need = flop.flop_workspace_bytes(flop.FLOP_OP_BWD, flop.FLOP_BF16, 2, 4, 4, 4)
    assert bwd(mis, need) in (-7, -6)
    assert L.flop_expected_l0(p, None, 8, flop.flop_hc(1.0, -0.1, 0.9), p, None, None, 0, None) == -5
    assert L.flop_expected_l0(p, None, 8, hc, None, None, None, 0, None) == -1
    assert L.flop_compact(0, 4, 4, 4, p, p, 4, p, 4, 0, None, p, p, 4, p, 4, p, None, 0, None) == -1
    assert L.flop_compact(0, 4, 4, 4, p, p, 3, p, 4, 0, p, p, p, 4, p, 4, p, None, 0, None) == -3
    assert L.flop_compact(0, 4, 4, 4, p, p, 4, p, 4, 0, p, p, p, 4, p, 3, p, None, 0, None) == -3
    assert L.flop_compact(5, 4, 4, 4, p, p, 4, p, 4, 0, p, p, p, 4, p, 4, p, None, 0, None) == -4
    # forward workspace is optional but must be aligned when given
    assert L.flop_fwd(0, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, p, 4, p, 4, mis, 1024, None) == -7
    # active-rank entry points, inference mask, size penalty, gate-gradient step, embedding
    fa = lambda ra: L.flop_fwd_active(0, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, ra, p, 4, p, 4, None, 0, None)
    assert fa(None) == -1
    ba = lambda ra, ws, nb: L.flop_bwd_active(1, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, 4, p, p, ra, p, 4,
                                              p, 4, p, 4, p, 4, p, 0, ws, nb, None)
    assert ba(None, p, 1 << 20) == -1 and ba(p, None, 0) == -6
    assert L.flop_gather_gates(p, p, None, 8, p, None) == -1
    assert L.flop_gather_gates(p, p, p, -1, p, None) == -2
    assert L.flop_gather_gates(None, None, None, 0, None, None) == 0
    ex = lambda dt, d, r, do, ra, idx, dQc, ldqc, dQ, ldq: L.flop_expand_grads(
        dt, d, r, do, ra, idx, dQc, ldqc, None, 0, None, dQ, ldq, None, 0, None, None)
    assert ex(7, 4, 4, 4, p, p, p, 4, p, 4) == -4
    assert ex(0, 4, 4, 4, None, p, p, 4, p, 4) == -1
    assert ex(0, 4, 4, 4, p, p, None, 4, p, 4) == -1
    assert ex(0, 4, 4, 4, p, p, p, 3, p, 4) == -3
    assert ex(0, 4, 0, 4, None, None, None, 0, None, 0) == 0
    assert L.flop_topk_mask(p, 8, 3, None, flop.flop_hc(1.0, 0.1, 1.1), p, None, None) == -5
    assert L.flop_topk_mask(None, 8, 3, None, hc, p, None, None) == -1
    assert L.flop_topk_mask(p, -1, 3, None, hc, p, None, None) == -2
    assert L.flop_lagrangian(None, p, 8, 1.0, 0.5, p, p, 0, p, None) == -1
    assert L.flop_lagrangian(p, None, 8, 1.0, 0.5, p, p, 0, p, None) == -1
    assert L.flop_lagrangian(p, p, 8, 1.0, 0.5, p, None, 0, None, None) == 0
    assert L.flop_gate_grad(0, 2, 4, p, 3, p, 4, p, p, p, 0, p, 1 << 20, None) == -3
    assert L.flop_gate_grad(0, 2, 4, p, 4, p, 4, p, p, p, 0, None, 0, None) == -6
    assert L.flop_gate_grad(4, 2, 4, p, 4, p, 4, p, p, p, 0, p, 1 << 20, None) == -4
    # deferred gate gradient: the pending item and dlog_alpha are required; items are checked on the host
    pend = flop.flop_gate_grad_pending()
    bwd_args = (0, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, 4, p, p, p, 4, p, 4, p, 4, p, 4)
    assert L.flop_bwd_deferred(*bwd_args, p, 0, p, 1 << 20, None, None) == -1
    assert L.flop_bwd_deferred(*bwd_args, None, 0, p, 1 << 20, None, ctypes.byref(pend)) == -1
    assert L.flop_gate_grad_finish(None, 0, None) == 0
    assert L.flop_gate_grad_finish(None, 2, None) == -1
    assert L.flop_gate_grad_finish(ctypes.byref(pend), -1, None) == -2
    assert L.flop_gate_grad_finish(ctypes.byref(pend), 1, None) == -2      # r == 0
    pend.r, pend.chunks = 8, 1
    assert L.flop_gate_grad_finish(ctypes.byref(pend), 1, None) == -1      # NULL gate vectors
    assert L.flop_mfma_probe(7, 10, 1, p, None, None) == -4
    assert L.flop_mfma_probe(1, 0, 1, p, None, None) == -2 and L.flop_mfma_probe(1, 10, 0, p, None, None) == -2
    assert L.flop_mfma_probe(1, 10, 1, None, None, None) == -1
    # step boundary: the new gates must not land in buffers the pending items still read
    buf = (ctypes.c_float * 64)()
    base = ctypes.addressof(buf)
    pend.partial, pend.z, pend.dzda, pend.dlog_alpha = base, base, base + 32, base + 64
    at = lambda off: ctypes.c_void_p(base + off)
    assert L.flop_step_boundary(ctypes.byref(pend), 1, p, p, 8, hc, at(16), at(128), None, at(192), None, None, 0, None) == -9
    assert L.flop_step_boundary(ctypes.byref(pend), 1, p, p, 8, hc, at(128), at(40), None, at(192), None, None, 0, None) == -9
    assert L.flop_step_boundary(ctypes.byref(pend), 1, p, p, 8, flop.flop_hc(1.0, 0.1, 1.1), at(128), at(160), None, at(192), None, None, 0, None) == -5
    assert L.flop_step_boundary(None, 1, p, p, 8, hc, at(128), at(160), None, at(192), None, None, 0, None) == -1
    assert L.flop_step_boundary(ctypes.byref(pend), 1, p, p, 8, hc, at(128), at(160), None, None, None, None, 0, None) == -1
    # flop_bwd_boundary: the job is checked before anything is launched
    job = flop.flop_boundary_job(None, 0, base, base, 8, hc, base + 128, base + 160, None, base + 192, None, None, 0)
    bwd_b = lambda j, z=base + 64, da=base + 96: L.flop_bwd_boundary(
        1, 2, 4, 4, 4, p, 4, p, 4, p, 4, p, 4, ctypes.c_void_p(z), ctypes.c_void_p(z), p, 4, p, 4, p, 4, p, 4,
        ctypes.c_void_p(da), 0, p, 1 << 20, j, None)
    assert bwd_b(None) == -1
    assert bwd_b(ctypes.byref(job), z=base + 128) == -9                     # next gates over this layer's gates
    assert bwd_b(ctypes.byref(job), da=base + 160) == -9                    # next dzda over this layer's dlog_alpha
    job.hc = flop.flop_hc(1.0, 0.1, 1.1)
    assert bwd_b(ctypes.byref(job)) == -5
    job.hc, job.count = hc, 1
    assert bwd_b(ctypes.byref(job)) == -1                                   # count without items
    # flop_fwd_sampling: no items, the layer's gates inside the model's, every gate output present
    job = flop.flop_boundary_job(None, 0, base, base, 8, hc, base + 128, base + 160, None, base + 192, None, None, 0)
    fwd_s = lambda j, off=0, r=4: L.flop_fwd_sampling(1, 2, 4, r, 4, p, 4, p, 4, p, r, j, off, p, r, p, 4, None, 0, None)
    assert fwd_s(None) == -1
    assert fwd_s(ctypes.byref(job), off=5) == -2 and fwd_s(ctypes.byref(job), off=-1) == -2
    job.count = 1
    assert fwd_s(ctypes.byref(job)) == -2
    job.count, job.dzda = 0, None
    assert fwd_s(ctypes.byref(job)) == -1
    job.dzda, job.l0_sum = base + 160, None
    assert fwd_s(ctypes.byref(job)) == -1


def test_workspace_sizes_cover_k_split(lib):
    wb = flop.flop_workspace_bytes
    # weight gradient at a long batch, tiny factors: the backward workspace holds the split's partial sums
    plain = 8192 * 64 * 2 + ((8192 + 31) // 32) * 64 * 4
    assert wb(flop.FLOP_OP_BWD, flop.FLOP_BF16, 8192, 128, 64, 128) >= plain + 2 * 64 * 128 * 4
    assert wb(flop.FLOP_OP_FWD, flop.FLOP_BF16, 256, 8200, 64, 4104) >= 2 * 256 * 64 * 4
    assert wb(flop.FLOP_OP_FWD, flop.FLOP_F32, 256, 8200, 64, 4104) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(flop, "_lib", None)
    monkeypatch.setattr(flop, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        flop.lib()

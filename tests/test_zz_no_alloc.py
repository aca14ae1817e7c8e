"""fftconv_pass_static: a pass whose spectral workspace is the library's own static device array,
for callers that cannot allocate.  Its results must be those of the ordinary entry points (same
kernels: the same bits) and the oracle's, call after call on the shared array."""
import numpy as np
import pytest
import torch

from oracle import direct
from paper_1312_5851_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_ABS_REL = 1e-4
REL_L2 = 1e-5


@pytest.fixture(scope="module")
def fc(fftconv_lib_path):
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_1312_5851_amd import fftconv
    return fftconv


def check(gpu, ref, what):
    gpu = gpu.cpu().numpy().astype(np.float64)
    assert gpu.shape == ref.shape and np.all(np.isfinite(gpu)), what
    diff = gpu - ref
    max_abs, scale = np.abs(diff).max(), np.abs(ref).max()
    rel_l2 = np.linalg.norm(diff.ravel()) / np.linalg.norm(ref.ravel())
    print(f"{what}: max_abs/scale={max_abs / scale:.3e} rel_l2={rel_l2:.3e}", flush=True)
    assert max_abs <= MAX_ABS_REL * scale and rel_l2 <= REL_L2, what


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def three_passes_both_ways(fc, layer, flags=0):
    """fprop, bprop, accGrad (+ accumulate) of one layer through fftconv_pass_static and through the
    ordinary entry points on a torch-owned workspace."""
    print(f"\ncase {layer} flags={flags}", flush=True)
    x, w, g = wl.make_inputs(layer)
    xd, wd, gd = dev(x), dev(w), dev(g)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k, flags=flags)
    assert plan.workspace_bytes <= fc.STATIC_SCRATCH_BYTES
    ref_plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k, flags=flags)
    want = (ref_plan.fprop(xd, wd), ref_plan.bprop(gd, wd), ref_plan.accgrad(gd, xd))
    y = torch.full(layer.shapes()[2], float("nan"), dtype=torch.float32, device="cuda")
    dx, dw = torch.full_like(xd, float("nan")), torch.full_like(wd, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    plan.pass_static(fc.FPROP, xd, wd, y)
    assert plan.valid_slots() == 0
    plan.pass_static(fc.BPROP, gd, wd, dx)
    plan.pass_static(fc.ACCGRAD, gd, xd, dw)
    assert plan.ws is None and torch.cuda.memory_allocated() == before   # no workspace was allocated on the way
    torch.cuda.synchronize()
    for name, got, ref in zip(("fprop", "bprop", "accgrad"), (y, dx, dw), want):
        check(got, ref.cpu().numpy().astype(np.float64), f"{layer.name} {name}: static scratch against caller workspace")
        # Same kernels on the same data: the same bits.  (Not for f <= 4, where the ordinary entry points
        # form dX and dW in one shared pass over the cached spectra, which nothing cached rules out here.)
        if layer.f > 4:
            assert torch.equal(got, ref), f"{layer.name} {name}: static scratch and caller workspace differ"
    check(y, direct.fprop(x, w), f"{layer.name} fprop (static scratch)")
    check(dx, direct.bprop(g, w, layer.n), f"{layer.name} bprop (static scratch)")
    ref_dw = direct.accgrad(g, x, layer.k)
    check(dw, ref_dw, f"{layer.name} accgrad (static scratch)")
    plan.pass_static(fc.ACCGRAD, gd, xd, dw, accumulate=True)
    check(dw, 2 * ref_dw, f"{layer.name} accgrad accumulating (static scratch)")
    return plan


def test_static_scratch_passes_match_the_ordinary_entry_points_call_after_call(fc):
    """Two layers in a row on the shared array, the second smaller (it must not see the first one's
    leftovers), then the first again; cached and memory-efficient plans, matrix-core and streaming
    contractions, and a tiled layer."""
    big = wl.Layer("static_big", 6, 10, 12, 32, 5, 0.05, 301)
    small = wl.Layer("static_small", 3, 5, 7, 13, 4, 0.1, 302)
    three_passes_both_ways(fc, big)
    three_passes_both_ways(fc, small)
    three_passes_both_ways(fc, big, flags=fc.RECOMPUTE)
    three_passes_both_ways(fc, wl.Layer("static_f3", 4, 3, 32, 30, 5, 0.1, 303))       # fused fprop, streaming bprop / accGrad
    three_passes_both_ways(fc, wl.Layer("static_tiled", 1, 2, 3, 100, 5, 0.1, 304))    # tiles, overlap-add
    three_passes_both_ways(fc, wl.TINY)


def test_static_scratch_leaves_a_caller_workspace_cache_consistent(fc):
    """A plan that also runs on a caller-owned workspace: a static call drops its cache bits, so the
    next ordinary call transforms its operands again instead of trusting stale slots."""
    layer = wl.Layer("static_mixed", 4, 6, 5, 16, 3, 0.1, 305)
    x, w, g = wl.make_inputs(layer)
    xd, wd, gd = dev(x), dev(w), dev(g)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    y1 = plan.fprop(xd, wd)
    assert plan.valid_slots() == fc.SPEC_X | fc.SPEC_W
    y2 = torch.empty_like(y1)
    plan.pass_static(fc.FPROP, xd, wd, y2)
    assert plan.valid_slots() == 0
    y3 = plan.fprop(xd, wd)
    assert plan.valid_slots() == fc.SPEC_X | fc.SPEC_W
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(y1, y3)


def test_static_scratch_rejects_what_does_not_fit(fc):
    layer = wl.MID
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    assert plan.workspace_bytes > fc.STATIC_SCRATCH_BYTES
    t = torch.zeros(8, device="cuda")
    with pytest.raises(fc.FftconvError) as ei:
        plan.pass_static(fc.FPROP, t, t, t)
    assert ei.value.status == 7 and "static scratch" in str(ei.value)
    with pytest.raises(fc.FftconvError) as ei:
        fc.Plan(2, 2, 2, 16, 3).pass_static(fc.FPROP, t, t, t, accumulate=True)
    assert ei.value.status == 1

"""GPU parity: the HIP path (through the C ABI) against the fp64 direct-sum oracle.

Tolerance (per output tensor, fp32 arithmetic on the GPU, fp64 oracle):
    max |gpu - oracle| <= 1e-4 * max |oracle|   and   ||gpu - oracle||_2 <= 1e-5 * ||oracle||_2
"""
import numpy as np
import pytest
import torch

from oracle import direct
from spectrum_layout import reference_spectrum, stored_bins
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
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, what
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite values"
    diff = gpu - ref
    scale = np.abs(ref).max()
    l2 = np.linalg.norm(ref.ravel())
    max_abs = np.abs(diff).max()
    rel_l2 = np.linalg.norm(diff.ravel()) / l2 if l2 > 0 else np.linalg.norm(diff.ravel())
    print(f"{what}: max_abs/scale={max_abs / max(scale, 1e-300):.3e} rel_l2={rel_l2:.3e}", flush=True)
    assert max_abs <= MAX_ABS_REL * scale + 1e-30, f"{what}: max-abs {max_abs:.3e} vs scale {scale:.3e}"
    assert rel_l2 <= REL_L2, f"{what}: rel L2 {rel_l2:.3e}"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_three(fc, layer, x, w, g):
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    xd, wd, gd = dev(x), dev(w), dev(g)
    y = plan.fprop(xd, wd)
    dx = plan.bprop(gd, wd)
    dw = plan.accgrad(gd, xd)
    torch.cuda.synchronize()
    expect = fc.SPEC_X | fc.SPEC_W | fc.SPEC_G | (fc.SPEC_G2 if plan.slot_maps(fc.SPEC_G2) > 0 else 0)
    assert plan.valid_slots() == expect
    return plan, y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()


SMALL_LAYERS = [
    wl.TINY,
    wl.Layer("ragged16", 3, 5, 7, 13, 4, 0.1, 11),      # N=16, odd map counts, ragged tiles
    wl.Layer("k1", 2, 3, 4, 16, 1, 0.1, 12),            # k = 1
    wl.Layer("k_eq_n", 2, 3, 2, 8, 8, 0.1, 13),         # k = n, single output pixel, N=8
    wl.Layer("n9", 2, 2, 3, 9, 3, 0.1, 14),             # n just above a power of two -> N=12
    wl.Layer("ragged32", 5, 7, 9, 29, 6, 0.05, 15),     # N=32, nothing a multiple of anything
    wl.Layer("n32k13", 4, 6, 5, 32, 13, 0.05, 16),
    wl.Layer("ragged64", 3, 3, 5, 50, 11, 0.05, 17),    # N=64
    wl.Layer("n64full", 2, 2, 2, 64, 3, 0.05, 18),
    wl.Layer("single", 1, 1, 1, 16, 3, 0.1, 19),
    wl.Layer("wide", 9, 40, 70, 16, 3, 0.05, 20),       # several GEMM tiles with tails
    wl.Layer("tall", 150, 33, 17, 12, 5, 0.05, 21),     # M tail beyond one 128 tile
]


@pytest.mark.parametrize("layer", SMALL_LAYERS, ids=lambda l: l.name)
def test_full_parity_small(fc, layer):
    print(f"\ncase {layer}", flush=True)
    x, w, g = wl.make_inputs(layer)
    plan, y, dx, dw = run_three(fc, layer, x, w, g)
    check(y, direct.fprop(x, w), f"{layer.name} fprop")
    check(dx, direct.bprop(g, w, layer.n), f"{layer.name} bprop")
    check(dw, direct.accgrad(g, x, layer.k), f"{layer.name} accgrad")


@pytest.mark.parametrize("name", ["mid", "first", "deep"])
def test_full_parity_full_size(fc, name):
    """The headline layer shapes at full size in the launch configuration bench.py times, every
    output element against the oracle (the direct sums of these layers take the host cores a
    few seconds each)."""
    layer = wl.CONFIGS[name]
    print(f"\ncase {layer}", flush=True)
    x, w, g = wl.make_inputs(layer)
    plan, y, dx, dw = run_three(fc, layer, x, w, g)
    check(y, direct.fprop(x, w), f"{name} fprop (all {y.size} elements)")
    check(dx, direct.bprop(g, w, layer.n), f"{name} bprop (all {dx.size} elements)")
    check(dw, direct.accgrad(g, x, layer.k), f"{name} accgrad (all {dw.size} elements)")
    # properties that hold at any size: adjoint identity on the full tensors (fp64 dot products)
    a = np.vdot(y.astype(np.float64), g.astype(np.float64))
    b = np.vdot(x.astype(np.float64), dx.astype(np.float64))
    c = np.vdot(w.astype(np.float64), dw.astype(np.float64))
    print(f"adjoint: {a:.9e} {b:.9e} {c:.9e}", flush=True)
    scale = np.linalg.norm(y.astype(np.float64)) * np.linalg.norm(g.astype(np.float64))
    assert abs(a - b) <= 1e-5 * scale and abs(a - c) <= 1e-5 * scale


def sampled_check(fc, layer, counts):
    x, w, g = wl.make_inputs(layer)
    plan, y, dx, dw = run_three(fc, layer, x, w, g)
    S, f, fo, n, k, no = layer.S, layer.f, layer.fo, layer.n, layer.k, layer.no
    u = wl.sample_units(S * fo, counts[0], layer.seed)
    check(y.reshape(S * fo, no, no)[u], direct.fprop(x, w, u), f"{layer.name} fprop sample")
    u = wl.sample_units(S * f, counts[1], layer.seed + 1)
    check(dx.reshape(S * f, n, n)[u], direct.bprop(g, w, n, u), f"{layer.name} bprop sample")
    u = wl.sample_units(fo * f, counts[2], layer.seed + 2)
    check(dw.reshape(fo * f, k, k)[u], direct.accgrad(g, x, k, u), f"{layer.name} accgrad sample")


def stratified_units(rows, cols, count, seed, block=32):
    """``count`` (at least) units r * cols + c of a rows x cols grid of output maps, chosen so that
    every block x block cell of the grid holds one of them, plus the first and the last unit.

    The grid's axes are the two free indices of the pass's per-bin matrix product (fprop: sample x
    output map, bprop: sample x input map, accGrad: output map x input map).  With block = 32, the
    side of one matrix-core tile, every workgroup tile and every wave tile of the contraction
    contributes a compared map whatever tile shape the plan picked (64x64, 128x32, 64x96, 32x32);
    the first and last units lie in the first and last workgroup of the inverse transform, and the
    rows 0 and rows-1 / columns 0 and cols-1 they and the corner cells touch are fed by the first
    and last workgroups of both forward transforms."""
    rng = np.random.Generator(np.random.Philox(key=seed ^ 0x57A7))
    picked = {0, rows * cols - 1}
    for r0 in range(0, rows, block):
        for c0 in range(0, cols, block):
            r = r0 + int(rng.integers(0, min(block, rows - r0)))
            c = c0 + int(rng.integers(0, min(block, cols - c0)))
            picked.add(r * cols + c)
    extra = min(count, rows * cols) - len(picked)
    if extra > 0:
        rest = np.setdiff1d(np.arange(rows * cols, dtype=np.int64), np.fromiter(picked, dtype=np.int64))
        picked.update(int(v) for v in rng.choice(rest, size=extra, replace=False))
    return np.sort(np.fromiter(picked, dtype=np.int64))


def adjoint_check(x, w, g, y, dx, dw, what):
    """<fprop(x,w), g> = <x, bprop(g,w)> = <w, accGrad(g,x)> on the whole device tensors (fp64 sums):
    a property of Eqs. 1-3 that holds at any size and touches every output element."""
    dot = lambda a, b: float((a.double().ravel() * b.double().ravel()).sum().item())
    a, b, c = dot(y, g), dot(x, dx), dot(w, dw)
    scale = float(torch.linalg.vector_norm(y.double()).item() * torch.linalg.vector_norm(g.double()).item())
    print(f"{what} adjoint: {a:.9e} {b:.9e} {c:.9e} (|y||g| = {scale:.3e})", flush=True)
    assert np.isfinite(a) and np.isfinite(b) and np.isfinite(c)
    assert abs(a - b) <= 1e-5 * scale and abs(a - c) <= 1e-5 * scale and abs(b - c) <= 1e-5 * scale


MIN_COMPARED = 100_000   # elements per output tensor that the oracle evaluates at a full-size sweep point


def stratified_check(fc, layer):
    """A layer at full size, in the launch configuration bench.py times.  Per pass the oracle evaluates
    whole output maps / kernels holding at least 1e5 elements, stratified over the tiles of the
    contraction and the ends of the transform launches (stratified_units); the adjoint identity then
    checks the whole tensors."""
    print(f"\ncase {layer}", flush=True)
    S, f, fo, n, k, no = layer.S, layer.f, layer.fo, layer.n, layer.k, layer.no
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(S, f, fo, n, k)
    xd, wd, gd = dev(x), dev(w), dev(g)
    y, dx, dw = plan.fprop(xd, wd), plan.bprop(gd, wd), plan.accgrad(gd, xd)
    torch.cuda.synchronize()
    grids = ((S, fo, no * no), (S, f, n * n), (fo, f, k * k))
    units = [stratified_units(r, c, -(-MIN_COMPARED // e), layer.seed + p) for p, (r, c, e) in enumerate(grids)]
    for u, (r, c, e) in zip(units, grids):
        assert len(u) * e >= min(MIN_COMPARED, r * c * e)
        cells = {(int(v) // c // 32, int(v) % c // 32) for v in u}
        assert len(cells) == -(-r // 32) * -(-c // 32), "a 32 x 32 cell of the product has no compared map"
    pick = lambda t, u, e: t.reshape(-1, e)[torch.from_numpy(u).cuda()].cpu().numpy()
    check(pick(y, units[0], no * no).reshape(-1, no, no), direct.fprop(x, w, units[0]),
          f"{layer.name} fprop ({len(units[0])} maps, {len(units[0]) * no * no} elements)")
    check(pick(dx, units[1], n * n).reshape(-1, n, n), direct.bprop(g, w, n, units[1]),
          f"{layer.name} bprop ({len(units[1])} maps, {len(units[1]) * n * n} elements)")
    check(pick(dw, units[2], k * k).reshape(-1, k, k), direct.accgrad(g, x, k, units[2]),
          f"{layer.name} accgrad ({len(units[2])} kernels, {len(units[2]) * k * k} elements)")
    adjoint_check(xd, wd, gd, y, dx, dw, layer.name)


@pytest.mark.parametrize("layer", wl.sweep_layers(), ids=lambda l: l.name)
def test_stratified_parity_every_sweep_point(fc, layer):
    """Every point of the n x k sweep (S=128, f=f'=256; n in 16, 32, 64; k in 3..13)."""
    stratified_check(fc, layer)


@pytest.mark.parametrize("layer", wl.paper_table_layers(), ids=lambda l: l.name)
def test_stratified_parity_paper_table_columns(fc, layer):
    """The five (k, n, f, f') columns of the paper's per-layer timing table at S=128."""
    stratified_check(fc, layer)


@pytest.mark.parametrize("name", ["fig3_n12", "fig3_n24", "fig3_n48", "fig3_k13", "fig3_S16", "fig3_S256"])
def test_stratified_parity_figure_axes(fc, name):
    """Points of the paper's speed figure axes (image size incl. sizes that are padded up,
    kernel size, minibatch size; f=96, f'=256)."""
    stratified_check(fc, wl.by_name(name))


@pytest.mark.parametrize("layer", [wl.TINY, SMALL_LAYERS[5], SMALL_LAYERS[7], wl.Layer("lean_wide", 9, 40, 70, 16, 3, 0.05, 81)],
                         ids=lambda l: l.name)
def test_memory_efficient_mode_parity(fc, layer):
    """Plan flag RECOMPUTE (Sec. 2.3's memory-efficient mode): three-slot workspace, every pass
    transforms its operands again and writes its result spectrum into the slot it does not read.
    Passes in an order in which a stale or clobbered slot would be used if anything were reused."""
    print(f"\ncase {layer} (recompute)", flush=True)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k, flags=fc.RECOMPUTE)
    plan.alloc_workspace()
    # the workspace tensor is exactly the three slots (+ alignment slack): guard what lies behind them
    assert plan.ws.numel() == plan.workspace_bytes + 256
    xd, wd, gd = dev(x), dev(w), dev(g)
    for _ in range(2):
        dw = plan.accgrad(gd, xd)
        assert plan.valid_slots() == 0
        y = plan.fprop(xd, wd)
        dx = plan.bprop(gd, wd)
        assert plan.valid_slots() == 0
    dw2 = plan.accgrad(gd, xd, dw.clone(), accumulate=True)
    torch.cuda.synchronize()
    check(y.cpu().numpy(), direct.fprop(x, w), f"{layer.name} fprop (recompute)")
    check(dx.cpu().numpy(), direct.bprop(g, w, layer.n), f"{layer.name} bprop (recompute)")
    ref_dw = direct.accgrad(g, x, layer.k)
    check(dw.cpu().numpy(), ref_dw, f"{layer.name} accgrad (recompute)")
    check(dw2.cpu().numpy(), 2 * ref_dw, f"{layer.name} accgrad accumulate (recompute)")
    with pytest.raises(ValueError):
        plan.slot_view(fc.SPEC_OUT)


def test_memory_efficient_mode_matches_cached_mode_at_full_size(fc):
    """Config mid: both modes run the same kernels on the same data, so the results are bit-identical."""
    layer = wl.MID
    x, w, g = wl.make_inputs(layer)
    xd, wd, gd = dev(x), dev(w), dev(g)
    cached = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    lean = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k, flags=fc.RECOMPUTE)
    for name, run in (("fprop", lambda p: p.fprop(xd, wd)), ("bprop", lambda p: p.bprop(gd, wd)),
                      ("accgrad", lambda p: p.accgrad(gd, xd))):
        a, b = run(cached), run(lean)
        torch.cuda.synchronize()
        assert torch.equal(a, b), name


TILED_LAYERS = [
    wl.Layer("n65_k3", 2, 3, 2, 65, 3, 0.1, 91),          # one past the largest transform
    wl.Layer("n100_k5", 2, 3, 4, 100, 5, 0.1, 92),
    wl.Layer("n128_k3", 1, 2, 3, 128, 3, 0.1, 93),
    wl.Layer("n96_k11", 2, 2, 2, 96, 11, 0.05, 94),
    wl.Layer("n70_k40", 1, 2, 2, 70, 40, 0.05, 95),       # large kernel: tiles are mostly overlap
    wl.Layer("n224_k11_f3", 1, 3, 4, 224, 11, 0.05, 96),  # first-layer-like image size
    wl.Layer("n80_k1", 2, 2, 2, 80, 1, 0.1, 97),          # k = 1: no overlap at all
    wl.Layer("n77_k6_ragged", 3, 5, 7, 77, 6, 0.1, 98),   # odd map counts: ragged transform groups
    wl.Layer("n72_k5", 2, 2, 3, 72, 5, 0.1, 101),         # tiles of a 5 * 2^m transform size
    # (f <= f' and blocks at least k - 1 wide: bprop adds the overlapping windows of the blocks of dL/dy into
    #  dx, overlap-add; otherwise it transforms windows of dL/dy of its own, overlap-save)
    wl.Layer("os_n100_k5", 2, 9, 4, 100, 5, 0.1, 123),          # more input than output maps: overlap-save
    wl.Layer("oa_n100_k5", 2, 2, 16, 100, 5, 0.1, 119),
    wl.Layer("oa_n224_k11_f3", 1, 3, 24, 224, 11, 0.05, 120),   # first-layer-like: 5 x 5 blocks, all four parity classes
    wl.Layer("oa_n70_k20", 1, 1, 8, 70, 20, 0.05, 121),         # windows overlap by more than half a block
    wl.Layer("oa_n130_k3", 3, 2, 17, 130, 3, 0.1, 122),         # odd map counts, 3 x 3 blocks
]


@pytest.mark.parametrize("layer", TILED_LAYERS, ids=lambda l: l.name)
def test_full_parity_tiled_layers(fc, layer):
    """n > 64: the maps are cut into overlapping tiles (overlap-save; for bprop with f <= f' overlap-add);
    all three passes against the oracle."""
    print(f"\ncase {layer}", flush=True)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    (L, _), (nt, _), (nt2, _) = plan.tiling
    print(f"N={plan.fft_size} L={L} tiles {nt}x{nt} (y), {nt2}x{nt2} (dx)", flush=True)
    assert L > 0
    xd, wd, gd = dev(x), dev(w), dev(g)
    G = 1024
    outs = []
    for shape in (layer.shapes()[2], layer.shapes()[0], layer.shapes()[1]):
        numel = int(np.prod(shape))
        buf = torch.full((numel + 2 * G,), float("nan"), dtype=torch.float32, device="cuda")
        outs.append((buf, buf[G:G + numel].view(shape)))
    # accGrad first, then bprop, then fprop: every pass finds a different set of cached spectra
    dw = plan.accgrad(gd, xd, outs[2][1])
    dx = plan.bprop(gd, wd, outs[1][1])
    y = plan.fprop(xd, wd, outs[0][1])
    torch.cuda.synchronize()
    g2 = fc.SPEC_G2 if plan.slot_maps(fc.SPEC_G2) > 0 else 0     # no second transform of dL/dy with overlap-add
    assert (g2 == 0) == (layer.f <= layer.fo and L >= layer.k - 1)
    assert plan.valid_slots() == fc.SPEC_X | fc.SPEC_W | fc.SPEC_G | g2
    for buf, _ in outs:
        assert torch.isnan(buf[:G]).all() and torch.isnan(buf[-G:]).all(), "stray write outside an output tensor"
    check(y.cpu().numpy(), direct.fprop(x, w), f"{layer.name} fprop")
    check(dx.cpu().numpy(), direct.bprop(g, w, layer.n), f"{layer.name} bprop")
    check(dw.cpu().numpy(), direct.accgrad(g, x, layer.k), f"{layer.name} accgrad")
    # invalidating dL/dy drops both of its transforms; the memory-efficient plan gives the same results
    plan.invalidate(fc.SPEC_G)
    assert plan.valid_slots() == fc.SPEC_X | fc.SPEC_W
    lean = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k, flags=fc.RECOMPUTE)
    dx2 = lean.bprop(gd, wd)
    dw2 = lean.accgrad(gd, xd)
    y2 = lean.fprop(xd, wd)
    dx3 = lean.bprop(gd, wd)
    torch.cuda.synchronize()
    assert torch.equal(dx3, dx2)
    same_scheme = lean.tiling == plan.tiling and fc.SPEC_G2 * (lean.slot_maps(fc.SPEC_G2) > 0) == g2
    if same_scheme:     # same tiles, same kernels: the same bits
        assert torch.equal(y2, y) and torch.equal(dx2, dx) and torch.equal(dw2, dw)
    else:               # without the cache, overlap-add has a higher bar: other tiles or another scheme for bprop
        check(y2.cpu().numpy(), direct.fprop(x, w), f"{layer.name} fprop (no cache)")
        check(dx2.cpu().numpy(), direct.bprop(g, w, layer.n), f"{layer.name} bprop (no cache)")
        check(dw2.cpu().numpy(), direct.accgrad(g, x, layer.k), f"{layer.name} accgrad (no cache)")
    assert lean.valid_slots() == 0


def test_sampled_parity_tiled_full_size(fc):
    """A first-layer-like tiled layer at a realistic size (S=32, 3 -> 64 maps, 128 x 128, k = 7), oracle on a sample."""
    layer = wl.Layer("tiled_first", 32, 3, 64, 128, 7, 0.05, 99)
    print(f"\ncase {layer}", flush=True)
    sampled_check_tiled = sampled_check
    sampled_check_tiled(fc, layer, (24, 24, 96))


def rect_inputs(seed, S, f, fo, nh, nw, kh, kw):
    rng = np.random.Generator(np.random.Philox(key=seed))
    x = rng.uniform(-1, 1, (S, f, nh, nw)).astype(np.float32)
    w = (rng.standard_normal((fo, f, kh, kw)) * 0.1).astype(np.float32)
    g = rng.standard_normal((S, fo, nh - kh + 1, nw - kw + 1)).astype(np.float32)
    return x, w, g


RECT_LAYERS = [
    (2, 3, 4, 20, 31, 3, 5),      # N = 32 from the width
    (3, 2, 2, 45, 12, 7, 2),      # tall maps, N = 48
    (2, 3, 2, 16, 64, 16, 1),     # kh = nh: one output row; kw = 1
    (5, 3, 4, 7, 8, 2, 8),        # one output column, N = 8
    (2, 2, 3, 64, 9, 5, 3),       # N = 64, narrow
    (1, 2, 2, 1, 24, 1, 4),       # a single row: 1-D correlation
    (2, 3, 2, 70, 41, 3, 6),      # tiled along both axes with different blocks
    (1, 2, 3, 30, 150, 4, 11),    # tiled because of the width only
    (2, 2, 2, 200, 10, 9, 2),     # tiled because of the height only
    (1, 1, 8, 30, 150, 4, 11),    # overlap-add along the width only
    (2, 2, 16, 90, 70, 5, 9),     # overlap-add, different blocks per axis
]


@pytest.mark.parametrize("dims", RECT_LAYERS, ids=lambda d: "x".join(map(str, d)))
def test_full_parity_rectangular(fc, dims):
    """Maps and kernels with different height and width (Sec. 2.1 writes square ones only to keep the
    notation short), through fftconv_plan2d, against the oracle."""
    S, f, fo, nh, nw, kh, kw = dims
    print(f"\ncase rect {dims}", flush=True)
    x, w, g = rect_inputs(500 + nh + nw, *dims)
    xd, wd, gd = dev(x), dev(w), dev(g)
    for flags in (0, fc.RECOMPUTE):
        plan = fc.Plan(S, f, fo, (nh, nw), (kh, kw), flags=flags)
        print(f"N={plan.fft_size} tiling {plan.tiling} flags {flags}", flush=True)
        dw = plan.accgrad(gd, xd)
        y = plan.fprop(xd, wd)
        dx = plan.bprop(gd, wd)
        torch.cuda.synchronize()
        assert y.shape == g.shape and dx.shape == x.shape and dw.shape == w.shape
        check(y.cpu().numpy(), direct.fprop(x, w), f"rect fprop flags={flags}")
        check(dx.cpu().numpy(), direct.bprop(g, w, (nh, nw)), f"rect bprop flags={flags}")
        check(dw.cpu().numpy(), direct.accgrad(g, x, (kh, kw)), f"rect accgrad flags={flags}")


def random_dims(rng):
    """A small random layer; sizes chosen so that every transform size, both tiling regimes,
    rectangular shapes, k = 1, k = n and ragged map counts all turn up over a few dozen draws."""
    nh = int(rng.choice([rng.integers(1, 13), rng.integers(13, 65), rng.integers(65, 110)]))
    nw = nh if rng.random() < 0.4 else int(rng.choice([rng.integers(1, 13), rng.integers(13, 65), rng.integers(65, 110)]))
    # (a tiled layer, n > 64, supports kernel sides up to 64)
    pick_k = lambda n: int(min(n, 64 if n > 64 else n, rng.choice([1, n, rng.integers(1, 8), rng.integers(1, 20)])))
    # f up to 9: layers with f <= 4 take the streaming contraction kernel in accGrad, the others the matrix-core one
    return (int(rng.integers(1, 5)), int(rng.integers(1, 10)), int(rng.integers(1, 6)), nh, nw, pick_k(nh), pick_k(nw))


@pytest.mark.parametrize("seed", range(4))
def test_random_layers_parity(fc, seed):
    """Twelve random layers per seed (square and rectangular, tiled and not, both plan modes)."""
    rng = np.random.default_rng(9000 + seed)
    for case in range(12):
        dims = random_dims(rng)
        S, f, fo, nh, nw, kh, kw = dims
        flags = fc.RECOMPUTE if case % 3 == 2 else 0
        print(f"\ncase seed={seed} #{case} dims={dims} flags={flags}", flush=True)
        x, w, g = rect_inputs(10000 + 100 * seed + case, *dims)
        plan = fc.Plan(S, f, fo, (nh, nw), (kh, kw), flags=flags)
        xd, wd, gd = dev(x), dev(w), dev(g)
        order = rng.permutation(3)
        out = {}
        for p in order:
            if p == 0:
                out["y"] = plan.fprop(xd, wd)
            elif p == 1:
                out["dx"] = plan.bprop(gd, wd)
            else:
                out["dw"] = plan.accgrad(gd, xd)
        torch.cuda.synchronize()
        check(out["y"].cpu().numpy(), direct.fprop(x, w), f"random fprop {dims}")
        check(out["dx"].cpu().numpy(), direct.bprop(g, w, (nh, nw)), f"random bprop {dims}")
        check(out["dw"].cpu().numpy(), direct.accgrad(g, x, (kh, kw)), f"random accgrad {dims}")


@pytest.mark.parametrize("layer", [SMALL_LAYERS[2], SMALL_LAYERS[7], wl.Layer("f3_wide", 5, 3, 70, 20, 5, 0.1, 82),
                                   wl.Layer("f4_tiled", 2, 4, 33, 70, 7, 0.1, 83), wl.Layer("f1", 3, 1, 40, 16, 3, 0.1, 84),
                                   wl.Layer("f2_rows", 150, 2, 130, 8, 3, 0.1, 85),
                                   # output maps a multiple of the transform group: fprop's product is fused
                                   wl.Layer("f3_fo32_n14", 3, 3, 32, 14, 3, 0.1, 102), wl.Layer("f3_fo16_n60", 2, 3, 16, 60, 7, 0.1, 103),
                                   wl.Layer("f4_fo32_tiled", 2, 4, 32, 70, 7, 0.1, 104), wl.Layer("f1_fo64_n8", 3, 1, 64, 8, 3, 0.1, 105),
                                   wl.Layer("f2_fo48_n30", 5, 2, 48, 30, 5, 0.1, 106), wl.Layer("f3_fo64_n37", 2, 3, 64, 37, 4, 0.1, 107)],
                         ids=lambda l: l.name)
def test_few_input_maps_both_contraction_paths(fc, layer, monkeypatch):
    """Layers with f <= 4 run the contractions of accGrad and bprop through streaming kernels on the
    vector ALU and form fprop's products inside the inverse transform; the matrix-core kernel must
    give the same results (to rounding) on the same layers."""
    print(f"\ncase {layer}", flush=True)
    x, w, g = wl.make_inputs(layer)
    ref = (direct.fprop(x, w), direct.bprop(g, w, layer.n), direct.accgrad(g, x, layer.k))
    for env in (None, "1"):
        if env:   # no streaming kernels, and fprop's product not fused into the inverse transform
            monkeypatch.setenv("FFTCONV_NO_SKINNY", env)
            monkeypatch.setenv("FFTCONV_NO_FUSED", env)
        plan, y, dx, dw = run_three(fc, layer, x, w, g)
        tag = "matrix cores" if env else "streaming / fused"
        check(y, ref[0], f"{layer.name} fprop ({tag})")
        check(dx, ref[1], f"{layer.name} bprop ({tag})")
        check(dw, ref[2], f"{layer.name} accgrad ({tag})")


@pytest.mark.parametrize("layer", [wl.Layer("shared_f3", 70, 3, 70, 20, 5, 0.1, 110), wl.Layer("shared_f4_rows", 200, 4, 33, 12, 3, 0.1, 111),
                                   wl.Layer("shared_f1", 5, 1, 130, 30, 7, 0.1, 112),
                                   wl.Layer("shared_f3_rows300", 300, 3, 33, 12, 3, 0.1, 124),     # two row groups per bin
                                   wl.Layer("shared_tiled_rows", 70, 2, 9, 70, 5, 0.1, 125),       # tiled, overlap-add
                                   # more than four input maps: both matrix-core contractions in one launch
                                   wl.Layer("pair_f8", 20, 8, 70, 20, 5, 0.1, 126),
                                   wl.Layer("pair_tails", 130, 65, 97, 16, 3, 0.05, 127),          # every dimension one past a tile multiple
                                   wl.Layer("pair_f5_fo3", 9, 5, 3, 12, 5, 0.1, 128),              # dX's spectrum larger than dW's
                                   wl.Layer("pair_tiled", 3, 6, 17, 100, 5, 0.1, 129)],            # tiled, overlap-add
                         ids=lambda l: l.name)
def test_bprop_and_accgrad_share_one_pass_over_the_gradient_spectrum(fc, layer):
    """With all three spectra cached, whichever of bprop / accGrad runs first forms both result spectra
    (f <= 4: one streaming kernel; more input maps: both matrix-core contractions in one launch) and
    leaves the other's for it.  Every order of calls, and every change of an
    operand in between, must give the oracle's results."""
    print(f"\ncase {layer}", flush=True)
    x, w, g = wl.make_inputs(layer)
    rng = np.random.default_rng(layer.seed)
    x2 = rng.uniform(-1, 1, x.shape).astype(np.float32)
    w2 = (rng.standard_normal(w.shape) * 0.1).astype(np.float32)
    g2 = rng.standard_normal(g.shape).astype(np.float32)
    n, k = layer.n, layer.k
    plan = fc.Plan(layer.S, layer.f, layer.fo, n, k)
    xd, wd, gd, x2d, w2d, g2d = (dev(a) for a in (x, w, g, x2, w2, g2))
    # the usual order
    plan.fprop(xd, wd)
    check(plan.bprop(gd, wd).cpu().numpy(), direct.bprop(g, w, n), "bprop first")
    check(plan.accgrad(gd, xd).cpu().numpy(), direct.accgrad(g, x, k), "accgrad second")
    # again, nothing invalidated: both are formed anew (the waiting result was used up)
    check(plan.accgrad(gd, xd).cpu().numpy(), direct.accgrad(g, x, k), "accgrad first")
    check(plan.bprop(gd, wd).cpu().numpy(), direct.bprop(g, w, n), "bprop second")
    # an operand of the waiting result changes between the two passes
    check(plan.bprop(gd, wd).cpu().numpy(), direct.bprop(g, w, n), "bprop before x changes")
    plan.invalidate(fc.SPEC_X)
    check(plan.accgrad(gd, x2d).cpu().numpy(), direct.accgrad(g, x2, k), "accgrad after x changed")
    check(plan.accgrad(gd, x2d).cpu().numpy(), direct.accgrad(g, x2, k), "accgrad before w changes")
    plan.invalidate(fc.SPEC_W)
    check(plan.bprop(gd, w2d).cpu().numpy(), direct.bprop(g, w2, n), "bprop after w changed")
    plan.invalidate(fc.SPEC_G)
    check(plan.accgrad(g2d, x2d).cpu().numpy(), direct.accgrad(g2, x2, k), "accgrad after g changed")
    check(plan.bprop(g2d, w2d).cpu().numpy(), direct.bprop(g2, w2, n), "bprop after g changed")
    # a pass in between that writes its own result spectrum
    check(plan.bprop(g2d, w2d).cpu().numpy(), direct.bprop(g2, w2, n), "bprop before fprop")
    y = torch.zeros(layer.S, layer.fo, n - k + 1, n - k + 1, device="cuda")
    plan.forward_transform(fc.SPEC_X, x2d); plan.contract(fc.FPROP); plan.inverse_transform(fc.FPROP, y)
    check(y.cpu().numpy(), direct.fprop(x2, w2), "fprop by stages")
    check(plan.accgrad(g2d, x2d).cpu().numpy(), direct.accgrad(g2, x2, k), "accgrad after the stages of fprop")
    # only two spectra at hand: the plain path
    plan.invalidate()
    check(plan.bprop(gd, wd).cpu().numpy(), direct.bprop(g, w, n), "bprop with no x spectrum")
    dw = plan.accgrad(gd, xd)
    check(plan.accgrad(gd, xd, dw, accumulate=True).cpu().numpy(), 2 * direct.accgrad(g, x, k), "accgrad accumulating")


@pytest.mark.parametrize("dims", [(2, 3, 4, 16, 16, 5, 5), (3, 2, 2, 29, 20, 6, 3), (2, 5, 3, 70, 41, 3, 6), (1, 2, 2, 8, 8, 8, 8)],
                         ids=lambda d: "x".join(map(str, d)))
def test_true_convolution_flag(fc, dims):
    """Plan flag TRUE_CONV: the kernels enter rotated by 180 degrees and their gradient leaves rotated."""
    S, f, fo, nh, nw, kh, kw = dims
    x, w, g = rect_inputs(600 + nh, *dims)
    xd, wd, gd = dev(x), dev(w), dev(g)
    for flags in (fc.TRUE_CONV, fc.TRUE_CONV | fc.RECOMPUTE):
        plan = fc.Plan(S, f, fo, (nh, nw), (kh, kw), flags=flags)
        y, dx, dw = plan.fprop(xd, wd), plan.bprop(gd, wd), plan.accgrad(gd, xd)
        dw2 = plan.accgrad(gd, xd, dw.clone(), accumulate=True)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), direct.fprop(x, w, true_conv=True), f"true conv fprop flags={flags}")
        check(dx.cpu().numpy(), direct.bprop(g, w, (nh, nw), true_conv=True), f"true conv bprop flags={flags}")
        ref = direct.accgrad(g, x, (kh, kw), true_conv=True)
        check(dw.cpu().numpy(), ref, f"true conv accgrad flags={flags}")
        check(dw2.cpu().numpy(), 2 * ref, f"true conv accgrad accumulate flags={flags}")


@pytest.mark.parametrize("dims", [(3, 5, 7, 64, 64, 11, 11), (2, 19, 3, 50, 60, 7, 16), (4, 3, 35, 41, 44, 1, 12),
                                  (2, 6, 5, 40, 33, 10, 3), (5, 4, 4, 56, 56, 14, 14)], ids=lambda d: "x".join(map(str, d)))
def test_kernel_gradient_inverse_split_over_lane_quads(fc, dims, monkeypatch):
    """Kernels of at most N/4 x N/4 on transforms of 40 points and up: with FFTCONV_QUAD set, the inverse
    transform of dL/dw splits every 1-D transform over four lanes (partial transforms summed across the quad
    by DPP adds; off by default because it measured slower).  Against the oracle and against the
    one-lane-per-transform kernel; overwriting, accumulating and with the rotated store of the
    true-convolution reading."""
    S, f, fo, nh, nw, kh, kw = dims
    print(f"\ncase quad {dims}", flush=True)
    x, w, g = rect_inputs(800 + nh + kw, *dims)
    xd, wd, gd = dev(x), dev(w), dev(g)
    for flags in (0, fc.TRUE_CONV):
        ref = direct.accgrad(g, x, (kh, kw), true_conv=bool(flags))
        one_lane = fc.Plan(S, f, fo, (nh, nw), (kh, kw), flags=flags).accgrad(gd, xd)
        monkeypatch.setenv("FFTCONV_QUAD", "1")
        plan = fc.Plan(S, f, fo, (nh, nw), (kh, kw), flags=flags)
        monkeypatch.delenv("FFTCONV_QUAD")
        assert plan.fft_size >= 40 and 4 * max(kh, kw) <= plan.fft_size
        dw = plan.accgrad(gd, xd)
        dw2 = plan.accgrad(gd, xd, dw.clone(), accumulate=True)
        torch.cuda.synchronize()
        assert not torch.equal(dw, one_lane), "the two kernels round differently: identical bits mean the switch did nothing"
        check(dw.cpu().numpy(), ref, f"quad accgrad flags={flags}")
        check(dw2.cpu().numpy(), 2 * ref, f"quad accgrad accumulating flags={flags}")
        check(one_lane.cpu().numpy(), ref, f"one lane per transform, flags={flags}")
        assert not torch.equal(dw, torch.zeros_like(dw))


def test_transposed_layer_gives_transposed_results(fc):
    """Swapping height and width of every tensor swaps them in every result (bitwise is not
    expected: the two axes are transformed in different phases)."""
    S, f, fo, nh, nw, kh, kw = 2, 3, 2, 18, 40, 3, 6
    x, w, g = rect_inputs(77, S, f, fo, nh, nw, kh, kw)
    a = fc.Plan(S, f, fo, (nh, nw), (kh, kw))
    b = fc.Plan(S, f, fo, (nw, nh), (kw, kh))
    tr = lambda t: np.ascontiguousarray(np.swapaxes(t, 2, 3))
    ya = a.fprop(dev(x), dev(w)).cpu().numpy()
    yb = b.fprop(dev(tr(x)), dev(tr(w))).cpu().numpy()
    check(tr(yb), ya.astype(np.float64), "transposed fprop")
    da = a.accgrad(dev(g), dev(x)).cpu().numpy()
    db = b.accgrad(dev(tr(g)), dev(tr(x))).cpu().numpy()
    check(tr(db), da.astype(np.float64), "transposed accgrad")


EDGE_LAYERS = [
    wl.Layer("n64_k1", 2, 3, 2, 64, 1, 0.1, 61),          # largest transform, k = 1
    wl.Layer("n64_k64", 2, 2, 3, 64, 64, 0.05, 62),       # k = n = 64: one output pixel
    wl.Layer("n33", 2, 3, 2, 33, 2, 0.1, 63),             # just above 32 -> N = 40
    wl.Layer("n49", 2, 3, 2, 49, 4, 0.1, 72),             # just above 48 -> N = 56
    wl.Layer("n57", 2, 3, 2, 57, 4, 0.1, 113),            # just above 56 -> N = 64
    wl.Layer("n56_k3", 3, 5, 4, 56, 3, 0.05, 114),        # N = 56 with no padding (a map size of image-classification networks)
    wl.Layer("n28_k5", 19, 3, 5, 28, 5, 0.1, 115),        # N = 28 with no padding, ragged tiles of 16 maps
    wl.Layer("n14_k3", 35, 3, 2, 14, 3, 0.1, 116),        # N = 14 with no padding, ragged tiles of 32 maps
    wl.Layer("n14_k14", 3, 2, 3, 14, 14, 0.1, 117),       # N = 14, k = n
    wl.Layer("n27_k13", 2, 3, 4, 27, 13, 0.05, 118),      # N = 28, middle extent classes
    wl.Layer("n17_k17", 3, 2, 2, 17, 17, 0.1, 64),        # N = 20, k = n
    wl.Layer("n25_k25", 3, 2, 2, 25, 25, 0.1, 73),        # N = 28, k = n
    wl.Layer("n48_k48", 2, 2, 3, 48, 48, 0.05, 74),       # N = 48 with no padding, k = n
    wl.Layer("n24_k2", 3, 4, 5, 24, 2, 0.1, 75),          # N = 24 with no padding
    wl.Layer("n12_k12", 5, 3, 2, 12, 12, 0.1, 76),        # N = 12, k = n
    wl.Layer("n11_k4", 35, 3, 2, 11, 4, 0.1, 77),         # N = 12, 105 / 70 maps: ragged tiles of 32
    wl.Layer("n40_k9", 2, 9, 4, 40, 9, 0.05, 78),         # N = 40 with no padding, w in the smallest extent class
    wl.Layer("n44_k20", 2, 3, 9, 44, 20, 0.05, 79),       # N = 48, middle extent classes
    wl.Layer("n34_k5", 3, 5, 4, 34, 5, 0.05, 86),         # the size Sec. 4 names as padded to 64: N = 40 here
    wl.Layer("n37_k13", 19, 3, 2, 37, 13, 0.05, 87),      # N = 40, middle extent classes, ragged tiles of 16 maps
    wl.Layer("n41_k3", 2, 3, 2, 41, 3, 0.1, 88),          # just above 40 -> N = 48
    wl.Layer("n18_k3", 35, 3, 2, 18, 3, 0.1, 89),         # N = 20, 105 / 70 maps: ragged tiles of 32
    wl.Layer("n20_k20", 3, 2, 3, 20, 20, 0.1, 90),        # N = 20 with no padding, k = n
    wl.Layer("n21_k6", 3, 4, 5, 21, 6, 0.1, 100),         # just above 20 -> N = 24
    wl.Layer("n8_k3", 5, 3, 4, 8, 3, 0.1, 65),            # N = 8
    wl.Layer("n5_k2", 3, 2, 2, 5, 2, 0.1, 66),            # n below the smallest transform
    wl.Layer("n1", 4, 3, 2, 1, 1, 0.1, 67),               # 1x1 maps
    wl.Layer("S1_f1", 1, 1, 5, 20, 7, 0.1, 68),
    wl.Layer("many_maps_tail", 7, 37, 41, 32, 3, 0.05, 69),   # map counts 259 / 1517 / 287: ragged FFT tiles
    wl.Layer("gemm_tails", 130, 65, 97, 16, 3, 0.05, 70),     # every GEMM dimension one past a tile multiple
]


@pytest.mark.parametrize("layer", EDGE_LAYERS, ids=lambda l: l.name)
def test_full_parity_edge_shapes(fc, layer):
    print(f"\ncase {layer}", flush=True)
    x, w, g = wl.make_inputs(layer)
    plan, y, dx, dw = run_three(fc, layer, x, w, g)
    check(y, direct.fprop(x, w), f"{layer.name} fprop")
    check(dx, direct.bprop(g, w, layer.n), f"{layer.name} bprop")
    check(dw, direct.accgrad(g, x, layer.k), f"{layer.name} accgrad")


def test_outputs_have_no_stray_writes(fc):
    """Each pass writes exactly its output tensor: guard bands around y, dx, dw stay untouched."""
    layer = wl.Layer("guards", 3, 5, 7, 29, 6, 0.05, 71)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    xd, wd, gd = dev(x), dev(w), dev(g)
    G = 4096
    outs = []
    for shape in (layer.shapes()[2], layer.shapes()[0], layer.shapes()[1]):
        numel = int(np.prod(shape))
        buf = torch.full((numel + 2 * G,), 12345.0, dtype=torch.float32, device="cuda")
        outs.append((buf, buf[G:G + numel].view(shape)))
    plan.fprop(xd, wd, outs[0][1])
    plan.bprop(gd, wd, outs[1][1])
    plan.accgrad(gd, xd, outs[2][1])
    torch.cuda.synchronize()
    for buf, view in outs:
        assert torch.all(buf[:G] == 12345.0) and torch.all(buf[-G:] == 12345.0)
        assert not torch.any(view == 12345.0)
    check(outs[0][1].cpu().numpy(), direct.fprop(x, w), "guards fprop")
    check(outs[1][1].cpu().numpy(), direct.bprop(g, w, layer.n), "guards bprop")
    check(outs[2][1].cpu().numpy(), direct.accgrad(g, x, layer.k), "guards accgrad")


def test_passes_in_any_order_and_on_a_side_stream(fc):
    """accGrad first (transforms g and x), then bprop (reuses g), then fprop (reuses x and w),
    all enqueued on a non-default stream."""
    layer = wl.Layer("order", 6, 10, 12, 16, 5, 0.05, 72)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    xd, wd, gd = dev(x), dev(w), dev(g)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        plan.alloc_workspace()
        dw = plan.accgrad(gd, xd)
        assert plan.valid_slots() == fc.SPEC_G | fc.SPEC_X
        dx = plan.bprop(gd, wd)
        y = plan.fprop(xd, wd)
        assert plan.valid_slots() == fc.SPEC_G | fc.SPEC_X | fc.SPEC_W
    side.synchronize()
    check(y.cpu().numpy(), direct.fprop(x, w), "order fprop")
    check(dx.cpu().numpy(), direct.bprop(g, w, layer.n), "order bprop")
    check(dw.cpu().numpy(), direct.accgrad(g, x, layer.k), "order accgrad")


@pytest.mark.parametrize("layer", [SMALL_LAYERS[5], SMALL_LAYERS[7]], ids=lambda l: l.name)
def test_step_can_be_captured_in_a_graph(fc, layer):
    """The passes only enqueue kernels on the given stream (no allocation, no host sync, no
    memset), so a caller may capture a whole step in a HIP graph.  Every replay, with eager
    work of the same plan in between, must reproduce the eager result bit for bit."""
    x, w, g = wl.make_inputs(layer)
    xd, wd, gd = dev(x), dev(w), dev(g)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    plan.alloc_workspace()
    y = torch.empty(layer.shapes()[2], dtype=torch.float32, device="cuda")
    dx, dw = torch.empty_like(xd), torch.empty_like(wd)

    def step():
        plan.invalidate()
        plan.fprop(xd, wd, y)
        plan.bprop(gd, wd, dx)
        plan.accgrad(gd, xd, dw)

    step()
    torch.cuda.synchronize()
    ref = (y.clone(), dx.clone(), dw.clone())
    check(ref[0].cpu().numpy(), direct.fprop(x, w), f"{layer.name} fprop (eager)")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in range(3):
        for t in (y, dx, dw):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref[0]) and torch.equal(dx, ref[1]) and torch.equal(dw, ref[2]), f"replay {i}"
        # eager work of the same plan between replays: other inputs through the same workspace
        plan.invalidate()
        plan.fprop(xd * 2.0, wd, y)
        torch.cuda.synchronize()
        assert torch.equal(y, 2.0 * ref[0])


def test_stage_calls_compose_to_a_pass(fc):
    layer = wl.Layer("stages", 4, 6, 5, 32, 7, 0.05, 73)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    xd, wd = dev(x), dev(w)
    plan.forward_transform(fc.SPEC_X, xd)
    plan.forward_transform(fc.SPEC_W, wd)
    plan.contract(fc.FPROP)
    y = torch.empty(layer.shapes()[2], dtype=torch.float32, device="cuda")
    plan.inverse_transform(fc.FPROP, y)
    y2 = plan.fprop(xd, wd)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    check(y.cpu().numpy(), direct.fprop(x, w), "stages fprop")


@pytest.mark.parametrize("n,N_expected", [(20, 20), (21, 24), (28, 28), (30, 32), (11, 12), (13, 14), (34, 40), (44, 48), (52, 56), (60, 64)])
def test_spectrum_stage_against_fft2(fc, n, N_expected):
    """Forward stage alone: slot contents equal the half spectrum of the zero-padded maps."""
    layer = wl.Layer("stage", 3, 5, 4, n, 6, 0.1, 31)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    N = plan.fft_size
    assert N == N_expected and plan.num_bins == N * N // 2 + 2
    for slot, arr in ((fc.SPEC_X, x), (fc.SPEC_W, w), (fc.SPEC_G, g)):
        plan.forward_transform(slot, dev(arr))
        torch.cuda.synchronize()
        spec = plan.slot_view(slot).cpu().numpy().astype(np.float64)
        spec = spec[..., 0] + 1j * spec[..., 1]
        maps = arr.reshape(-1, arr.shape[-2], arr.shape[-1]).astype(np.float64)
        ref = reference_spectrum(maps, N)
        err = np.abs(spec - ref).max() / np.abs(ref).max()
        print(f"slot {slot}: rel max err {err:.3e}", flush=True)
        assert err < 2e-6
    # impulse -> flat spectrum; constant -> only the DC bin
    imp = np.zeros_like(x); imp[:, :, 0, 0] = 1.0
    plan.forward_transform(fc.SPEC_X, dev(imp)); torch.cuda.synchronize()
    s = plan.slot_view(fc.SPEC_X).cpu().numpy()
    assert np.array_equal(s[..., 0], np.ones_like(s[..., 0])) and np.all(s[..., 1] == 0)
    # constant map filling the whole transform -> only the DC bin (needs n == N)
    plan16 = fc.Plan(2, 3, 2, 16, 3)
    plan16.forward_transform(fc.SPEC_X, torch.ones((2, 3, 16, 16), device="cuda")); torch.cuda.synchronize()
    s = plan16.slot_view(fc.SPEC_X).cpu().numpy()
    assert np.array_equal(s[0, :, 0], np.full(6, 256.0, np.float32)) and np.abs(s[1:]).max() < 1e-4
    # the four self-conjugate bins are exactly real, and Parseval holds with the stored bins
    # (every stored bin except those four stands for itself and its conjugate)
    plan.forward_transform(fc.SPEC_X, dev(x)); torch.cuda.synchronize()
    s = plan.slot_view(fc.SPEC_X).cpu().numpy().astype(np.float64)
    z = s[..., 0] + 1j * s[..., 1]
    ky, kx = stored_bins(N)
    self_conj = ((ky == 0) | (ky == N // 2)) & ((kx == 0) | (kx == N // 2))
    assert self_conj.sum() == 4 and np.all(z[self_conj].imag == 0)
    weight = np.where(self_conj, 1.0, 2.0)[:, None]
    energy = (weight * np.abs(z) ** 2).sum(0) / (N * N)
    np.testing.assert_allclose(energy, (x.astype(np.float64) ** 2).reshape(-1, layer.n ** 2).sum(1), rtol=1e-5)


def test_cache_bits_invalidate_and_accumulate(fc):
    layer = wl.Layer("cache", 4, 6, 5, 16, 3, 0.1, 41)
    x, w, g = wl.make_inputs(layer)
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    xd, wd, gd = dev(x), dev(w), dev(g)
    assert plan.valid_slots() == 0
    y1 = plan.fprop(xd, wd)
    assert plan.valid_slots() == fc.SPEC_X | fc.SPEC_W
    # a changed tensor is ignored until invalidated: the cache is explicit
    x2 = (x * 2).astype(np.float32)
    y_stale = plan.fprop(dev(x2), wd)
    assert torch.equal(y_stale, y1)
    plan.invalidate(fc.SPEC_X)
    assert plan.valid_slots() == fc.SPEC_W
    y2 = plan.fprop(dev(x2), wd)
    check(y2.cpu().numpy(), direct.fprop(x2, w), "after invalidate")
    # stage-level contract refuses a missing operand
    plan.invalidate(fc.SPEC_X | fc.SPEC_W | fc.SPEC_G)
    with pytest.raises(fc.FftconvError) as ei:
        plan.contract(fc.FPROP)
    assert ei.value.status == 5
    # accumulate adds the gradient to dw
    dw = plan.accgrad(gd, xd)
    ref = direct.accgrad(g, x, layer.k)
    check(dw.cpu().numpy(), ref, "accgrad overwrite")
    dw2 = plan.accgrad(gd, xd, dw=dw.clone(), accumulate=True)
    check(dw2.cpu().numpy(), 2 * ref, "accgrad accumulate")
    # a different workspace address drops every slot
    plan.alloc_workspace()
    plan.fprop(xd, wd)
    assert plan.valid_slots() == fc.SPEC_X | fc.SPEC_W


def test_bitwise_reproducible(fc):
    layer = wl.Layer("repro", 8, 24, 40, 16, 5, 0.05, 51)
    x, w, g = wl.make_inputs(layer)
    a = run_three(fc, layer, x, w, g)[1:]
    b = run_three(fc, layer, x, w, g)[1:]
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_argument_errors_launch_nothing(fc):
    plan = fc.Plan(2, 2, 2, 16, 3)
    t = torch.zeros(4, device="cuda")
    with pytest.raises(ValueError):
        plan.fprop(t.double(), t, t)
    import ctypes
    rc = fc._lib.fftconv_fprop(plan._h, None, None, None, None, None)
    assert rc == 1
    rc = fc._lib.fftconv_fprop(plan._h, ctypes.c_void_p(t.data_ptr()), ctypes.c_void_p(t.data_ptr()),
                               ctypes.c_void_p(t.data_ptr()), ctypes.c_void_p(t.data_ptr() + 4), None)
    assert rc == 3

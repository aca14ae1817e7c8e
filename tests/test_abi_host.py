"""CPU-only checks of the C-ABI library: it loads, exports what include/fftconv.h declares,
and its host logic (validation, workspace layout, closed forms) is right.  No kernel runs here."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def fc(fftconv_lib_path):
    from paper_1312_5851_amd import fftconv
    return fftconv


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fftconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fftconv_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree_and_every_symbol_is_exported(fc, fftconv_lib_path):
    names = declared_functions()
    assert len(names) >= 18
    assert sorted(fc.EXPORTS) == names
    lib = ctypes.CDLL(fftconv_lib_path)
    for n in names:
        assert hasattr(lib, n), n


def test_signatures_carry_no_torch_types():
    text = open(os.path.join(ROOT, "include", "fftconv.h")).read()
    assert "torch" not in text.lower() and "at::" not in text and "hipStream_t stream" not in text


@pytest.mark.parametrize("n,N", [(1, 8), (8, 8), (9, 12), (12, 12), (13, 14), (14, 14), (15, 16), (16, 16), (17, 20),
                                 (20, 20), (21, 24), (24, 24), (25, 28), (28, 28), (29, 32), (32, 32), (33, 40),
                                 (34, 40), (40, 40), (41, 48), (48, 48), (49, 56), (56, 56), (57, 64), (64, 64)])
def test_fft_size_is_smallest_compiled_size(fc, n, N):
    # Sec. 4 pads sizes that are not a power of two to the next one (34 -> 64) and names that as the
    # method's limitation; here the sizes 3 * 2^m, 5 * 2^m and 7 * 2^m are compiled as well (34 -> 40)
    p = fc.Plan(2, 3, 4, n, 1)
    assert p.fft_size == N and p.num_bins == N * N // 2 + 2


def test_workspace_layout(fc):
    p = fc.Plan(128, 96, 256, 32, 5)
    B = p.num_bins
    # the result slot holds the largest result spectrum, and dX's and dW's side by side (plus one map of
    # room for the 256-byte alignment of the second) for the joint bprop + accGrad launch
    maps = {fc.SPEC_X: 128 * 96, fc.SPEC_W: 256 * 96, fc.SPEC_G: 128 * 256,
            fc.SPEC_OUT: max(128 * 256, 128 * 96 + 256 * 96 + 1)}
    off = 0
    for slot in (fc.SPEC_X, fc.SPEC_W, fc.SPEC_G, fc.SPEC_OUT):
        assert p.slot_maps(slot) == maps[slot]
        assert p.slot_offset(slot) == off and off % 256 == 0
        off += (8 * B * maps[slot] + 255) // 256 * 256
    assert p.workspace_bytes == off
    # the three cached spectra are the S f + S f' + f f' frequency representations of Sec. 2.3
    assert p.slot_offset(fc.SPEC_OUT) == 8 * B * (128 * 96 + 128 * 256 + 96 * 256)
    assert p.slot_maps(3) == -1
    assert B == 514 and p.contraction_flops == 6.0 * 128 * 96 * 256 * B


@pytest.mark.parametrize("args,status", [
    ((0, 1, 1, 8, 3), 1), ((1, 0, 1, 8, 3), 1), ((1, 1, 0, 8, 3), 1), ((1, 1, 1, 0, 1), 1),
    ((1, 1, 1, 8, 0), 1), ((1, 1, 1, 8, 9), 1), ((1, 1, 1, 200, 65), 2), ((1, 1, 1, 65, 65), 2),
    ((65536, 65536, 1, 8, 3), 2),            # 2^32 transforms in a slot
])
def test_plan_rejects_bad_layers(fc, args, status):
    with pytest.raises(fc.FftconvError) as ei:
        fc.Plan(*args)
    assert ei.value.status == status


def test_plan_rejects_flags_and_nulls(fc):
    for flags in (4, 8, 5, 0x80000000):
        with pytest.raises(fc.FftconvError) as ei:
            fc.Plan(1, 1, 1, 8, 3, flags=flags)
        assert ei.value.status == 2
    assert fc._lib.fftconv_plan(None, None) == 1
    assert fc._lib.fftconv_plan_destroy(None) == 1
    assert fc._lib.fftconv_fft_size(None) == -1


def test_memory_efficient_plan_has_three_slots(fc):
    """Sec. 2.3: S f + S f' + f f' frequency representations and nothing else."""
    S, f, fo, n, k = 128, 96, 256, 32, 5
    cached, lean = fc.Plan(S, f, fo, n, k), fc.Plan(S, f, fo, n, k, flags=fc.RECOMPUTE)
    B = lean.num_bins
    assert B == cached.num_bins == 514
    assert lean.workspace_bytes == 8 * B * (S * f + fo * f + S * fo)       # every slot size is a multiple of 256 here
    out_maps = max(S * f, fo * f, S * fo, S * f + fo * f + 1)
    assert cached.workspace_bytes == lean.workspace_bytes + (8 * B * out_maps + 255) // 256 * 256
    for slot in (fc.SPEC_X, fc.SPEC_W, fc.SPEC_G):
        assert lean.slot_offset(slot) == cached.slot_offset(slot) and lean.slot_maps(slot) == cached.slot_maps(slot)
    assert lean.slot_maps(fc.SPEC_OUT) == -1 and lean.slot_offset(fc.SPEC_OUT) == 2 ** 64 - 1
    # below the paper's own closed form (it counts n(n+1)/2 complex numbers per map, more than the B stored here)
    assert lean.workspace_bytes <= fc.paper_ram_bytes(S, n, f, fo)
    assert lean.valid_slots() == 0
    assert fc._lib.fftconv_contract(lean._h, 0, ctypes.c_void_p(256), None) == 5


def ceil_div(a, b):
    return -(-a // b)


@pytest.mark.parametrize("n,k", [(65, 3), (100, 5), (128, 3), (128, 11), (224, 11), (70, 64), (96, 7)])
def test_large_maps_are_tiled(fc, n, k):
    """n > 64: L x L output tiles with L = N - k + 1, the N among 16..64 that needs the fewest
    transformed points; slots hold one transform per tile; an extra slot for bprop's windows
    (more input than output maps: bprop by overlap-save)."""
    S, f, fo = 2, 5, 4
    p = fc.Plan(S, f, fo, n, k)
    N, ((L, Lx), (nt, ntx), (nt2, ntx2)) = p.fft_size, p.tiling
    assert (L, nt, nt2) == (Lx, ntx, ntx2)
    no = n - k + 1
    assert N in (16, 20, 24, 28, 32, 40, 48, 56, 64) and L == N - k + 1 >= 1
    assert nt == ceil_div(no, L) and nt2 == ceil_div(n, L)
    cost = lambda c: (ceil_div(no, c - k + 1) ** 2 + ceil_div(n, c - k + 1) ** 2) * c * c
    assert all(cost(N) <= cost(c) for c in (16, 20, 24, 28, 32, 40, 48, 56, 64) if c - k + 1 >= 1)
    B = p.num_bins
    assert B == N * N // 2 + 2
    assert p.slot_maps(fc.SPEC_X) == S * nt * nt * f and p.slot_maps(fc.SPEC_W) == fo * f
    assert p.slot_maps(fc.SPEC_G) == S * nt * nt * fo and p.slot_maps(fc.SPEC_G2) == S * nt2 * nt2 * fo
    assert p.slot_maps(fc.SPEC_OUT) == max(S * nt * nt * fo, S * nt2 * nt2 * f, fo * f)
    off = 0
    for slot in (fc.SPEC_X, fc.SPEC_W, fc.SPEC_G, fc.SPEC_G2, fc.SPEC_OUT):
        assert p.slot_offset(slot) == off
        off += (8 * B * p.slot_maps(slot) + 255) // 256 * 256
    assert p.workspace_bytes == off
    assert p.contraction_flops == 6.0 * S * f * fo * B * (2 * nt * nt + nt2 * nt2) / 3
    lean = fc.Plan(S, f, fo, n, k, flags=fc.RECOMPUTE)
    tmax = max(nt, nt2) ** 2
    sizes = [(8 * B * m + 255) // 256 * 256 for m in (S * f * tmax, fo * f, S * fo * tmax)]
    assert lean.workspace_bytes == sum(sizes)
    assert lean.slot_offset(fc.SPEC_G2) == lean.slot_offset(fc.SPEC_G) == sizes[0] + sizes[1]


@pytest.mark.parametrize("n,k", [(100, 5), (224, 11), (70, 20)])
def test_tiled_layers_with_few_input_maps_use_overlap_add(fc, n, k, monkeypatch):
    """f <= f': bprop multiplies the blocks of dL/dy that accGrad transforms and adds the overlapping
    windows into dx, so there is no slot for a second transform of dL/dy and dx has one window per block."""
    S, f, fo = 2, 3, 12
    p = fc.Plan(S, f, fo, n, k)
    N, ((L, _), (nt, _), (nt2, _)) = p.fft_size, p.tiling
    assert L == N - k + 1 and nt == ceil_div(n - k + 1, L) and nt2 == nt
    assert p.slot_maps(fc.SPEC_G2) == -1 and p.slot_offset(fc.SPEC_G2) == 2 ** 64 - 1
    B = p.num_bins
    sizes = [(8 * B * m + 255) // 256 * 256 for m in (S * nt * nt * f, fo * f, S * nt * nt * fo, S * nt * nt * fo)]
    assert p.workspace_bytes == sum(sizes)      # x, w, dL/dy and a result spectrum as large as that of y
    assert p.contraction_flops == 6.0 * S * f * fo * B * nt * nt
    monkeypatch.setenv("FFTCONV_NO_OVERLAP_ADD", "1")       # read when the plan is made
    q = fc.Plan(S, f, fo, n, k)
    Lq = q.tiling[0][0]
    assert q.tiling[2][0] == ceil_div(n, Lq) and q.slot_maps(fc.SPEC_G2) == S * q.tiling[2][0] ** 2 * fo
    assert q.workspace_bytes > p.workspace_bytes
    # the tile size is the one with the fewest transformed points, counting the blocks of dL/dy twice
    cost = lambda c: 2 * ceil_div(n - k + 1, c - k + 1) ** 2 * c * c
    assert all(cost(N) <= cost(c) for c in (16, 20, 24, 28, 32, 40, 48, 56, 64) if c - k + 1 >= k - 1 and c - k + 1 >= 1)
    # windows of one parity class must not overlap: a kernel larger than the block keeps the other scheme
    monkeypatch.delenv("FFTCONV_NO_OVERLAP_ADD")
    r = fc.Plan(S, f, fo, 70, 40)
    assert r.tiling[0][0] < 39 and r.slot_maps(fc.SPEC_G2) > 0
    assert fc.Plan(S, 13, 12, n, k).slot_maps(fc.SPEC_G2) > 0     # more input than output maps


def test_rectangular_plans(fc):
    """Height and width of maps and kernels per axis; the transform stays square and covers the longer side."""
    p = fc.Plan(2, 3, 4, (20, 45), (3, 7))
    assert p.fft_size == 48 and p.num_bins == 48 * 48 // 2 + 2 and p.tiling == ((0, 0), (1, 1), (1, 1))
    assert p.slot_maps(fc.SPEC_X) == 6 and p.slot_maps(fc.SPEC_G) == 8 and p.slot_maps(fc.SPEC_W) == 12
    sq, rect = fc.Plan(2, 3, 4, 20, 3), fc.Plan(2, 3, 4, (20, 20), (3, 3))
    assert sq.fft_size == rect.fft_size and sq.workspace_bytes == rect.workspace_bytes
    # tiled, different block sizes and counts per axis (more input than output maps: bprop by overlap-save)
    p = fc.Plan(2, 5, 4, (70, 200), (3, 9))
    N, ((Ly, Lx), (ty, tx), (ty2, tx2)) = p.fft_size, p.tiling
    assert (Ly, Lx) == (N - 2, N - 8)
    assert (ty, tx) == (ceil_div(68, Ly), ceil_div(192, Lx)) and (ty2, tx2) == (ceil_div(70, Ly), ceil_div(200, Lx))
    assert p.slot_maps(fc.SPEC_X) == 2 * 5 * ty * tx and p.slot_maps(fc.SPEC_G2) == 2 * 4 * ty2 * tx2
    q = fc.Plan(2, 3, 12, (70, 200), (3, 9))    # overlap-add: dx is assembled from the windows of the blocks of dL/dy
    assert q.tiling == ((Ly, Lx), (ty, tx), (ty, tx)) and q.slot_maps(fc.SPEC_G2) == -1
    for bad in (((8, 8), (9, 3)), ((8, 8), (3, 9)), ((0, 8), (1, 1)), ((8, 8), (0, 1))):
        with pytest.raises(fc.FftconvError) as ei:
            fc.Plan(1, 1, 1, *bad)
        assert ei.value.status == 1
    with pytest.raises(fc.FftconvError) as ei:
        fc.Plan(1, 1, 1, (100, 100), (3, 65))
    assert ei.value.status == 2
    assert fc._lib.fftconv_plan2d(None, None) == 1


def test_small_maps_are_not_tiled(fc):
    p = fc.Plan(2, 3, 4, 64, 3)
    assert p.tiling == ((0, 0), (1, 1), (1, 1)) and p.slot_maps(fc.SPEC_G2) == -1 and p.slot_offset(fc.SPEC_G2) == 2 ** 64 - 1
    assert fc._lib.fftconv_forward_transform(p._h, fc.SPEC_G2, ctypes.c_void_p(256), ctypes.c_void_p(256), None) == 1
    assert fc._lib.fftconv_tiling(p._h, None, None, None) == 1


def test_invalidate_bookkeeping_and_null_pointer_errors(fc):
    p = fc.Plan(2, 2, 2, 16, 3)
    assert p.valid_slots() == 0
    p.invalidate(fc.SPEC_X | fc.SPEC_G)
    with pytest.raises(fc.FftconvError):
        p.invalidate(fc.SPEC_OUT)
    lib = fc._lib
    one = ctypes.c_void_p(256)
    assert lib.fftconv_fprop(p._h, None, one, one, one, None) == 1
    assert lib.fftconv_bprop(p._h, one, one, None, one, None) == 1
    assert lib.fftconv_accgrad(p._h, one, one, one, None, None, 0) == 3       # null workspace
    assert lib.fftconv_accgrad(p._h, one, one, one, ctypes.c_void_p(260), None, 0) == 3  # misaligned
    assert lib.fftconv_forward_transform(p._h, 3, one, one, None) == 1
    assert lib.fftconv_forward_transform(p._h, fc.SPEC_G2, one, one, None) == 1   # not a tiled layer
    assert lib.fftconv_contract(p._h, 7, one, None) == 1
    assert lib.fftconv_contract(p._h, 0, one, None) == 5                      # nothing cached: launches nothing
    assert lib.fftconv_inverse_transform(p._h, 0, None, one, None, 0) == 1
    for s in range(8):
        assert fc.strerror(s) and fc.strerror(s) != "unknown status"
    assert fc.strerror(99) == "unknown status"


def test_static_scratch_pass_checks_its_arguments_before_anything_else(fc):
    """fftconv_pass_static answers argument and size errors without touching a GPU."""
    lib, one = fc._lib, ctypes.c_void_p(256)
    small, big = fc.Plan(2, 2, 2, 16, 3), fc.Plan(128, 96, 256, 32, 5)
    assert small.workspace_bytes <= fc.STATIC_SCRATCH_BYTES < big.workspace_bytes
    assert lib.fftconv_pass_static(None, 0, one, one, one, None, 0) == 1
    assert lib.fftconv_pass_static(small._h, 3, one, one, one, None, 0) == 1
    assert lib.fftconv_pass_static(small._h, 0, None, one, one, None, 0) == 1
    assert lib.fftconv_pass_static(small._h, 0, one, one, one, None, 1) == 1     # only accGrad accumulates
    assert lib.fftconv_pass_static(big._h, 0, one, one, one, None, 0) == 7
    assert "static scratch" in fc.strerror(7)
    # the limit in the header is the one the binding quotes
    text = open(os.path.join(ROOT, "include", "fftconv.h")).read()
    assert "#define FFTCONV_STATIC_SCRATCH_BYTES ((size_t)32 << 20)" in text and fc.STATIC_SCRATCH_BYTES == 32 << 20


def test_tiled_inverse_refuses_to_accumulate_into_y_and_dx(fc):
    """accumulate on the tiled inverse of y / dx is refused (nothing launched), not silently ignored."""
    p = fc.Plan(1, 2, 3, 100, 5)
    assert p.tiling[0] != (0, 0)
    one = ctypes.c_void_p(256)
    for pass_id in (fc.FPROP, fc.BPROP):
        assert fc._lib.fftconv_inverse_transform(p._h, pass_id, one, one, None, 1) == 2


def test_paper_ram_closed_form_and_table(fc):
    gold = json.load(open(os.path.join(GOLD, "paper_ram_table.json")))
    for row in gold["rows"]:
        b = fc.paper_ram_bytes(row["S_formula"], row["n"], row["f"], row["fo"])
        assert b == 4 * row["n"] * (row["n"] + 1) * (row["S_formula"] * row["f"] + row["S_formula"] * row["fo"] + row["f"] * row["fo"])
        assert abs(b / 1e6 - row["MB"]) < 1.0, row
    # rows printed with S=128 that only match at S=64 do NOT match at the printed value
    for row in gold["rows"]:
        if row["S_printed"] != row["S_formula"]:
            b = fc.paper_ram_bytes(row["S_printed"], row["n"], row["f"], row["fo"])
            assert abs(b / 1e6 - row["MB"]) > 10
    assert fc.paper_ram_bytes(0, 1, 1, 1) == 0


def test_stored_bins_are_the_non_redundant_half(fc):
    # paper counts n(n+1)/2 complex per map; exactly N*N/2 + 2 bins are not conjugates of one
    # another (N*N real degrees of freedom: N*N/2 - 2 complex bins plus 4 real ones)
    for n in (16, 32, 64):
        p = fc.Plan(1, 1, 1, n, 3)
        assert p.num_bins == n * n // 2 + 2 <= n * (n + 1) // 2


def test_workloads_are_seeded_and_shaped():
    from paper_1312_5851_amd import workloads as wl
    x, w, g = wl.make_inputs(wl.TINY)
    x2, w2, g2 = wl.make_inputs(wl.TINY)
    assert np.array_equal(x, x2) and np.array_equal(w, w2) and np.array_equal(g, g2)
    assert x.dtype == np.float32 and x.shape == (4, 8, 16, 16) and w.shape == (8, 8, 5, 5) and g.shape == (4, 8, 12, 12)
    assert np.abs(x).max() <= 1 and abs(w.std() - 0.05) < 0.01 and abs(g.std() - 1) < 0.1
    assert wl.MID.direct_flops == 2 * 128 * 96 * 256 * 28 * 28 * 25
    assert len(wl.sweep_layers()) == 18 and len(wl.paper_table_layers()) == 5 and len(wl.fig3_layers()) == 22
    assert wl.by_name("sweep_n32_k7").k == 7 and wl.by_name("fig3_S256").S == 256
    every = list(wl.CONFIGS.values()) + wl.sweep_layers() + wl.paper_table_layers() + wl.fig3_layers()
    assert all(l.n > 64 for l in wl.large_layers())
    assert len({l.name for l in every}) == len(every) == len({l.seed for l in every})
    assert all(1 <= l.k <= l.n <= 64 for l in every)
    u = wl.sample_units(100, 10, 3)
    assert len(set(u.tolist())) == 10 and np.array_equal(u, wl.sample_units(100, 10, 3))


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU: bench.py --gpus N with N > 1 exits with a message before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_header_is_plain_c(tmp_path):
    """include/fftconv.h is a C interface: it compiles as C99 with warnings as errors."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "fftconv.h"\nint main(void) { fftconv_desc d = {1, 1, 1, 8, 3, 0}; return d.S - 1 + (int)(FFTCONV_STATIC_SCRATCH_BYTES == 0); }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)

"""CPU replay of the FFT kernels' two phases (same source as the device kernels, run
lane by lane on the host) against a naive O(N^4) fp64 DFT and numpy's fft2.

This checks the transform conventions, the pair packing, the row-0 packing, the LDS
indexing and the zero-padding / cropping pruning of every compiled tile geometry
without a GPU.  It is a test of the HIP path's index arithmetic, not the oracle."""
import ctypes

import numpy as np
import pytest

from spectrum_layout import reference_spectrum, stored_bins


@pytest.fixture(scope="module")
def replay():
    from paper_1312_5851_amd import build
    lib = ctypes.CDLL(build.build_host_replay())
    return lib


FP = ctypes.POINTER(ctypes.c_float)


def forward(lib, src, N, flip=0):
    M, ext_y, ext_x = src.shape
    B = N * N // 2 + 2
    spec = np.full((B, M, 2), np.nan, np.float32)
    assert lib.replay_fft2d_r2c(N, src.ctypes.data_as(FP), spec.ctypes.data_as(FP), M, ext_y, ext_x, flip) == 0
    return spec[..., 0].astype(np.float64) + 1j * spec[..., 1]


def inverse(lib, spec, N, crop, into=None, flip=0):
    """crop: an int (square window) or (rows, columns)."""
    cy, cx = crop if isinstance(crop, tuple) else (crop, crop)
    s = np.ascontiguousarray(np.stack([spec.real, spec.imag], -1).astype(np.float32))
    M = spec.shape[1]
    dst = np.full((M, cy, cx), np.nan, np.float32) if into is None else into.copy()
    assert lib.replay_ifft2d_c2r_crop(N, s.ctypes.data_as(FP), dst.ctypes.data_as(FP), M, cy, cx, 0 if into is None else 1, flip) == 0
    return dst


def naive_dft2(pad):
    """X[ky,kx] = sum_{y,x} pad[y,x] exp(-2 pi i (ky y + kx x)/N), written out as sums."""
    N = pad.shape[-1]
    idx = np.arange(N)
    W = np.exp(-2j * np.pi * np.outer(idx, idx) / N)
    return np.einsum("ky,myx,lx->mkl", W, pad, W)


SIZES = [8, 12, 14, 16, 20, 24, 28, 32, 40, 48, 56, 64]


def test_size_rules(replay):
    assert [replay.replay_fft_size(n) for n in (1, 8, 9, 12, 13, 14, 15, 16, 17, 20, 21, 24, 25, 28, 29, 32, 33, 34, 40, 41, 48, 49, 56, 57, 64)] == \
        [8, 8, 12, 12, 14, 14, 16, 16, 20, 20, 24, 24, 28, 28, 32, 32, 40, 40, 40, 48, 48, 56, 56, 64, 64]
    assert replay.replay_fft_size(65) == -1
    assert [replay.replay_maps_per_block(N) for N in SIZES] == [64, 32, 32, 32, 32, 16, 16, 16, 16, 16, 16, 16]
    assert replay.replay_extent_class(12, 3) == 6 and replay.replay_extent_class(24, 5) == 6
    assert replay.replay_extent_class(48, 13) == 24 and replay.replay_extent_class(48, 25) == 48
    assert replay.replay_extent_class(20, 5) == 5 and replay.replay_extent_class(40, 11) == 20
    assert replay.replay_extent_class(14, 3) == 7 and replay.replay_extent_class(28, 7) == 7 and replay.replay_extent_class(56, 29) == 56
    assert replay.replay_extent_class(32, 5) == 8 and replay.replay_extent_class(32, 9) == 16
    assert replay.replay_extent_class(32, 28) == 32 and replay.replay_extent_class(8, 2) == 4


@pytest.mark.parametrize("N", SIZES)
def test_forward_matches_naive_dft_and_fft2(replay, N):
    rng = np.random.default_rng(N)
    T = replay.replay_maps_per_block(N)
    for ext in sorted({1, 3, N // 4, N // 4 + 1, N // 2, N // 2 + 1, N - 3, N}):
        for M in (1, T - 1, T + 3):
            src = rng.uniform(-1, 1, (M, ext, ext)).astype(np.float32)
            pad = np.zeros((M, N, N)); pad[:, :ext, :ext] = src
            got = forward(replay, src, N)
            ref = reference_spectrum(src, N)
            assert np.abs(got - ref).max() <= 3e-6 * max(np.abs(ref).max(), 1), (N, ext, M)
            if N <= 24 and M == 1:
                ky, kx = stored_bins(N)
                nv = naive_dft2(pad)[:, ky, kx].T
                assert np.abs(got - nv).max() <= 3e-6 * max(np.abs(nv).max(), 1)


@pytest.mark.parametrize("N", SIZES)
def test_inverse_crops_scales_and_accumulates(replay, N):
    rng = np.random.default_rng(100 + N)
    T = replay.replay_maps_per_block(N)
    for crop in sorted({1, 3, N // 4, N // 4 + 1, N // 2 + 1, N - 2, N}):
        for M in (2, T + 1):
            full = rng.uniform(-1, 1, (M, N, N))
            spec = reference_spectrum(full, N)
            got = inverse(replay, spec, N, crop)
            assert np.abs(got - full[:, :crop, :crop]).max() < 3e-6, (N, crop, M)
            base = rng.uniform(-1, 1, (M, crop, crop)).astype(np.float32)
            acc = inverse(replay, spec, N, crop, into=base)
            assert np.abs(acc - (base + full[:, :crop, :crop])).max() < 3e-6


@pytest.mark.parametrize("N", SIZES)
def test_small_batch_geometries(replay, N):
    """The geometries with few maps per workgroup (one or two waves; launches of few maps take them): forward
    and inverse, every extent class, ragged map counts, flipped loads and accumulating stores."""
    rng = np.random.default_rng(900 + N)
    T = replay.replay_small_maps_per_block(N)
    assert T * N // 2 >= 48 and T < replay.replay_maps_per_block(N)
    B = N * N // 2 + 2
    for ext in sorted({1, N // 4, N // 4 + 1, N // 2 + 1, N}):
        for M in (1, T + 1, 3 * T):
            src = rng.uniform(-1, 1, (M, ext, ext)).astype(np.float32)
            for flip in (0, 1):
                spec = np.full((B, M, 2), np.nan, np.float32)
                assert replay.replay_fft2d_r2c_small(N, src.ctypes.data_as(FP), spec.ctypes.data_as(FP), M, ext, ext, flip) == 0
                got = spec[..., 0].astype(np.float64) + 1j * spec[..., 1]
                ref = reference_spectrum(src[:, ::-1, ::-1] if flip else src, N)
                assert np.abs(got - ref).max() <= 3e-6 * max(np.abs(ref).max(), 1), (N, ext, M, flip)
            full = rng.uniform(-1, 1, (M, N, N))
            sp = reference_spectrum(full, N)
            s = np.ascontiguousarray(np.stack([sp.real, sp.imag], -1).astype(np.float32))
            base = rng.uniform(-1, 1, (M, ext, ext)).astype(np.float32)
            for acc in (0, 1):
                dst = base.copy() if acc else np.full((M, ext, ext), np.nan, np.float32)
                assert replay.replay_ifft2d_c2r_crop_small(N, s.ctypes.data_as(FP), dst.ctypes.data_as(FP), M, ext, ext, acc, 0) == 0
                want = full[:, :ext, :ext] + (base if acc else 0)
                assert np.abs(dst - want).max() < 3e-6, (N, ext, M, acc)


@pytest.mark.parametrize("N", [40, 48, 56, 64])
def test_quad_split_inverse_for_small_windows(replay, N):
    """The inverse for windows of at most N/4 x N/4 with every 1-D transform split over four lanes
    (partial transforms of N/4 points, twiddled, summed across the quad): same results as the
    one-lane-per-transform kernel, for square and rectangular crops, ragged map counts, accumulating
    and flipped stores."""
    rng = np.random.default_rng(700 + N)
    T = replay.replay_maps_per_block(N)
    for crop in (1, 3, 5, (2, N // 4), (N // 4, 1), N // 4):
        cy, cx = crop if isinstance(crop, tuple) else (crop, crop)
        for M in (1, 2, T + 3):
            full = rng.uniform(-1, 1, (M, N, N))
            spec = reference_spectrum(full, N)
            s = np.ascontiguousarray(np.stack([spec.real, spec.imag], -1).astype(np.float32))
            for flip in (0, 1):
                want = full[:, :cy, :cx][:, ::-1, ::-1] if flip else full[:, :cy, :cx]
                dst = np.full((M, cy, cx), np.nan, np.float32)
                assert replay.replay_ifft2d_c2r_crop_quad(N, s.ctypes.data_as(FP), dst.ctypes.data_as(FP), M, cy, cx, 0, flip) == 0
                assert np.abs(dst - want).max() < 3e-6, (N, crop, M, flip)
                base = rng.uniform(-1, 1, (M, cy, cx)).astype(np.float32)
                acc = base.copy()
                assert replay.replay_ifft2d_c2r_crop_quad(N, s.ctypes.data_as(FP), acc.ctypes.data_as(FP), M, cy, cx, 1, flip) == 0
                assert np.abs(acc - (base + want)).max() < 3e-6
                ref = inverse(replay, spec, N, (cy, cx), flip=flip)
                assert np.abs(dst - ref).max() < 2e-6
    big = np.zeros((1, N // 4 + 1, 1), np.float32)
    assert replay.replay_ifft2d_c2r_crop_quad(N, s.ctypes.data_as(FP), big.ctypes.data_as(FP), 1, N // 4 + 1, 1, 0, 0) == 2


@pytest.mark.parametrize("N", [16, 20, 24, 28])
def test_impulse_constant_and_round_trip(replay, N):
    imp = np.zeros((3, N, N), np.float32); imp[:, 0, 0] = 1
    s = forward(replay, imp, N)
    assert np.array_equal(s, np.ones_like(s))
    s = forward(replay, np.ones((2, N, N), np.float32), N)
    assert np.array_equal(s[0], [N * N, N * N]) and np.abs(s[1:]).max() < 1e-4
    x = np.random.default_rng(5).uniform(-1, 1, (5, 11, 11)).astype(np.float32)
    back = inverse(replay, forward(replay, x, N), N, 11)
    assert np.abs(back - x).max() < 1e-6


# ---------------------------------------------------------------- tiled (overlap-save) variants

def tile_windows(img, N, tiles_x, tiles, step, org, ext):
    """[S, C, H, W] images -> zero-filled windows [S * tiles * C, N, N] in transform order
    m = (s * tiles + t) * C + c, window origin (ty * step_y + org_y, tx * step_x + org_x), extent
    ext_y x ext_x (step, org, ext: ints or (y, x) pairs)."""
    pair = lambda v: v if isinstance(v, tuple) else (v, v)
    (sy, sx), (gy, gx), (ey, ex) = pair(step), pair(org), pair(ext)
    S, C, H, W = img.shape
    out = np.zeros((S * tiles * C, N, N))
    for s in range(S):
        for t in range(tiles):
            oy, ox = (t // tiles_x) * sy + gy, (t % tiles_x) * sx + gx
            for c in range(C):
                for y in range(ey):
                    for x in range(ex):
                        if 0 <= oy + y < H and 0 <= ox + x < W:
                            out[(s * tiles + t) * C + c, y, x] = img[s, c, oy + y, ox + x]
    return out


@pytest.mark.parametrize("N,H,k", [(16, 37, 5), (20, 45, 4), (24, 50, 3), (28, 60, 5), (32, 70, 11), (40, 90, 7), (48, 65, 4), (56, 120, 8), (64, 100, 9)])
def test_tiled_forward_windows(replay, N, H, k):
    """The three kinds of windows a tiled layer transforms: dense N x N windows of x (stride L),
    L x L blocks of dL/dy, and the windows of dL/dy that start k-1 before a tile of dx."""
    rng = np.random.default_rng(N + H)
    L = N - k + 1
    S, C = 2, 3
    no = H - k + 1
    nt, nt2 = -(-no // L), -(-H // L)
    B = N * N // 2 + 2
    cases = [("x windows", H, nt, 0, N), ("g blocks", no, nt, 0, L), ("g windows", no, nt2, -(k - 1), N)]
    for what, size, tx, org, ext in cases:
        img = rng.uniform(-1, 1, (S, C, size, size)).astype(np.float32)
        M = S * tx * tx * C
        spec = np.full((B, M, 2), np.nan, np.float32)
        rc = replay.replay_fft2d_r2c_tiled(N, img.ctypes.data_as(FP), spec.ctypes.data_as(FP), M, ext, ext, size, size, C,
                                           tx, tx * tx, L, L, org, org, 0)
        assert rc == 0
        got = spec[..., 0].astype(np.float64) + 1j * spec[..., 1]
        ref = reference_spectrum(tile_windows(img, N, tx, tx * tx, L, org, ext), N)
        assert np.abs(got - ref).max() <= 3e-6 * max(np.abs(ref).max(), 1), (what, N, H, k)


@pytest.mark.parametrize("N,H,k,c0", [(16, 37, 5, 0), (16, 37, 5, 4), (20, 45, 4, 3), (24, 50, 3, 2), (28, 60, 5, 4), (40, 90, 7, 6), (48, 65, 4, 0), (56, 120, 8, 7), (64, 100, 9, 8)])
def test_tiled_inverse_scatters_each_tile_once(replay, N, H, k, c0):
    """Rows / columns [c0, c0 + L) of every transform's output land at the tile's place;
    the tiles cover the image exactly once and nothing else is written."""
    rng = np.random.default_rng(7 * N + c0)
    L = N - k + 1
    S, C = 2, 3
    tx = -(-H // L)
    M = S * tx * tx * C
    patches = rng.uniform(-1, 1, (M, N, N))
    spec = reference_spectrum(patches, N)
    sp = np.ascontiguousarray(np.stack([spec.real, spec.imag], -1).astype(np.float32))
    dst = np.full((S, C, H, H), np.nan, np.float32)
    guard = np.full(64, np.nan, np.float32)
    buf = np.concatenate([guard, dst.ravel(), guard])
    view = buf[64:64 + dst.size]
    rc = replay.replay_ifft2d_c2r_tiled(N, sp.ctypes.data_as(FP), view.ctypes.data_as(FP), M, L, L, c0, c0, H, H, C,
                                        tx, tx * tx, L, L, 0, -1, 0)
    assert rc == 0
    assert np.all(np.isnan(buf[:64])) and np.all(np.isnan(buf[-64:]))
    got = view.reshape(S, C, H, H)
    assert not np.isnan(got).any()
    for s in range(S):
        for t in range(tx * tx):
            oy, ox = (t // tx) * L, (t % tx) * L
            for c in range(C):
                h, w = min(L, H - oy), min(L, H - ox)
                ref = patches[(s * tx * tx + t) * C + c, c0:c0 + h, c0:c0 + w]
                assert np.abs(got[s, c, oy:oy + h, ox:ox + w] - ref).max() < 3e-6


# ---------------------------------------------------------------- rectangular extents

@pytest.mark.parametrize("N", SIZES)
def test_rectangular_maps_forward_and_inverse(replay, N):
    """Maps and windows with different height and width inside a square transform."""
    rng = np.random.default_rng(300 + N)
    T = replay.replay_maps_per_block(N)
    for ey, ex in ((1, N), (N, 1), (N // 2, N - 1), (N - 1, N // 4 + 1), (3, 2), (N // 4, N // 2 + 1)):
        M = T + 1
        src = rng.uniform(-1, 1, (M, ey, ex)).astype(np.float32)
        pad = np.zeros((M, N, N)); pad[:, :ey, :ex] = src
        ky, kx = stored_bins(N)
        ref = np.fft.fft2(pad)[:, ky, kx].T
        got = forward(replay, src, N)
        assert np.abs(got - ref).max() <= 3e-6 * max(np.abs(ref).max(), 1), (N, ey, ex)
        full = rng.uniform(-1, 1, (M, N, N))
        back = inverse(replay, reference_spectrum(full, N), N, (ey, ex))
        assert back.shape == (M, ey, ex) and np.abs(back - full[:, :ey, :ex]).max() < 3e-6, (N, ey, ex)


def test_tiled_rectangular_windows_and_scatter(replay):
    """Tiles of a 70 x 41 image with a 3 x 6 kernel at N = 32: different steps, origins,
    extents and stored windows per axis."""
    rng = np.random.default_rng(77)
    N, H, W, kh, kw, S, C = 32, 70, 41, 3, 6, 2, 3
    Ly, Lx = N - kh + 1, N - kw + 1
    noh, now = H - kh + 1, W - kw + 1
    B = N * N // 2 + 2
    cases = [("x windows", (H, W), (-(-noh // Ly), -(-now // Lx)), (0, 0), (N, N)),
             ("g blocks", (noh, now), (-(-noh // Ly), -(-now // Lx)), (0, 0), (Ly, Lx)),
             ("g windows", (noh, now), (-(-H // Ly), -(-W // Lx)), (-(kh - 1), -(kw - 1)), (N, N))]
    for what, (h, w), (ty, tx), org, ext in cases:
        img = rng.uniform(-1, 1, (S, C, h, w)).astype(np.float32)
        M = S * ty * tx * C
        spec = np.full((B, M, 2), np.nan, np.float32)
        rc = replay.replay_fft2d_r2c_tiled(N, img.ctypes.data_as(FP), spec.ctypes.data_as(FP), M, ext[0], ext[1], h, w, C,
                                           tx, ty * tx, Ly, Lx, org[0], org[1], 0)
        assert rc == 0
        got = spec[..., 0].astype(np.float64) + 1j * spec[..., 1]
        ref = reference_spectrum(tile_windows(img, N, tx, ty * tx, (Ly, Lx), org, ext), N)
        assert np.abs(got - ref).max() <= 3e-6 * max(np.abs(ref).max(), 1), what
    # scatter of dx tiles: rows [kh-1, N), columns [kw-1, N) of each transform
    ty, tx = -(-H // Ly), -(-W // Lx)
    M = S * ty * tx * C
    patches = rng.uniform(-1, 1, (M, N, N))
    spec = reference_spectrum(patches, N)
    sp = np.ascontiguousarray(np.stack([spec.real, spec.imag], -1).astype(np.float32))
    dst = np.full((S, C, H, W), np.nan, np.float32)
    rc = replay.replay_ifft2d_c2r_tiled(N, sp.ctypes.data_as(FP), dst.ctypes.data_as(FP), M, Ly, Lx, kh - 1, kw - 1, H, W, C,
                                        tx, ty * tx, Ly, Lx, 0, -1, 0)
    assert rc == 0 and not np.isnan(dst).any()
    for s in range(S):
        for t in range(ty * tx):
            oy, ox = (t // tx) * Ly, (t % tx) * Lx
            for c in range(C):
                h, w = min(Ly, H - oy), min(Lx, W - ox)
                ref = patches[(s * ty * tx + t) * C + c, kh - 1:kh - 1 + h, kw - 1:kw - 1 + w]
                assert np.abs(dst[s, c, oy:oy + h, ox:ox + w] - ref).max() < 3e-6


def tiles_in_order(ty, tx, by_class):
    """(row, column) of tile number t: row-major, or parity class by parity class (class 2 (row % 2) + column % 2,
    row-major inside a class)."""
    tiles = [(y, x) for y in range(ty) for x in range(tx)]
    return sorted(tiles, key=lambda p: (2 * (p[0] % 2) + p[1] % 2, p)) if by_class else tiles


@pytest.mark.parametrize("ty,tx", [(1, 1), (1, 4), (3, 1), (2, 2), (3, 5), (4, 3), (5, 5)])
def test_tile_numbering_by_parity_class(replay, ty, tx):
    for by_class in (0, 1):
        want = tiles_in_order(ty, tx, by_class)
        for t in range(ty * tx):
            y, x = ctypes.c_int(-1), ctypes.c_int(-1)
            replay.replay_tile_row_col(t, tx, ty * tx, by_class, ctypes.byref(y), ctypes.byref(x))
            assert (y.value, x.value) == want[t], (t, by_class)


@pytest.mark.parametrize("by_class", [0, 1])
@pytest.mark.parametrize("N,Hy,Hx,kh,kw", [(16, 37, 30, 5, 3), (28, 70, 90, 6, 9), (48, 224, 100, 11, 11), (64, 65, 130, 3, 20),
                                          (16, 14, 60, 3, 3),      # one row of tiles
                                          (16, 40, 44, 9, 9),      # blocks exactly k - 1 wide: windows two apart touch
                                          (20, 100, 21, 1, 2)])    # kh = 1: no vertical overlap at all
def test_tiled_inverse_overlap_add(replay, N, Hy, Hx, kh, kw, by_class):
    """Overlap-add: the whole N x N output of every block's transform is added at the block's origin
    (blocks (N-kh+1) x (N-kw+1) apart, so neighbours overlap by kh-1 / kw-1), one parity class of
    tiles per call, in class order; after the four calls every pixel holds the sum of the windows that
    cover it, whatever the destination held before (the first class covering a pixel stores, the later
    ones add: nothing is cleared beforehand).  With either numbering of the tiles."""
    rng = np.random.default_rng(11 * N + Hy)
    Ly, Lx = N - kh + 1, N - kw + 1
    S, C = 2, 3
    ty, tx = -(-(Hy - kh + 1) // Ly), -(-(Hx - kw + 1) // Lx)      # blocks of the (Hy-kh+1) x (Hx-kw+1) gradient
    M = S * ty * tx * C
    patches = rng.uniform(-1, 1, (M, N, N))
    spec = reference_spectrum(patches, N)
    sp = np.ascontiguousarray(np.stack([spec.real, spec.imag], -1).astype(np.float32))
    dst = np.full((S, C, Hy, Hx), np.nan, np.float32)
    for parity in range(4):
        rc = replay.replay_ifft2d_c2r_tiled(N, sp.ctypes.data_as(FP), dst.ctypes.data_as(FP), M, N, N, 0, 0, Hy, Hx, C,
                                            tx, ty * tx, Ly, Lx, 1, parity, by_class)
        assert rc == 0
    ref = np.zeros((S, C, Hy, Hx))
    order = tiles_in_order(ty, tx, by_class)
    for s in range(S):
        for t in range(ty * tx):
            oy, ox = order[t][0] * Ly, order[t][1] * Lx
            h, w = min(N, Hy - oy), min(N, Hx - ox)
            for c in range(C):
                ref[s, c, oy:oy + h, ox:ox + w] += patches[(s * ty * tx + t) * C + c, :h, :w]
    assert np.abs(dst - ref).max() < 1e-5


@pytest.mark.parametrize("N", [8, 14, 24, 32, 40, 56, 64])
def test_flipped_load_and_store(replay, N):
    """The kernels of a true convolution are read rotated by 180 degrees, their gradient is stored rotated."""
    rng = np.random.default_rng(400 + N)
    T = replay.replay_maps_per_block(N)
    for ey, ex in ((3, 3), (N // 4, N // 2 + 1), (1, 5), (N, N - 1)):
        M = T + 1
        src = rng.uniform(-1, 1, (M, ey, ex)).astype(np.float32)
        got = forward(replay, src, N, flip=1)
        ref = reference_spectrum_rect(np.ascontiguousarray(src[:, ::-1, ::-1]), N)
        assert np.abs(got - ref).max() <= 3e-6 * max(np.abs(ref).max(), 1), (N, ey, ex)
        full = rng.uniform(-1, 1, (M, N, N))
        back = inverse(replay, reference_spectrum(full, N), N, (ey, ex), flip=1)
        assert np.abs(back - full[:, :ey, :ex][:, ::-1, ::-1]).max() < 3e-6
        base = rng.uniform(-1, 1, (M, ey, ex)).astype(np.float32)
        acc = inverse(replay, reference_spectrum(full, N), N, (ey, ex), into=base, flip=1)
        assert np.abs(acc - (base + full[:, :ey, :ex][:, ::-1, ::-1])).max() < 3e-6


def reference_spectrum_rect(maps, N):
    M, ey, ex = maps.shape
    pad = np.zeros((M, N, N)); pad[:, :ey, :ex] = maps
    ky, kx = stored_bins(N)
    return np.fft.fft2(pad)[:, ky, kx].T


@pytest.mark.parametrize("N,k", [(8, 2), (14, 3), (16, 3), (20, 2), (40, 5), (56, 6), (64, 9)])
def test_fused_product_inverse_is_the_valid_correlation(replay, N, k):
    """fprop with three input maps: the inverse transform forms its bins from the spectra of x and w
    (Sec. 2.2) and must leave the valid cross-correlation, summed over the input maps, written out
    here as plain sums.  64 output maps per sample: one to four groups of maps."""
    rng = np.random.default_rng(500 + N)
    Sn, f, fo = 3, 3, 64
    x = rng.uniform(-1, 1, (Sn, f, N, N)).astype(np.float32)
    w = rng.normal(0, 0.3, (fo, f, k, k)).astype(np.float32)
    no = N - k + 1
    ref = np.zeros((Sn, fo, no, no))
    for a in range(k):
        for b in range(k):
            ref += np.einsum("sipq,ji->sjpq", x[:, :, a:a + no, b:b + no].astype(np.float64), w[:, :, a, b].astype(np.float64))
    def planar(spec):
        return np.ascontiguousarray(np.stack([spec.real, spec.imag], -1).astype(np.float32))
    xs = planar(reference_spectrum_rect(x.reshape(-1, N, N), N))
    ws = planar(reference_spectrum_rect(w.reshape(-1, k, k), N))
    M = Sn * fo
    dst = np.full((M, no, no), np.nan, np.float32)
    assert replay.replay_ifft2d_c2r_crop_fused3(N, xs.ctypes.data_as(FP), ws.ctypes.data_as(FP), dst.ctypes.data_as(FP),
                                               M, fo, Sn * f, fo * f, no, no) == 0
    assert np.abs(dst.reshape(ref.shape) - ref).max() <= 2e-5 * np.abs(ref).max(), N


def test_tiled_forward_with_tiles_numbered_by_class(replay):
    """The forward transform of windows numbered class by class is the row-major one, reordered."""
    rng = np.random.default_rng(77)
    N, k, S, C, H, W = 16, 4, 2, 3, 50, 37
    L = N - k + 1
    ty, tx = -(-(H - k + 1) // L), -(-(W - k + 1) // L)
    M = S * ty * tx * C
    B = N * N // 2 + 2
    img = rng.uniform(-1, 1, (S, C, H, W)).astype(np.float32)
    out = []
    for by_class in (0, 1):
        spec = np.full((B, M, 2), np.nan, np.float32)
        assert replay.replay_fft2d_r2c_tiled(N, img.ctypes.data_as(FP), spec.ctypes.data_as(FP), M, N, N, H, W, C,
                                             tx, ty * tx, L, L, 0, 0, by_class) == 0
        out.append(spec.reshape(B, S, ty * tx, C, 2))
    row_major = tiles_in_order(ty, tx, 0)
    perm = [row_major.index(p) for p in tiles_in_order(ty, tx, 1)]
    # (to rounding: two maps share a complex transform, and the reordering changes the pairs when C is odd)
    assert not np.isnan(out[1]).any() and np.abs(out[1] - out[0][:, :, perm]).max() <= 3e-6 * np.abs(out[0]).max()

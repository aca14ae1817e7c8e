// Batched 2-D real-to-complex FFT of zero-padded maps, and the complex-to-real
// inverse fused with cropping (paper Sec. 2.2: transform every map once, crop
// the circular result; Sec. 2.3: a 2-D FFT is two sets of 1-D FFTs).
//
// Spectrum layout ("bin-major"): spec[c * M + m] is stored bin c of map m, complex
// interleaved.  A real map determines only half of its N x N spectrum (Sec. 2.3,
// symmetry of FFTs of real inputs).  Stored are exactly the bins that are not the
// conjugate of another stored bin, B = N*N/2 + 2 of them, in this order:
//     c in [0, N/2]            (ky = 0,   kx = c)
//     c in [N/2+1, N+1]        (ky = N/2, kx = c - (N/2+1))
//     c = N+2 + (ky-1)*N + kx  (ky in [1, N/2-1], kx in [0, N))
// (rows ky = 0 and ky = N/2 are Hermitian in kx, so only kx <= N/2 is kept).
// For a fixed bin the M maps are contiguous, which makes every bin a dense
// row-major matrix for the per-frequency contraction.
//
// One workgroup transforms T consecutive maps so that each bin is written (or
// read) as one contiguous run of T complex numbers.  The work is two phases
// separated by a workgroup barrier:
//
//   forward  A: lane <-> (map pair, column x).  Two real maps are packed as
//               one complex column (re = map a, im = map b), transformed along
//               y in registers, and split back into the two half spectra.
//            B: lane <-> (row ky, map).  Complex transform along x in
//               registers, then the bin-major store with lanes along maps.
//               The purely real rows ky = 0 and ky = N/2 of a map are packed
//               into one complex row ("row 0") and split after the transform.
//   inverse  runs the same two phases backwards and stores only the cropped
//            window, scaled by 1/N^2.
//
// Between the phases the data sits in LDS as lds[r][x][m] (m fastest) with
// strides padded so that both phases touch distinct banks.  With ROUNDS = 2 the
// rows go through LDS in two halves, rows [0, N/4) first, then [N/4, N/2), which
// halves the LDS of a workgroup (at N = 64 the whole tile would not fit).  The
// lanes form two teams, one per half.  LDS is only a hand-over point: forward,
// a team copies its rows from LDS into registers and the next half can be written
// at once, so both teams run their x-transforms and stores side by side; inverse,
// both teams load and transform their rows side by side and only take turns
// writing them to LDS.
//
// Each phase step is a plain function of (thread id, block id, per-lane state):
// the device kernels call them around __syncthreads(), and a host build replays
// them in loops to check the index arithmetic without a GPU.
#pragma once
#include "fft_core.hpp"

namespace fftconv {

// Maps larger than the largest transform are cut into tiles (overlap-save, see the tiled
// kernels below).  Transform m of a tiled tensor [S][C][H][W] is tile t of image s * C + c with
//     m = (s * tiles + t) * C + c,   t = ty * tiles_x + tx,
// i.e. the tiles of a sample are extra samples for the contraction.  A tile's window starts
// at (ty * step_y + org_y, tx * step_x + org_x) of its image.
struct Tiling {
    int H, W;             // image size
    int C;                // images per sample (f or f')
    int tiles_x, tiles;   // tiles per image row, tiles per image
    int step_y, step_x;   // distance between neighbouring tile origins
    int org_y, org_x;     // offset of the first origin (0, or -(k-1) for the windows of bprop)
    // 0: tile t is (t / tiles_x, t % tiles_x).  1: the tiles are numbered parity class by parity class
    // (class 2 * (ty % 2) + tx % 2, classes in order 0..3, row-major inside a class), so that the
    // transforms an overlap-add launch reads are neighbours in the spectrum.
    int by_class;
};

// Row and column of tile t of a Tiling.
FC_HD void tile_row_col(int t, const Tiling &tl, int &ty, int &tx)
{
    if (!tl.by_class) {
        ty = t / tl.tiles_x;
        tx = t % tl.tiles_x;
        return;
    }
    const int tiles_y = tl.tiles / tl.tiles_x;
    const int cy0 = (tiles_y + 1) / 2, cx0 = (tl.tiles_x + 1) / 2, cx1 = tl.tiles_x / 2;
    const int n0 = cy0 * cx0, n1 = cy0 * cx1, n2 = (tiles_y / 2) * cx0;
    int cls = 0, local = t;
    if (local >= n0) { local -= n0; cls = 1; }
    if (cls == 1 && local >= n1) { local -= n1; cls = 2; }
    if (cls == 2 && local >= n2) { local -= n2; cls = 3; }
    const int cx = (cls % 2) ? cx1 : cx0;
    ty = 2 * (local / cx) + cls / 2;
    tx = 2 * (local % cx) + cls % 2;
}

// First tile number of parity class cls under by_class numbering.
FC_HD int tile_class_start(int cls, const Tiling &tl)
{
    const int tiles_y = tl.tiles / tl.tiles_x;
    const int cy0 = (tiles_y + 1) / 2, cx0 = (tl.tiles_x + 1) / 2, cx1 = tl.tiles_x / 2;
    const int n0 = cy0 * cx0, n1 = cy0 * cx1, n2 = (tiles_y / 2) * cx0;
    return cls == 0 ? 0 : (cls == 1 ? n0 : (cls == 2 ? n0 + n1 : n0 + n1 + n2));
}

struct FwdArgs {
    const float *src;     // [M][ext_y][ext_x] real maps (tiled kernels: [S][C][H][W] images)
    cf *spec;             // [B][M] bin-major spectrum, B = N*N/2 + 2 stored bins
    int M;                // number of transforms
    int ext_y, ext_x;     // spatial extent of a map or window; everything beyond is zero padding
    Tiling t;             // read by the tiled kernels only
    int flip;             // untiled kernels: read every map rotated by 180 degrees (kernels of a true convolution)
};

struct InvArgs {
    const cf *spec;       // [B][M]
    float *dst;           // [M][crop_y][crop_x] (tiled kernels: [S][C][H][W] images)
    int M;
    int crop_y, crop_x;   // stored window [0,crop_y) x [0,crop_x)
                          // (tiled kernels: [c0_y, c0_y + crop_y) x [c0_x, c0_x + crop_x), stored at the tile origin)
    float scale;          // 1 / N^2
    int c0_y, c0_x;       // tiled kernels: first stored row / column of the transform's output
    Tiling t;             // read by the tiled kernels only
    int add;              // tiled kernels: 1 = overlap-add of the windows (see inv_y_finish_tiled), 0 = overwrite
    // Overlap-add launches handle one parity class of tiles, 2 * (ty % 2) + tx % 2 == parity, whose windows
    // do not overlap each other; they must run in the order parity = 0, 1, 2, 3, each complete before the
    // next (later classes add to what earlier ones stored; what dst held before the first is never read): the launch's transform ml = (s * cls_tiles + t') * C + c stands for tile
    // (2 * (t' / cls_cx) + parity / 2, 2 * (t' % cls_cx) + parity % 2) of sample s.  parity = -1: every
    // tile, in the order of the spectrum.
    int parity, cls_cx, cls_tiles;
    int bin_stride;       // transforms per bin in spec (equals M unless the launch handles one class)
    int flip;             // untiled kernels: store every window rotated by 180 degrees
    // Read by the fused kernels only (fprop of a layer with very few input maps): instead of
    // reading `spec`, bin c of output map m = s * fo + j is formed on the fly as
    // sum_i xs[c * Mx + s * F + i] * conj(wsp[c * Mw + j * F + i]), the product of Sec. 2.2.
    // These kernels need fo to be a multiple of T (the T maps of a workgroup then share a sample)
    // and F * B complex numbers to fit the workgroup's LDS buffer.
    const cf *xs, *wsp;   // spectra of x [B][Mx] and of w [B][Mw]
    int fo, Mx, Mw;       // output maps per sample; transforms in xs (samples x F) and in wsp (fo x F)
    int groups_per_sample;   // fo / T, or 0 to keep the plain order of the map groups (see fused_block_order)
};

struct TileOrigin {
    int image, oy, ox;
};

// Position in the spectrum (and in the order tile_origin expects) of transform ml of a launch.
FC_HD int launch_to_spectrum_index(int ml, const InvArgs &a)
{
    if (a.parity < 0) return ml;
    const int C = a.t.C, sp = ml / C, c = ml % C;
    const int s = sp / a.cls_tiles, tc = sp % a.cls_tiles;
    if (a.t.by_class) return (s * a.t.tiles + tile_class_start(a.parity, a.t) + tc) * C + c;
    const int ty = 2 * (tc / a.cls_cx) + a.parity / 2, tx = 2 * (tc % a.cls_cx) + a.parity % 2;
    return (s * a.t.tiles + ty * a.t.tiles_x + tx) * C + c;
}

FC_HD TileOrigin tile_origin(int m, const Tiling &t)
{
    const int sp = m / t.C, c = m % t.C;
    const int s = sp / t.tiles, tile = sp % t.tiles;
    TileOrigin o;
    o.image = s * t.C + c;
    int ty, tx;
    tile_row_col(tile, t, ty, tx);
    o.oy = ty * t.step_y + t.org_y;
    o.ox = tx * t.step_x + t.org_x;
    return o;
}

template <int N_, int T_, int NX_, int ROUNDS_ = 1>
struct TileGeom {
    static constexpr int N = N_;     // transform size
    static constexpr int T = T_;     // maps per workgroup (even)
    static constexpr int NX = NX_;   // columns that can be non-zero (forward) / are needed (inverse)
    static constexpr int ROUNDS = ROUNDS_;             // LDS hand-overs between the phases
    static constexpr int ROWS = N / 2;                 // packed row 0 + rows 1..N/2-1
    static constexpr int RPR = ROWS / ROUNDS;          // rows per round
    static constexpr int THREADS = T * ROWS;           // lanes per workgroup
    static constexpr int XTHREADS = T * RPR;           // lanes of one x-phase team: (row of its half, map)
    static constexpr int SX = T + 1;                   // complex elements between consecutive x
    static constexpr int SR_BASE = NX * SX;
    // row stride: congruent to T modulo 32 complex (= 64 dwords) so that the row groups
    // sharing a half-wave in the x-phase start T complex apart in bank space
    static constexpr int SR = SR_BASE + ((((T - SR_BASE) % 32) + 32) % 32);
    static constexpr int LDS_ELEMS = RPR * SR;
    static constexpr int LDS_BYTES = LDS_ELEMS * 8;
    static constexpr int YITEMS = (T / 2) * NX;        // lanes active in the y-phase: (map pair, column)
    // waves per SIMD the register allocation should allow (what LDS lets a CU hold):
    // N = 64 and 56 need 128 and 112 registers for one transform alone, so two; N = 48 (96 registers,
    // two workgroups of six waves per CU) and N = 40 (two of five waves) three; N = 32 fits four
    static constexpr int WAVES_PER_SIMD = N >= 56 ? 2 : (N >= 40 ? 3 : (N == 32 && ROUNDS == 2 ? 4 : 1));
    static_assert(T % 2 == 0, "maps are processed in pairs");
    static_assert(NX <= N, "extent class cannot exceed the transform size");
    static_assert(ROWS % ROUNDS == 0 && YITEMS <= THREADS, "geometry");
};

// ------------------------------------------------------------------ forward

// y-phase, step 1: load the two columns of a map pair, transform along y.  Leaves the
// bit-reversed transform in z.  Returns false for lanes without a column.
template <class G>
FC_HD bool fwd_y_compute(int tid, int blk, const FwdArgs &a, cf (&z)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    if (tid >= G::YITEMS) return false;
    const int p = tid / NX, x = tid % NX;
    const int ma = blk * G::T + 2 * p, mb = ma + 1;
    // Loads are unconditional from clamped (always valid) addresses and masked
    // afterwards, so that they issue back to back; rows beyond the extent are
    // skipped by a wave-uniform branch.
    const bool va = (ma < a.M) && (x < a.ext_x), vb = (mb < a.M) && (x < a.ext_x);
    const int xc = x < a.ext_x ? x : a.ext_x - 1;
    const int mac = ma < a.M ? ma : a.M - 1, mbc = mb < a.M ? mb : a.M - 1;
    // element (y, x) of the transform's input is map element (y, x), or (ext_y-1-y, ext_x-1-x) if flipped
    const int first = a.flip ? (a.ext_y - 1) * a.ext_x + (a.ext_x - 1 - xc) : xc;
    const int rstep = a.flip ? -a.ext_x : a.ext_x;
    const float *pa = a.src + ((size_t)mac * a.ext_y) * a.ext_x + first;
    const float *pb = a.src + ((size_t)mbc * a.ext_y) * a.ext_x + first;
    float fa[NX], fb[NX];
    static_for<0, NX>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        if (y < a.ext_y) {
            fa[y] = pa[y * rstep];
            fb[y] = pb[y * rstep];
        } else {
            fa[y] = 0.0f;
            fb[y] = 0.0f;
        }
    });
    static_for<0, NX>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        z[y] = mk(va ? fa[y] : 0.0f, vb ? fb[y] : 0.0f);
    });
    fft_dif<N, false, ~low_mask(NX)>(z);
    return true;
}

// Tiled variant of step 1: the column comes from a window of a larger image.  Window rows
// and columns outside the image (the windows of bprop start k-1 before the tile, the last
// tiles of a row or column stick out) and beyond `ext` read as zero.  Loads are unconditional
// from clamped addresses, masked afterwards.
template <class G>
FC_HD bool fwd_y_compute_tiled(int tid, int blk, const FwdArgs &a, cf (&z)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    if (tid >= G::YITEMS) return false;
    const int p = tid / NX, x = tid % NX;
    float f[2][NX];
    static_for<0, 2>([&](auto wi) {
        constexpr int which = decltype(wi)::value;
        const int m = blk * G::T + 2 * p + which;
        const TileOrigin o = tile_origin(m < a.M ? m : a.M - 1, a.t);
        const int xg = o.ox + x;
        const bool vx = (m < a.M) && (x < a.ext_x) && xg >= 0 && xg < a.t.W;
        const int xc = xg < 0 ? 0 : (xg < a.t.W ? xg : a.t.W - 1);
        // valid window rows [ylo, yhi)
        const int ylo = o.oy < 0 ? -o.oy : 0;
        const int yhi = a.ext_y < a.t.H - o.oy ? a.ext_y : a.t.H - o.oy;
        const float *col = a.src + (size_t)o.image * a.t.H * a.t.W + xc;
        static_for<0, NX>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            int r = o.oy + (y < ylo ? ylo : (y < yhi ? y : yhi - 1));
            r = r < 0 ? 0 : (r < a.t.H ? r : a.t.H - 1);
            f[which][y] = col[(size_t)r * a.t.W];
        });
        static_for<0, NX>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            if (!(vx && y >= ylo && y < yhi)) f[which][y] = 0.0f;
        });
    });
    static_for<0, NX>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        z[y] = mk(f[0][y], f[1][y]);
    });
    fft_dif<N, false, ~low_mask(NX)>(z);
    return true;
}

// y-phase, step 2: split the packed transform into the two maps' half spectra and hand
// rows [round * RPR, (round + 1) * RPR) to LDS.
template <class G, int ROUND>
FC_HD void fwd_y_write(int tid, const cf (&z)[G::N], cf *lds)
{
    constexpr int N = G::N, NX = G::NX;
    const int p = tid / NX, x = tid % NX;
    cf *base = lds + x * G::SX + 2 * p;
    static_for<ROUND * G::RPR, (ROUND + 1) * G::RPR>([&](auto ri) {
        constexpr int r = decltype(ri)::value;
        constexpr int slot = r - ROUND * G::RPR;
        if constexpr (r == 0) {   // packed row 0: (ky = 0, ky = N/2), both real for a real map
            const cf z0 = z[brev<N>(0)], zh = z[brev<N>(N / 2)];
            base[0] = mk(z0.x, zh.x);
            base[1] = mk(z0.y, zh.y);
        } else {
            const cf zk = z[brev<N>(r)], zn = z[brev<N>(N - r)];
            // A = (Z[k] + conj Z[N-k]) / 2,  B = (Z[k] - conj Z[N-k]) / (2i)
            base[slot * G::SR + 0] = mk(0.5f * (zk.x + zn.x), 0.5f * (zk.y - zn.y));
            base[slot * G::SR + 1] = mk(0.5f * (zk.y + zn.y), 0.5f * (zn.x - zk.x));
        }
    });
}

// x-phase, step 1: lane xt = (slot, map) of its team copies its row from LDS into registers.
template <class G>
FC_HD void fwd_x_read(int xt, const cf *lds, cf (&v)[G::N])
{
    const int slot = xt / G::T, m = xt % G::T;
    const cf *base = lds + slot * G::SR + m;
    static_for<0, G::NX>([&](auto xi) {
        constexpr int x = decltype(xi)::value;
        v[x] = base[x * G::SX];
    });
}

// x-phase, step 2: transform the row along x, store bin-major.  `round` is the team's half.
template <class G>
FC_HD void fwd_x_finish(int xt, int blk, int round, const FwdArgs &a, cf (&v)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    const int slot = xt / G::T, m = xt % G::T;
    const int r = round * G::RPR + slot;
    const int mg = blk * G::T + m;
    fft_dif<N, false, ~low_mask(NX)>(v);
    if (mg >= a.M) return;
    cf *out = a.spec + mg;
    const size_t M = (size_t)a.M;
    if (r != 0) {
        static_for<0, N>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            out[((size_t)(N + 2) + (size_t)(r - 1) * N + kx) * M] = v[brev<N>(kx)];
        });
    } else {
        // C = FFT(row0 + i rowH)  ->  row0[k] = (C[k] + conj C[-k]) / 2,  rowH[k] = (C[k] - conj C[-k]) / (2i);
        // both rows are Hermitian in k, only k <= N/2 is stored
        static_for<0, N / 2 + 1>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            const cf c = v[brev<N>(kx)], d = v[brev<N>((N - kx) % N)];
            out[(size_t)kx * M] = mk(0.5f * (c.x + d.x), 0.5f * (c.y - d.y));
            out[(size_t)(N / 2 + 1 + kx) * M] = mk(0.5f * (c.y + d.y), 0.5f * (d.x - c.x));
        });
    }
}

// ------------------------------------------------------------------ inverse

// Fused kernels, step 0: copy the part of xs that belongs to the workgroup's sample,
// xs[c][s * F + i] for every stored bin c, to xl[c * F + i] in LDS.  Every lane would
// otherwise load these values itself, T times over (measured on S=128, f=3, f'=96, N=64:
// 99 -> 91 us for the kernel).
template <class G, int FUSE>
FC_HD void fused_stage_x(int tid, int blk, const InvArgs &a, cf *xl)
{
    constexpr int B = G::N * G::N / 2 + 2;
    const cf *xp = a.xs + (size_t)((blk * G::T) / a.fo) * FUSE;
    cf tmp[(B * FUSE + G::THREADS - 1) / G::THREADS];
    static_for<0, (B * FUSE + G::THREADS - 1) / G::THREADS>([&](auto pi) {
        constexpr int p = decltype(pi)::value;
        const int e = p * G::THREADS + tid;
        const int ec = e < B * FUSE ? e : B * FUSE - 1;
        tmp[p] = xp[(size_t)(ec / FUSE) * a.Mx + ec % FUSE];
    });
    static_for<0, (B * FUSE + G::THREADS - 1) / G::THREADS>([&](auto pi) {
        constexpr int p = decltype(pi)::value;
        const int e = p * G::THREADS + tid;
        if (e < B * FUSE) xl[e] = tmp[p];
    });
}

// x-phase, step 1: lane xt = (slot, map) of its team loads a row of one map's spectrum
// (natural order in v).
// FUSE = F > 0: the bins are not read but formed from the copy of the sample's x spectrum that
// fused_stage_x made at xl and from the spectrum of w (see InvArgs).
template <class G, int FUSE = 0>
FC_HD void inv_x_load(int xt, int blk, int round, const InvArgs &a, const cf *xl, cf (&v)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    const int slot = xt / G::T, m = xt % G::T;
    const int r = round * G::RPR + slot;
    const int mg = blk * G::T + m;
    // Lanes beyond the last map read the last map's bins (valid memory) instead of
    // branching around each load; what they compute is never stored.
    const int mc = launch_to_spectrum_index(mg < a.M ? mg : a.M - 1, a);
    const size_t M = (size_t)a.bin_stride;
    const cf *src = nullptr, *xp = nullptr, *wp = nullptr;
    if constexpr (FUSE > 0) {
        xp = xl;
        wp = a.wsp + (size_t)(mc % a.fo) * FUSE;
    } else {
        src = a.spec + mc;
    }
    struct Bins {
        const cf *src, *xp, *wp;
        size_t M, Mw;
        FC_HD cf operator[](size_t c) const   // stored bin c of the lane's map
        {
            if constexpr (FUSE == 0) {
                return src[c * M];
            } else {
                const cf *x = xp + c * FUSE, *w = wp + c * Mw;
                cf acc = mk(x[0].x * w[0].x + x[0].y * w[0].y, x[0].y * w[0].x - x[0].x * w[0].y);   // x conj(w)
                static_for<1, FUSE>([&](auto ii) {
                    constexpr int i = decltype(ii)::value;
                    acc = mk(acc.x + (x[i].x * w[i].x + x[i].y * w[i].y), acc.y + (x[i].y * w[i].x - x[i].x * w[i].y));
                });
                return acc;
            }
        }
    };
    const Bins in{src, xp, wp, M, (size_t)a.Mw};
    if (r != 0) {
        static_for<0, N>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            v[kx] = in[(size_t)(N + 2) + (size_t)(r - 1) * N + kx];
        });
    } else {
        // rows ky = 0 and ky = N/2 are Hermitian in kx, so their inverse transforms are
        // real: send both through one complex transform as row0 + i rowH, rebuilding the
        // bins kx > N/2 that are not stored from their conjugates
        cf y0[N / 2 + 1], yh[N / 2 + 1];
        static_for<0, N / 2 + 1>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            y0[kx] = in[(size_t)kx];
            yh[kx] = in[(size_t)(N / 2 + 1 + kx)];
        });
        static_for<0, N / 2 + 1>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            v[kx] = mk(y0[kx].x - yh[kx].y, y0[kx].y + yh[kx].x);                 // y0 + i yh
            if constexpr (kx > 0 && kx < N / 2)
                v[N - kx] = mk(y0[kx].x + yh[kx].y, yh[kx].x - y0[kx].y);        // conj y0 + i conj yh
        });
        // The two branches end in stores to different elements of v.  Left alone, the compiler merges
        // them into one store through a selected address, after which those elements live in scratch
        // memory instead of registers; an empty statement it must keep makes the branch ends differ.
        asm volatile("");
    }
}

// x-phase, step 1b: inverse transform of the row along kx.  Leaves the bit-reversed transform in v.
template <class G>
FC_HD void inv_x_transform(cf (&v)[G::N])
{
    fft_dif<G::N, true, 0, first_outputs_mask<G::N>(G::NX)>(v);
}

// x-phase, step 2: hand the needed columns of the row to LDS.
template <class G>
FC_HD void inv_x_write(int xt, cf *lds, const cf (&v)[G::N])
{
    constexpr int N = G::N;
    const int slot = xt / G::T, m = xt % G::T;
    cf *base = lds + slot * G::SR + m;
    static_for<0, G::NX>([&](auto xi) {
        constexpr int x = decltype(xi)::value;
        base[x * G::SX] = v[brev<N>(x)];
    });
}

// y-phase, step 1 (per round): collect rows [round * RPR, (round + 1) * RPR) of the map pair's
// column from LDS into the packed spectrum z (natural order).
template <class G, int ROUND>
FC_HD void inv_y_gather(int tid, const cf *lds, cf (&z)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    if (tid >= G::YITEMS) return;
    const int p = tid / NX, x = tid % NX;
    const cf *base = lds + x * G::SX + 2 * p;
    static_for<ROUND * G::RPR, (ROUND + 1) * G::RPR>([&](auto ri) {
        constexpr int r = decltype(ri)::value;
        constexpr int slot = r - ROUND * G::RPR;
        if constexpr (r == 0) {
            const cf ra = base[0], rb = base[1];    // (row 0, row N/2) of map a / map b, all real
            z[0] = mk(ra.x, rb.x);
            z[N / 2] = mk(ra.y, rb.y);
        } else {
            const cf A = base[slot * G::SR + 0], B = base[slot * G::SR + 1];
            z[r] = mk(A.x - B.y, A.y + B.x);        // A + i B
            z[N - r] = mk(A.x + B.y, B.x - A.y);    // conj A + i conj B
        }
    });
}

// Stores one cropped output column (rows y < crop of one map at one x), scaled;
// with ACC the old values are all loaded first, then added, then stored.
template <class G, bool ACC, class Get>
FC_HD void store_column(float *col, int rstep, bool valid, const InvArgs &a, Get &&get)
{
    if (!valid) return;
    float old[G::NX];
    if constexpr (ACC) {
        static_for<0, G::NX>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            old[y] = (y < a.crop_y) ? col[y * rstep] : 0.0f;
        });
    }
    static_for<0, G::NX>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        if (y < a.crop_y) {
            if constexpr (ACC) col[y * rstep] = old[y] + get(yi) * a.scale;
            else col[y * rstep] = get(yi) * a.scale;
        }
    });
}

// y-phase, step 2: inverse transform along y of the packed pair, store the cropped columns.
template <class G, bool ACC>
FC_HD void inv_y_finish(int tid, int blk, const InvArgs &a, cf (&z)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    if (tid >= G::YITEMS) return;
    const int p = tid / NX, x = tid % NX;
    const int ma = blk * G::T + 2 * p, mb = ma + 1;
    fft_dif<N, true, 0, first_outputs_mask<N>(NX)>(z);
    if (x >= a.crop_x) return;
    // output (y, x) goes to window element (y, x), or (crop_y-1-y, crop_x-1-x) if flipped
    const int first = a.flip ? (a.crop_y - 1) * a.crop_x + (a.crop_x - 1 - x) : x;
    const int rstep = a.flip ? -a.crop_x : a.crop_x;
    store_column<G, ACC>(a.dst + ((size_t)ma * a.crop_y) * a.crop_x + first, rstep, ma < a.M, a, [&](auto yi) {
        return z[brev<N>(decltype(yi)::value)].x;
    });
    store_column<G, ACC>(a.dst + ((size_t)mb * a.crop_y) * a.crop_x + first, rstep, mb < a.M, a, [&](auto yi) {
        return z[brev<N>(decltype(yi)::value)].y;
    });
}

// Tiled variant of step 2: rows and columns [c0, c0 + crop) of the transform's output go to
// the tile's place in a larger image, clipped at the image border.  With ADD (and a.add) the windows of
// neighbouring tiles overlap and are summed (overlap-add): one launch handles the tiles of one parity
// class, which do not overlap each other.
template <class G, bool ADD = false>
FC_HD void inv_y_finish_tiled(int tid, int blk, const InvArgs &a, cf (&z)[G::N])
{
    constexpr int N = G::N, NX = G::NX;
    static_assert(NX == N, "tiled transforms keep every output column");
    if (tid >= G::YITEMS) return;
    const int p = tid / NX, x = tid % NX;
    fft_dif<N, true>(z);
    const int xs = x - a.c0_x;
    if (xs < 0 || xs >= a.crop_x) return;
    static_for<0, 2>([&](auto wi) {
        constexpr int which = decltype(wi)::value;
        const int m = blk * G::T + 2 * p + which;
        if (m >= a.M) return;
        const TileOrigin o = tile_origin(launch_to_spectrum_index(m, a), a.t);
        if (o.ox + xs >= a.t.W) return;
        const int rows = a.crop_y < a.t.H - o.oy ? a.crop_y : a.t.H - o.oy;
        float *col = a.dst + ((size_t)o.image * a.t.H + o.oy) * a.t.W + o.ox + xs;
        if constexpr (ADD) {
            // Overlap-add (c0 = 0, windows placed at multiples of the step).  A pixel lies in the windows of up
            // to four tiles, one per parity class; the launches run in class order 0..3, and the tile of the
            // lowest class among those covering a pixel stores its value plainly while the later ones add to
            // what they find.  So dx needs no clearing, only the overlap strips are ever read, and every sum
            // has a fixed order.  With a = ty % 2, b = tx % 2 and classes 2a + b, a tile is not the first
            // writer of a pixel exactly if a horizontal neighbour covers it and b = 1, or a vertical one and a = 1.
            const int ty = o.oy / a.t.step_y, tx = o.ox / a.t.step_x, tiles_y = a.t.tiles / a.t.tiles_x;
            const int ovy = N - a.t.step_y, ovx = N - a.t.step_x;   // kh - 1, kw - 1: rows / columns shared with a neighbour
            const bool add_x = (tx & 1) && ((xs < ovx) || (xs >= a.t.step_x && tx + 1 < a.t.tiles_x));
            const bool odd_ty = (ty & 1) != 0, below = ty + 1 < tiles_y;
            // the old values of a group of rows are all loaded before the first of them is needed, so that
            // their latencies overlap instead of adding up row by row
            constexpr int GROUP = N < 16 ? N : 16;
            static_for<0, (N + GROUP - 1) / GROUP>([&](auto gi) {
                constexpr int y0 = decltype(gi)::value * GROUP;
                constexpr int CNT = N - y0 < GROUP ? N - y0 : GROUP;
                float old[CNT];
                static_for<0, CNT>([&](auto yi) {
                    constexpr int y = y0 + decltype(yi)::value;
                    const bool adds = add_x || (odd_ty && (y < ovy || (y >= a.t.step_y && below)));
                    old[y - y0] = (y < rows && adds) ? col[(size_t)y * a.t.W] : 0.0f;
                });
                static_for<0, CNT>([&](auto yi) {
                    constexpr int y = y0 + decltype(yi)::value;
                    const cf v = z[brev<N>(y)];
                    if (y < rows) col[(size_t)y * a.t.W] = old[y - y0] + (which == 0 ? v.x : v.y) * a.scale;
                });
            });
            return;
        }
        static_for<0, N>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            const int ys = y - a.c0_y;
            if (ys >= 0 && ys < rows) {
                const cf v = z[brev<N>(y)];
                col[(size_t)ys * a.t.W] = (which == 0 ? v.x : v.y) * a.scale;
            }
        });
    });
}

// The order of steps and barriers of one workgroup, shared by the device kernels and the
// host replay.  `sync` is __syncthreads() on the device; the host replay runs every step for
// all lanes before the next one, which is what a barrier after each step guarantees.
// Lane tid belongs to team tid / XTHREADS and is lane xt = tid % XTHREADS of it.
//   forward: y_compute | per round r: (barrier,) y_write<r>, barrier, team r: x_read | x_finish
//   inverse: (fused: stage_x, barrier,) x_load (, barrier) | x_transform |
//            per round r: (barrier,) team r: x_write, barrier, y_gather<r> | y_finish

#if defined(__HIPCC__)
// Workgroups are dealt round-robin to the 8 XCDs of an MI355X (each with its own L2).  Renumber
// them so that every XCD walks a contiguous range of map groups: neighbouring groups, whose
// bin runs are neighbours in memory, then go through the same L2 (measured at N = 64 on 32768
// maps in isolation: forward 243 -> 229 us, inverse 276 -> 264 us; 2-5 % inside a full step).
__device__ __forceinline__ int xcd_contiguous_block()
{
    constexpr int kXcdCount = 8;
    const int total = (int)gridDim.x, id = (int)blockIdx.x;
    const int xcd = id % kXcdCount, slot = id / kXcdCount;
    const int per = total / kXcdCount, rem = total % kXcdCount;
    return xcd * per + (xcd < rem ? xcd : rem) + slot;
}

// Order of the map groups in a fused kernel.  A group reads its sample's part of xs and its
// T output maps' part of wsp, every bin of both.  Walking the groups sample by sample makes the
// groups that run together cover all of wsp (4.7 MB for f = 3, f' = 96, N = 64, more than an
// XCD's 4 MB of L2, which then misses all the time: measured 129 MB fetched per launch for 11 MB
// of operands).  Inside chunks of 16 samples the groups are therefore walked output-map range
// first, so that the groups in flight share one or two ranges of wsp and 16 samples of xs.
__device__ __forceinline__ int fused_block_order(int blk, int groups_per_sample)
{
    if (groups_per_sample <= 1) return blk;
    const int chunk = 16 * groups_per_sample;
    const int c = blk / chunk, r = blk % chunk;
    if ((c + 1) * chunk > (int)gridDim.x) return blk;   // a ragged last chunk keeps its order
    return c * chunk + (r % 16) * groups_per_sample + r / 16;
}

// Steps 0 to 1b of one lane of a device workgroup (the host replay calls the steps one by one).
template <class G, int FUSE>
__device__ __forceinline__ void inv_x_phase(int tid, int xt, int blk, int team, const InvArgs &a, cf *lds, cf (&v)[G::N])
{
    if constexpr (FUSE > 0) {
        fused_stage_x<G, FUSE>(tid, blk, a, lds);
        __syncthreads();
        inv_x_load<G, FUSE>(xt, blk, team, a, lds, v);
        __syncthreads();   // the copy has been read: the buffer is free for the hand-over
    } else {
        inv_x_load<G, 0>(xt, blk, team, a, nullptr, v);
    }
    inv_x_transform<G>(v);
}

// Device kernels.  Launch with G::THREADS threads, ceil(M / G::T) blocks and G::LDS_BYTES
// of dynamic LDS.
// (the second launch bound is the number of waves per SIMD the register budget must allow)
template <class G, bool TILED = false>
__global__ __launch_bounds__(G::THREADS, G::WAVES_PER_SIMD) void fft2d_r2c_kernel(FwdArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    const int tid = (int)threadIdx.x, blk = xcd_contiguous_block();
    const int team = tid / G::XTHREADS, xt = tid % G::XTHREADS;
    cf z[G::N], v[G::N];
    const bool has = TILED ? fwd_y_compute_tiled<G>(tid, blk, a, z) : fwd_y_compute<G>(tid, blk, a, z);
    static_for<0, G::ROUNDS>([&](auto ri) {
        constexpr int r = decltype(ri)::value;
        if constexpr (r > 0) __syncthreads();   // the previous team has its rows in registers
        if (has) fwd_y_write<G, r>(tid, z, lds);
        __syncthreads();
        if (team == r) fwd_x_read<G>(xt, lds, v);
    });
    fwd_x_finish<G>(xt, blk, team, a, v);
}

template <class G, bool ACC, int FUSE = 0>   // ACC: dst += result instead of dst = result
__global__ __launch_bounds__(G::THREADS, G::WAVES_PER_SIMD) void ifft2d_c2r_crop_kernel(InvArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    const int tid = (int)threadIdx.x;
    const int blk = FUSE > 0 ? fused_block_order(xcd_contiguous_block(), a.groups_per_sample) : xcd_contiguous_block();
    const int team = tid / G::XTHREADS, xt = tid % G::XTHREADS;
    cf z[G::N], v[G::N];
    inv_x_phase<G, FUSE>(tid, xt, blk, team, a, lds, v);
    static_for<0, G::ROUNDS>([&](auto ri) {
        constexpr int r = decltype(ri)::value;
        if constexpr (r > 0) __syncthreads();   // every lane has gathered the previous rows
        if (team == r) inv_x_write<G>(xt, lds, v);
        __syncthreads();
        inv_y_gather<G, r>(tid, lds, z);
    });
    inv_y_finish<G, ACC>(tid, blk, a, z);
}

// Same schedule, output scattered to tiles of a larger image (never accumulating).
template <class G, int FUSE = 0, bool ADD = false>   // ADD: overlap-add of the windows (a.add must be set)
__global__ __launch_bounds__(G::THREADS, G::WAVES_PER_SIMD) void ifft2d_c2r_tiled_kernel(InvArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    const int tid = (int)threadIdx.x;
    const int blk = FUSE > 0 ? fused_block_order(xcd_contiguous_block(), a.groups_per_sample) : xcd_contiguous_block();
    const int team = tid / G::XTHREADS, xt = tid % G::XTHREADS;
    cf z[G::N], v[G::N];
    inv_x_phase<G, FUSE>(tid, xt, blk, team, a, lds, v);
    static_for<0, G::ROUNDS>([&](auto ri) {
        constexpr int r = decltype(ri)::value;
        if constexpr (r > 0) __syncthreads();
        if (team == r) inv_x_write<G>(xt, lds, v);
        __syncthreads();
        inv_y_gather<G, r>(tid, lds, z);
    });
    inv_y_finish_tiled<G, ADD>(tid, blk, a, z);
}
#endif

}  // namespace fftconv

// Host replay of the FFT kernels' two phases (no GPU, no HIP): every block and
// every lane is run in a loop, phase by phase, on an ordinary array standing in
// for LDS.  Used only by CPU tests to check the kernels' index arithmetic and
// the transform conventions against a naive DFT; it is not part of the product
// path and is not linked into the GPU library.
#include <array>
#include <cstring>
#include <vector>

#include "fft_dispatch.hpp"
#include "fft_quad_kernels.hpp"

using namespace fftconv;

template <class G>
using LaneRegs = std::vector<std::array<cf, G::N>>;

template <class G>
static cf (&regs(LaneRegs<G> &r, int tid))[G::N]
{
    return reinterpret_cast<cf(&)[G::N]>(*r[tid].data());
}

template <class G, bool TILED = false>
static void replay_forward(const FwdArgs &a)
{
    std::vector<cf> lds(G::LDS_ELEMS);
    LaneRegs<G> z(G::THREADS), v(G::THREADS);
    std::vector<char> has(G::THREADS);
    const int blocks = (a.M + G::T - 1) / G::T;
    for (int blk = 0; blk < blocks; ++blk) {
        for (int tid = 0; tid < G::THREADS; ++tid) {
            // poison: a read of something an earlier step did not write shows up as NaN
            std::memset(z[tid].data(), 0xFF, sizeof(cf) * G::N);
            std::memset(v[tid].data(), 0xFF, sizeof(cf) * G::N);
            has[tid] = TILED ? fwd_y_compute_tiled<G>(tid, blk, a, regs<G>(z, tid))
                             : fwd_y_compute<G>(tid, blk, a, regs<G>(z, tid));
        }
        static_for<0, G::ROUNDS>([&](auto ri) {
            constexpr int r = decltype(ri)::value;
            std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
            for (int tid = 0; tid < G::THREADS; ++tid)
                if (has[tid]) fwd_y_write<G, r>(tid, regs<G>(z, tid), lds.data());
            for (int tid = 0; tid < G::THREADS; ++tid)
                if (tid / G::XTHREADS == r) fwd_x_read<G>(tid % G::XTHREADS, lds.data(), regs<G>(v, tid));
        });
        for (int tid = 0; tid < G::THREADS; ++tid)
            fwd_x_finish<G>(tid % G::XTHREADS, blk, tid / G::XTHREADS, a, regs<G>(v, tid));
    }
}

template <class G, bool TILED = false, int FUSE = 0>
static void replay_inverse(const InvArgs &a, bool acc)
{
    std::vector<cf> lds(G::LDS_ELEMS);
    LaneRegs<G> z(G::THREADS), v(G::THREADS);
    const int blocks = (a.M + G::T - 1) / G::T;
    for (int blk = 0; blk < blocks; ++blk) {
        for (int tid = 0; tid < G::THREADS; ++tid) {
            std::memset(z[tid].data(), 0xFF, sizeof(cf) * G::N);
            std::memset(v[tid].data(), 0xFF, sizeof(cf) * G::N);
        }
        if constexpr (FUSE > 0) {
            std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
            for (int tid = 0; tid < G::THREADS; ++tid) fused_stage_x<G, FUSE>(tid, blk, a, lds.data());
        }
        for (int tid = 0; tid < G::THREADS; ++tid) {
            inv_x_load<G, FUSE>(tid % G::XTHREADS, blk, tid / G::XTHREADS, a, lds.data(), regs<G>(v, tid));
            inv_x_transform<G>(regs<G>(v, tid));
        }
        static_for<0, G::ROUNDS>([&](auto ri) {
            constexpr int r = decltype(ri)::value;
            std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
            for (int tid = 0; tid < G::THREADS; ++tid)
                if (tid / G::XTHREADS == r) inv_x_write<G>(tid % G::XTHREADS, lds.data(), regs<G>(v, tid));
            for (int tid = 0; tid < G::THREADS; ++tid) inv_y_gather<G, r>(tid, lds.data(), regs<G>(z, tid));
        });
        for (int tid = 0; tid < G::THREADS; ++tid) {
            if constexpr (TILED) {
                if (a.add) inv_y_finish_tiled<G, true>(tid, blk, a, regs<G>(z, tid));
                else inv_y_finish_tiled<G, false>(tid, blk, a, regs<G>(z, tid));
            }
            else if (acc) inv_y_finish<G, true>(tid, blk, a, regs<G>(z, tid));
            else inv_y_finish<G, false>(tid, blk, a, regs<G>(z, tid));
        }
    }
}

// The quad-split inverse: the cross-lane sums of a quad, two DPP adds on the device, are formed here from the
// four lanes' stored partial results in the same order, (a + b) + (c + d).
template <class G>
static void quad_sums(const std::vector<std::array<cf, G::M>> &part, int tid, cf (&out)[G::M])
{
    const int q0 = tid & ~3, q = tid & 3;
    for (int i = 0; i < G::M; ++i) {
        // lane q: (own + neighbour) + (the other pair's sum), each pair's sum formed the same way
        const cf own = part[q0 + q][i], nb = part[q0 + (q ^ 1)][i];
        const cf oa = part[q0 + (q ^ 2)][i], ob = part[q0 + (q ^ 3)][i];
        out[i] = (own + nb) + (oa + ob);
    }
}

template <class G>
static void replay_inverse_quad(const InvArgs &a, bool acc)
{
    std::vector<cf> lds(G::LDS_ELEMS);
    std::vector<std::array<cf, G::M>> part(G::THREADS);
    const int blocks = (a.M + G::T - 1) / G::T;
    for (int blk = 0; blk < blocks; ++blk) {
        std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
        for (int round = 0; round < G::ROUNDS; ++round) {
            for (int tid = 0; tid < G::THREADS; ++tid) {
                cf v[G::M];
                quad_inv_x_load<G>(tid, blk, round, a, v);
                quad_inv_x_partial<G>(tid, v, reinterpret_cast<cf(&)[G::M]>(*part[tid].data()));
            }
            for (int tid = 0; tid < G::THREADS; ++tid) {
                cf u[G::M];
                quad_sums<G>(part, tid, u);
                quad_inv_x_write<G>(tid, round, lds.data(), u);
            }
        }
        for (int tid = 0; tid < G::YITEMS; ++tid)
            quad_inv_y_partial<G>(tid, lds.data(), reinterpret_cast<cf(&)[G::M]>(*part[tid].data()));
        for (int tid = 0; tid < G::YITEMS; ++tid) {
            cf z[G::M];
            quad_sums<G>(part, tid, z);
            if (acc) quad_inv_y_store<G, true>(tid, blk, a, z);
            else quad_inv_y_store<G, false>(tid, blk, a, z);
        }
    }
}

extern "C" {

// Inverse + crop of the extent class N / 4 (crop <= N / 4) with each transform split over four lanes; N in 40, 48, 56, 64.
int replay_ifft2d_c2r_crop_quad(int N, const float *spec, float *dst, int M, int crop_y, int crop_x, int accumulate, int flip)
{
    InvArgs a{reinterpret_cast<const cf *>(spec), dst, M, crop_y, crop_x, 1.0f / (float)(N * N)};
    a.flip = flip;
    a.parity = -1;
    a.bin_stride = M;
    if (crop_y > N / 4 || crop_x > N / 4) return 2;
    switch (N) {
        case 40: replay_inverse_quad<QuadGeom<40, maps_per_block(40)>>(a, accumulate != 0); return 0;
        case 48: replay_inverse_quad<QuadGeom<48, maps_per_block(48)>>(a, accumulate != 0); return 0;
        case 56: replay_inverse_quad<QuadGeom<56, maps_per_block(56)>>(a, accumulate != 0); return 0;
        case 64: replay_inverse_quad<QuadGeom<64, maps_per_block(64)>>(a, accumulate != 0); return 0;
        default: return 1;
    }
}

int replay_fft_size(int n) { return fft_size_for(n); }
int replay_extent_class(int N, int ext) { return extent_class(N, ext); }
int replay_maps_per_block(int N) { return maps_per_block(N); }

// src: [M][ext_y][ext_x] floats; spec: [B][M] complex (2 floats each), B = N*N/2 + 2.
int replay_fft2d_r2c(int N, const float *src, float *spec, int M, int ext_y, int ext_x, int flip)
{
    FwdArgs a{src, reinterpret_cast<cf *>(spec), M, ext_y, ext_x};
    a.flip = flip;
    const int T = maps_per_block(N), NX = extent_class(N, ext_y > ext_x ? ext_y : ext_x);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && NX == nx_) { replay_forward<Geom<n_, t_, nx_>>(a); return 0; }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

int replay_ifft2d_c2r_crop(int N, const float *spec, float *dst, int M, int crop_y, int crop_x, int accumulate, int flip)
{
    InvArgs a{reinterpret_cast<const cf *>(spec), dst, M, crop_y, crop_x, 1.0f / (float)(N * N)};
    a.flip = flip;
    a.parity = -1;
    a.bin_stride = M;
    const int T = maps_per_block(N), NX = extent_class(N, crop_y > crop_x ? crop_y : crop_x);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && NX == nx_) { replay_inverse<Geom<n_, t_, nx_>>(a, accumulate != 0); return 0; }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

// The same two with the few-maps-per-workgroup geometries that launches of few maps take.
int replay_small_maps_per_block(int N) { return small_maps_per_block(N); }

int replay_fft2d_r2c_small(int N, const float *src, float *spec, int M, int ext_y, int ext_x, int flip)
{
    FwdArgs a{src, reinterpret_cast<cf *>(spec), M, ext_y, ext_x};
    a.flip = flip;
    const int T = small_maps_per_block(N), NX = extent_class(N, ext_y > ext_x ? ext_y : ext_x);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && NX == nx_) { replay_forward<Geom<n_, t_, nx_>>(a); return 0; }
    FFTCONV_FOR_EACH_SMALL_GEOM(X)
#undef X
    return 1;
}

int replay_ifft2d_c2r_crop_small(int N, const float *spec, float *dst, int M, int crop_y, int crop_x, int accumulate, int flip)
{
    InvArgs a{reinterpret_cast<const cf *>(spec), dst, M, crop_y, crop_x, 1.0f / (float)(N * N)};
    a.flip = flip;
    a.parity = -1;
    a.bin_stride = M;
    const int T = small_maps_per_block(N), NX = extent_class(N, crop_y > crop_x ? crop_y : crop_x);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && NX == nx_) { replay_inverse<Geom<n_, t_, nx_>>(a, accumulate != 0); return 0; }
    FFTCONV_FOR_EACH_SMALL_GEOM(X)
#undef X
    return 1;
}

// Row and column of tile t under either numbering (for the tests' expected values).
void replay_tile_row_col(int t, int tiles_x, int tiles, int by_class, int *ty, int *tx)
{
    const Tiling tl{0, 0, 1, tiles_x, tiles, 0, 0, 0, 0, by_class};
    tile_row_col(t, tl, *ty, *tx);
}

// Tiled variants: src / dst are [S][C][H][W] images, M = S * tiles * C transforms of size N
// (the full-extent geometry of N), tile t of an image at (ty * step + org, tx * step + org).
int replay_fft2d_r2c_tiled(int N, const float *src, float *spec, int M, int ext_y, int ext_x, int H, int W, int C,
                           int tiles_x, int tiles, int step_y, int step_x, int org_y, int org_x, int by_class)
{
    FwdArgs a{src, reinterpret_cast<cf *>(spec), M, ext_y, ext_x, {H, W, C, tiles_x, tiles, step_y, step_x, org_y, org_x, by_class}};
    const int T = maps_per_block(N);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && n_ == nx_) { replay_forward<Geom<n_, t_, nx_>, true>(a); return 0; }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

// add / parity: overlap-add of the windows of one parity class of tiles (parity -1: every tile).
int replay_ifft2d_c2r_tiled(int N, const float *spec, float *dst, int M, int crop_y, int crop_x, int c0_y, int c0_x,
                            int H, int W, int C, int tiles_x, int tiles, int step_y, int step_x, int add, int parity,
                            int by_class)
{
    InvArgs a{reinterpret_cast<const cf *>(spec), dst, M, crop_y, crop_x, 1.0f / (float)(N * N), c0_y, c0_x,
              {H, W, C, tiles_x, tiles, step_y, step_x, 0, 0, by_class}};
    a.add = add;
    a.parity = parity;
    a.bin_stride = M;
    if (parity >= 0) {   // one parity class of tiles: the launch covers S * cls_tiles * C transforms
        const int tiles_y = tiles / tiles_x;
        const int cy = (tiles_y - parity / 2 + 1) / 2, cx = (tiles_x - parity % 2 + 1) / 2;
        if (cy < 1 || cx < 1) return 0;
        a.cls_cx = cx;
        a.cls_tiles = cy * cx;
        a.M = (M / (tiles * C)) * a.cls_tiles * C;
    }
    const int T = maps_per_block(N);
#define X(n_, t_, nx_) \
    if constexpr (n_ == nx_) { if (N == n_ && T == t_) { replay_inverse<Geom<n_, t_, nx_>, true>(a, false); return 0; } }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

// Fused fprop of a layer with F = 3 input maps (full-extent geometries only): the bins of output
// map m = s * fo + j are formed from xs [B][Mx] and wsp [B][Mw] instead of being read.  fo must be
// a multiple of the geometry's maps per workgroup.
int replay_ifft2d_c2r_crop_fused3(int N, const float *xs, const float *wsp, float *dst, int M, int fo, int Mx, int Mw,
                                  int crop_y, int crop_x)
{
    if (fo % maps_per_block(N) != 0) return 2;
    InvArgs a{nullptr, dst, M, crop_y, crop_x, 1.0f / (float)(N * N)};
    a.parity = -1;
    a.bin_stride = M;
    a.xs = reinterpret_cast<const cf *>(xs);
    a.wsp = reinterpret_cast<const cf *>(wsp);
    a.fo = fo; a.Mx = Mx; a.Mw = Mw;
    const int T = maps_per_block(N);
#define X(n_, t_, nx_) \
    if constexpr (n_ == nx_) { if (N == n_ && T == t_) { replay_inverse<Geom<n_, t_, nx_>, false, 3>(a, false); return 0; } }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

}  // extern "C"

// Host replay of the FFT kernels' two phases (no GPU, no HIP): every block and
// every lane is run in a loop, phase by phase, on an ordinary array standing in
// for LDS.  Used only by CPU tests to check the kernels' index arithmetic and
// the transform conventions against a naive DFT; it is not part of the product
// path and is not linked into the GPU library.
#include <array>
#include <cstring>
#include <vector>

#include "fft_dispatch.hpp"

using namespace fftconv;

template <class G>
static void replay_forward(const FwdArgs &a)
{
    std::vector<cf> lds(G::LDS_ELEMS);
    std::vector<std::array<cf, G::N>> z(G::THREADS);
    std::vector<char> has(G::THREADS);
    const int blocks = (a.M + G::T - 1) / G::T;
    for (int blk = 0; blk < blocks; ++blk) {
        // poison: an x-phase read of something the y-phase did not write shows up as NaN
        std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
        for (int tid = 0; tid < G::THREADS; ++tid) {
            std::memset(z[tid].data(), 0xFF, sizeof(cf) * G::N);
            has[tid] = fwd_y_compute<G>(tid, blk, a, reinterpret_cast<cf(&)[G::N]>(*z[tid].data()));
        }
        for (int tid = 0; tid < G::THREADS; ++tid)
            if (has[tid]) fwd_y_write<G, 0>(tid, reinterpret_cast<cf(&)[G::N]>(*z[tid].data()), lds.data());
        for (int tid = 0; tid < G::THREADS; ++tid) fwd_x<G>(tid, blk, 0, a, lds.data());
        if constexpr (G::ROUNDS == 2) {
            std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
            for (int tid = 0; tid < G::THREADS; ++tid)
                if (has[tid]) fwd_y_write<G, 1>(tid, reinterpret_cast<cf(&)[G::N]>(*z[tid].data()), lds.data());
            for (int tid = 0; tid < G::THREADS; ++tid) fwd_x<G>(tid, blk, 1, a, lds.data());
        }
    }
}

template <class G>
static void replay_inverse(const InvArgs &a, bool acc)
{
    std::vector<cf> lds(G::LDS_ELEMS);
    std::vector<std::array<cf, G::N>> z(G::THREADS);
    const int blocks = (a.M + G::T - 1) / G::T;
    for (int blk = 0; blk < blocks; ++blk) {
        std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
        for (int tid = 0; tid < G::THREADS; ++tid) std::memset(z[tid].data(), 0xFF, sizeof(cf) * G::N);
        for (int tid = 0; tid < G::THREADS; ++tid) inv_x<G>(tid, blk, 0, a, lds.data());
        for (int tid = 0; tid < G::THREADS; ++tid)
            inv_y_gather<G, 0>(tid, lds.data(), reinterpret_cast<cf(&)[G::N]>(*z[tid].data()));
        if constexpr (G::ROUNDS == 2) {
            std::memset(lds.data(), 0xFF, sizeof(cf) * lds.size());
            for (int tid = 0; tid < G::THREADS; ++tid) inv_x<G>(tid, blk, 1, a, lds.data());
            for (int tid = 0; tid < G::THREADS; ++tid)
                inv_y_gather<G, 1>(tid, lds.data(), reinterpret_cast<cf(&)[G::N]>(*z[tid].data()));
        }
        for (int tid = 0; tid < G::THREADS; ++tid) {
            if (acc) inv_y_finish<G, true>(tid, blk, a, reinterpret_cast<cf(&)[G::N]>(*z[tid].data()));
            else inv_y_finish<G, false>(tid, blk, a, reinterpret_cast<cf(&)[G::N]>(*z[tid].data()));
        }
    }
}

extern "C" {

int replay_fft_size(int n) { return fft_size_for(n); }
int replay_extent_class(int N, int ext) { return extent_class(N, ext); }

// src: [M][ext][ext] floats; spec: [B][M] complex (2 floats each), B = (N/2+1)*N.
int replay_fft2d_r2c(int N, const float *src, float *spec, int M, int ext)
{
    FwdArgs a{src, reinterpret_cast<cf *>(spec), M, ext};
    const int T = maps_per_block(N), NX = extent_class(N, ext);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && NX == nx_) { replay_forward<TileGeom<n_, t_, nx_, rounds_for(n_)>>(a); return 0; }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

int replay_ifft2d_c2r_crop(int N, const float *spec, float *dst, int M, int crop, int accumulate)
{
    InvArgs a{reinterpret_cast<const cf *>(spec), dst, M, crop, 1.0f / (float)(N * N)};
    const int T = maps_per_block(N), NX = extent_class(N, crop);
#define X(n_, t_, nx_) \
    if (N == n_ && T == t_ && NX == nx_) { replay_inverse<TileGeom<n_, t_, nx_, rounds_for(n_)>>(a, accumulate != 0); return 0; }
    FFTCONV_FOR_EACH_GEOM(X)
#undef X
    return 1;
}

}  // extern "C"

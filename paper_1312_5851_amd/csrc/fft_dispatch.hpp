// The set of compiled FFT tile geometries and the rule that picks one.
// Shared by the device dispatcher and by the host replay used in tests, so the
// two can never disagree on which instantiation handles a given layer.
#pragma once
#include "fft_kernels.hpp"

namespace fftconv {

// X(N, T, NX): transform size, maps per workgroup, non-zero / needed extent class.
// T * N / 2 lanes.  T is at least 16 so that a bin is stored as a full 128-byte run.
#define FFTCONV_FOR_EACH_GEOM(X) \
    X(8, 64, 8)   X(8, 64, 4)                 \
    X(12, 32, 12) X(12, 32, 6)                \
    X(14, 32, 14) X(14, 32, 7)                \
    X(16, 32, 16) X(16, 32, 8)  X(16, 32, 4)  \
    X(20, 32, 20) X(20, 32, 10) X(20, 32, 5)  \
    X(24, 16, 24) X(24, 16, 12) X(24, 16, 6)  \
    X(28, 16, 28) X(28, 16, 14) X(28, 16, 7)  \
    X(32, 16, 32) X(32, 16, 16) X(32, 16, 8)  \
    X(40, 16, 40) X(40, 16, 20) X(40, 16, 10) \
    X(48, 16, 48) X(48, 16, 24) X(48, 16, 12) \
    X(56, 16, 56) X(56, 16, 28) X(56, 16, 14) \
    X(64, 16, 64) X(64, 16, 32) X(64, 16, 16)

// The same geometries with few maps per workgroup (one or two waves), for launches of so few maps that the
// usual workgroups would leave most of the chip idle (the 384 maps of a minibatch of RGB images are 24
// workgroups of 16 maps on 256 CUs).  Such a launch takes as long as one workgroup's chain of loads, two 1-D
// transforms and stores, whatever its size, so it pays to spread it over more CUs; the short runs per bin
// (16 to 64 bytes instead of 128) cost nothing at these sizes.  Measured on S=128, f=3, f'=96, n=64, k=11 with
// 8 instead of 16 maps per workgroup at N = 64: fft_x 19.3 -> 15.2 us, ifft_dx 18.7 -> 17.4, while the large
// launches lose (fft_g 88 -> 96 us; S=128, f=f'=256: fft_w 238 -> 351 us).
#define FFTCONV_FOR_EACH_SMALL_GEOM(X) \
    X(8, 16, 8)   X(8, 16, 4)               \
    X(12, 8, 12)  X(12, 8, 6)               \
    X(14, 8, 14)  X(14, 8, 7)               \
    X(16, 8, 16)  X(16, 8, 8)   X(16, 8, 4)  \
    X(20, 8, 20)  X(20, 8, 10)  X(20, 8, 5)  \
    X(24, 8, 24)  X(24, 8, 12)  X(24, 8, 6)  \
    X(28, 8, 28)  X(28, 8, 14)  X(28, 8, 7)  \
    X(32, 4, 32)  X(32, 4, 16)  X(32, 4, 8)  \
    X(40, 4, 40)  X(40, 4, 20)  X(40, 4, 10) \
    X(48, 4, 48)  X(48, 4, 24)  X(48, 4, 12) \
    X(56, 4, 56)  X(56, 4, 28)  X(56, 4, 14) \
    X(64, 2, 64)  X(64, 2, 32)  X(64, 2, 16)

// Transform size for an n x n input: the smallest of 8, 12, 14, 16, 20, 24, 28, 32, 40, 48, 56,
// 64 that holds it.  The paper pads to the next power of two and names the waste for sizes just
// above one as its limitation (Sec. 4), with n = 34 -> 64 as its example; the sizes 3 * 2^m,
// 5 * 2^m and 7 * 2^m bring that case down to 40, fit the map sizes 14, 28 and 56 of
// image-classification networks exactly, and keep the padded area below 1.5 x the map for n >= 10.
inline int fft_size_for(int n)
{
    static const int sizes[] = {8, 12, 14, 16, 20, 24, 28, 32, 40, 48, 56, 64};
    for (int N : sizes)
        if (N >= n) return N;
    return -1;
}

constexpr int maps_per_block(int N) { return N <= 8 ? 64 : (N <= 20 ? 32 : 16); }
constexpr int small_maps_per_block(int N) { return N <= 8 ? 16 : (N <= 28 ? 8 : (N <= 56 ? 4 : 2)); }

// Maps per workgroup for a launch of M maps: the small geometry when the usual one would give at most
// kSmallBatchBlocks workgroups (a quarter of the CUs).
constexpr int kSmallBatchBlocks = 64;
inline int maps_per_block_for(int N, long M, bool allow_small)
{
    const int T = maps_per_block(N);
    return allow_small && (M + T - 1) / T <= kSmallBatchBlocks ? small_maps_per_block(N) : T;
}

// LDS hand-overs between the two phases: two from N = 40 up, where one would not fit the
// 160 KB of LDS or would leave room for a single workgroup per CU.  (At N = 32 two rounds
// let four workgroups share a CU instead of two; inside the full step that measured the same
// as one round, so N = 32 keeps the simpler single round.  The narrow extent classes of
// N >= 40, whose hand-over would fit one round, measured no better with one: forward of 5 x 5
// kernels at N = 64 234 against 238 us, the inverse to 5 x 5 at N = 48 and 56 a quarter and a tenth
// slower, so every class of a size keeps the same two-team schedule.)
constexpr int rounds_for(int N) { return N >= 40 ? 2 : 1; }

template <int N, int T, int NX>
using Geom = TileGeom<N, T, NX, rounds_for(N)>;

// Smallest compiled extent class that covers `ext` columns of an N-point transform.
inline int extent_class(int N, int ext)
{
    if (N >= 16 && ext <= N / 4) return N / 4;
    if (ext <= N / 2) return N / 2;
    return N;
}

}  // namespace fftconv

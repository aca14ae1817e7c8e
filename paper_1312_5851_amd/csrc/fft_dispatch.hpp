// The set of compiled FFT tile geometries and the rule that picks one.
// Shared by the device dispatcher and by the host replay used in tests, so the
// two can never disagree on which instantiation handles a given layer.
#pragma once
#include "fft_kernels.hpp"

namespace fftconv {

// X(N, T, NX): transform size, maps per workgroup, non-zero / needed extent class.
// T * N / 2 lanes: 256, except 512 at N = 64 (16 maps, so that a bin is still stored as one
// full 128-byte run).
#define FFTCONV_FOR_EACH_GEOM(X) \
    X(8, 64, 8)   X(8, 64, 4)                 \
    X(16, 32, 16) X(16, 32, 8)  X(16, 32, 4)  \
    X(32, 16, 32) X(32, 16, 16) X(32, 16, 8)  \
    X(64, 16, 64) X(64, 16, 32) X(64, 16, 16)

// Transform size for an n x n input: n rounded up to a power of two (Sec. 4 of
// the paper: sizes that are not a power of two are padded to the next one).
inline int fft_size_for(int n)
{
    int N = 8;
    while (N < n) N *= 2;
    return N;
}

inline int maps_per_block(int N) { return N >= 64 ? 16 : 512 / N; }

// LDS hand-overs between the two phases: two at N = 64, where one would not fit the 160 KB
// of LDS.  (At N = 32 two rounds let four workgroups share a CU instead of two; inside the
// full step that measured the same as one round, so N = 32 keeps the simpler single round.)
constexpr int rounds_for(int N) { return N >= 64 ? 2 : 1; }

// Smallest compiled extent class that covers `ext` columns of an N-point transform.
inline int extent_class(int N, int ext)
{
    if (N >= 16 && ext <= N / 4) return N / 4;
    if (ext <= N / 2) return N / 2;
    return N;
}

}  // namespace fftconv

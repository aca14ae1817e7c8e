// The set of compiled FFT tile geometries and the rule that picks one.
// Shared by the device dispatcher and by the host replay used in tests, so the
// two can never disagree on which instantiation handles a given layer.
#pragma once
#include "fft_kernels.hpp"

namespace fftconv {

// X(N, T, NX): transform size, maps per workgroup, non-zero / needed extent class.
// T * N / 2 = 256 lanes in every case.
#define FFTCONV_FOR_EACH_GEOM(X) \
    X(8, 64, 8)   X(8, 64, 4)                 \
    X(16, 32, 16) X(16, 32, 8)  X(16, 32, 4)  \
    X(32, 16, 32) X(32, 16, 16) X(32, 16, 8)  \
    X(64, 8, 64)  X(64, 8, 32)  X(64, 8, 16)

// Transform size for an n x n input: n rounded up to a power of two (Sec. 4 of
// the paper: sizes that are not a power of two are padded to the next one).
inline int fft_size_for(int n)
{
    int N = 8;
    while (N < n) N *= 2;
    return N;
}

inline int maps_per_block(int N) { return 512 / N; }

// Smallest compiled extent class that covers `ext` columns of an N-point transform.
inline int extent_class(int N, int ext)
{
    if (N >= 16 && ext <= N / 4) return N / 4;
    if (ext <= N / 2) return N / 2;
    return N;
}

}  // namespace fftconv

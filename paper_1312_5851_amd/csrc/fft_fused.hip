// fprop of a layer with very few input maps (an RGB first layer): the per-bin product of Sec. 2.2
// is three complex multiply-adds per output bin, and its result, written to HBM by one kernel and
// read back by the next, would be the largest array of the whole pass.  These instantiations of
// the inverse-transform kernels compute each bin from the (small, cache-resident) spectra of x and
// w at the moment the transform needs it, so the output spectrum never exists in memory.
//
// Compiled once per number of input maps, -DFFTCONV_FUSED_F=1 .. 4, into objects of their own.
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"

#ifndef FFTCONV_FUSED_F
#error "compile with -DFFTCONV_FUSED_F=<number of input maps, 1 to 4>"
#endif

namespace fftconv {
namespace {

constexpr int F = FFTCONV_FUSED_F;

struct FusedEntry {
    int N, T, NX;
    InvKernel plain, tiled;
};

template <int N, int T, int NX>
constexpr InvKernel tiled_kernel()
{
    if constexpr (NX == N && N >= 16) return ifft2d_c2r_tiled_kernel<Geom<N, T, NX>, F>;
    else return nullptr;
}

#define X(n_, t_, nx_) \
    {n_, t_, nx_, ifft2d_c2r_crop_kernel<Geom<n_, t_, nx_>, false, F>, tiled_kernel<n_, t_, nx_>()},
const FusedEntry kFusedTable[] = {FFTCONV_FOR_EACH_GEOM(X)};
#undef X

}  // namespace

#define FUSED_LOOKUP_NAME_(f) fused_inverse_kernel_f##f
#define FUSED_LOOKUP_NAME(f) FUSED_LOOKUP_NAME_(f)
InvKernel FUSED_LOOKUP_NAME(FFTCONV_FUSED_F)(int N, int T, int NX, bool tiled)
{
    for (const FusedEntry &e : kFusedTable)
        if (e.N == N && e.T == T && e.NX == NX) return tiled ? e.tiled : e.plain;
    return nullptr;
}

}  // namespace fftconv

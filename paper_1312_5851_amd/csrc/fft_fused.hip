// fprop of a layer with very few input maps (an RGB first layer): the per-bin product of Sec. 2.2
// is three complex multiply-adds per output bin, and its result, written to HBM by one kernel and
// read back by the next, would be the largest array of the whole pass.  These instantiations of
// the inverse-transform kernels compute each bin from the (small, cache-resident) spectra of x and
// w at the moment the transform needs it, so the output spectrum never exists in memory.
#include <hip/hip_runtime.h>

#include "fft_fused.hpp"

namespace fftconv {
namespace {

struct FusedEntry {
    int N, T, NX;
    InvKernel plain[kMaxFusedMaps], tiled[kMaxFusedMaps];
};

template <int N, int T, int NX, int F>
constexpr InvKernel tiled_kernel()
{
    if constexpr (NX == N && N >= 16) return ifft2d_c2r_tiled_kernel<TileGeom<N, T, NX, rounds_for(N)>, F>;
    else return nullptr;
}

#define X(n_, t_, nx_)                                                                    \
    {n_, t_, nx_,                                                                         \
     {ifft2d_c2r_crop_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>, false, 1>,            \
      ifft2d_c2r_crop_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>, false, 2>,            \
      ifft2d_c2r_crop_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>, false, 3>,            \
      ifft2d_c2r_crop_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>, false, 4>},           \
     {tiled_kernel<n_, t_, nx_, 1>(), tiled_kernel<n_, t_, nx_, 2>(), tiled_kernel<n_, t_, nx_, 3>(), \
      tiled_kernel<n_, t_, nx_, 4>()}},
const FusedEntry kFusedTable[] = {FFTCONV_FOR_EACH_GEOM(X)};
#undef X

}  // namespace

InvKernel fused_inverse_kernel(int N, int T, int NX, int F, bool tiled)
{
    if (F < 1 || F > kMaxFusedMaps) return nullptr;
    for (const FusedEntry &e : kFusedTable)
        if (e.N == N && e.T == T && e.NX == NX) return tiled ? e.tiled[F - 1] : e.plain[F - 1];
    return nullptr;
}

}  // namespace fftconv

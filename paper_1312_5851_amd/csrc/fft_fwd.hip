// Forward-transform kernels (fft_kernels.hpp), one instantiation per compiled geometry.
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"

namespace fftconv {
namespace {

template <int N, int T, int NX>
constexpr FwdKernel tiled_fwd_kernel()
{
    if constexpr (NX == N && N >= 16 && T == maps_per_block(N)) return fft2d_r2c_kernel<Geom<N, T, NX>, true>;
    else return nullptr;
}

#define X(n_, t_, nx_)                                                                                              \
    {n_, t_, nx_, Geom<n_, t_, nx_>::THREADS, Geom<n_, t_, nx_>::LDS_BYTES, \
     fft2d_r2c_kernel<Geom<n_, t_, nx_>>, tiled_fwd_kernel<n_, t_, nx_>()},
const FwdEntry kFwdTable[] = {FFTCONV_FOR_EACH_GEOM(X)};
#undef X

}  // namespace

const FwdEntry *find_fwd_kernels(int N, int T, int NX)
{
    for (const FwdEntry &e : kFwdTable)
        if (e.N == N && e.T == T && e.NX == NX) return &e;
    return find_fwd_kernels_small(N, T, NX);
}

}  // namespace fftconv

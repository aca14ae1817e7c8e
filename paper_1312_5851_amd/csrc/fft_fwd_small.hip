// Forward-transform kernels of the geometries with few maps per workgroup (fft_dispatch.hpp).
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"

namespace fftconv {
namespace {

#define X(n_, t_, nx_) \
    {n_, t_, nx_, Geom<n_, t_, nx_>::THREADS, Geom<n_, t_, nx_>::LDS_BYTES, fft2d_r2c_kernel<Geom<n_, t_, nx_>>, nullptr},
const FwdEntry kFwdSmallTable[] = {FFTCONV_FOR_EACH_SMALL_GEOM(X)};
#undef X

}  // namespace

const FwdEntry *find_fwd_kernels_small(int N, int T, int NX)
{
    for (const FwdEntry &e : kFwdSmallTable)
        if (e.N == N && e.T == T && e.NX == NX) return &e;
    return nullptr;
}

}  // namespace fftconv

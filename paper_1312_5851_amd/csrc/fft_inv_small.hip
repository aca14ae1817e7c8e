// Inverse-transform kernels of the geometries with few maps per workgroup (fft_dispatch.hpp).
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"

namespace fftconv {
namespace {

#define X(n_, t_, nx_)                                                                           \
    {n_, t_, nx_, Geom<n_, t_, nx_>::THREADS, Geom<n_, t_, nx_>::LDS_BYTES,                      \
     ifft2d_c2r_crop_kernel<Geom<n_, t_, nx_>, false>, ifft2d_c2r_crop_kernel<Geom<n_, t_, nx_>, true>},
const InvEntry kInvSmallTable[] = {FFTCONV_FOR_EACH_SMALL_GEOM(X)};
#undef X

}  // namespace

const InvEntry *find_inv_kernels_small(int N, int T, int NX)
{
    for (const InvEntry &e : kInvSmallTable)
        if (e.N == N && e.T == T && e.NX == NX) return &e;
    return nullptr;
}

}  // namespace fftconv

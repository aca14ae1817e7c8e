// Inverse-transform kernels with crop (fft_kernels.hpp), overwriting and accumulating, one pair
// per compiled geometry.
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"

namespace fftconv {
namespace {

#define X(n_, t_, nx_)                                                                                              \
    {n_, t_, nx_, Geom<n_, t_, nx_>::THREADS, Geom<n_, t_, nx_>::LDS_BYTES, \
     ifft2d_c2r_crop_kernel<Geom<n_, t_, nx_>, false>,                                          \
     ifft2d_c2r_crop_kernel<Geom<n_, t_, nx_>, true>},
const InvEntry kInvTable[] = {FFTCONV_FOR_EACH_GEOM(X)};
#undef X

}  // namespace

const InvEntry *find_inv_kernels(int N, int T, int NX)
{
    for (const InvEntry &e : kInvTable)
        if (e.N == N && e.T == T && e.NX == NX) return &e;
    return find_inv_kernels_small(N, T, NX);
}

}  // namespace fftconv

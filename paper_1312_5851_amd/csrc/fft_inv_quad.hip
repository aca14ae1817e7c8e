// Inverse transforms for small windows with each 1-D transform split over four lanes
// (fft_quad_kernels.hpp): the extent class N / 4 of the sizes N >= 40.
#include <hip/hip_runtime.h>

#include "fft_quad_kernels.hpp"
#include "kernel_tables.hpp"

namespace fftconv {
namespace {

#define Q(n_)                                                                                       \
    {n_, maps_per_block(n_), QuadGeom<n_, maps_per_block(n_)>::THREADS, QuadGeom<n_, maps_per_block(n_)>::LDS_BYTES, \
     ifft2d_c2r_crop_quad_kernel<QuadGeom<n_, maps_per_block(n_)>, false>,                           \
     ifft2d_c2r_crop_quad_kernel<QuadGeom<n_, maps_per_block(n_)>, true>},
const InvQuadEntry kInvQuadTable[] = {Q(40) Q(48) Q(56) Q(64)};
#undef Q

}  // namespace

const InvQuadEntry *find_inv_quad_kernels(int N)
{
    for (const InvQuadEntry &e : kInvQuadTable)
        if (e.N == N) return &e;
    return nullptr;
}

}  // namespace fftconv

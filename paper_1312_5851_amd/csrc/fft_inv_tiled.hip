// Inverse-transform kernels that scatter their windows into larger images (maps above 64 x 64,
// fft_kernels.hpp): overlap-save (each window written once) and overlap-add.
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"

namespace fftconv {
namespace {

template <int N, int T, int NX, bool ADD>
constexpr InvKernel tiled_inv_kernel()
{
    if constexpr (NX == N && N >= 16) return ifft2d_c2r_tiled_kernel<Geom<N, T, NX>, 0, ADD>;
    else return nullptr;
}

#define X(n_, t_, nx_) {n_, t_, nx_, tiled_inv_kernel<n_, t_, nx_, false>(), tiled_inv_kernel<n_, t_, nx_, true>()},
const InvTiledEntry kInvTiledTable[] = {FFTCONV_FOR_EACH_GEOM(X)};
#undef X

}  // namespace

const InvTiledEntry *find_inv_tiled_kernels(int N, int T, int NX)
{
    for (const InvTiledEntry &e : kInvTiledTable)
        if (e.N == N && e.T == T && e.NX == NX) return e.tiled ? &e : nullptr;
    return nullptr;
}

}  // namespace fftconv

// Inverse-transform kernels that form their input bins on the fly (fprop of layers with at most
// four input maps).  The instantiations live in a translation unit of their own so that the two
// halves of the library compile side by side.
#pragma once
#include "fft_dispatch.hpp"

namespace fftconv {

typedef void (*InvKernel)(InvArgs);

constexpr int kMaxFusedMaps = 4;

// The kernel for geometry (N, T, NX) and F input maps, untiled or tiled; nullptr if there is none
// (F outside [1, kMaxFusedMaps], unknown geometry, or a tiled kernel of a geometry tiles do not use).
InvKernel fused_inverse_kernel(int N, int T, int NX, int F, bool tiled);

}  // namespace fftconv

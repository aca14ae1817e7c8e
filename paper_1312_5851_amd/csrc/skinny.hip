// Streaming contraction kernels for layers with at most four input maps (skinny_kernels.hpp).
#include <hip/hip_runtime.h>

#include "kernel_tables.hpp"
#include "skinny_kernels.hpp"

namespace fftconv {

SkinnyKernel skinny_accgrad(int F)
{
    static const SkinnyKernel k[4] = {skinny_accgrad_kernel<1>, skinny_accgrad_kernel<2>, skinny_accgrad_kernel<3>,
                                      skinny_accgrad_kernel<4>};
    return F >= 1 && F <= 4 ? k[F - 1] : nullptr;
}

SkinnyKernel skinny_bprop(int F)
{
    static const SkinnyKernel k[4] = {skinny_bprop_kernel<1>, skinny_bprop_kernel<2>, skinny_bprop_kernel<3>,
                                      skinny_bprop_kernel<4>};
    return F >= 1 && F <= 4 ? k[F - 1] : nullptr;
}

SharedPassKernel skinny_bprop_accgrad(int F)
{
    static const SharedPassKernel k[4] = {skinny_bprop_accgrad_kernel<1>, skinny_bprop_accgrad_kernel<2>,
                                          skinny_bprop_accgrad_kernel<3>, skinny_bprop_accgrad_kernel<4>};
    return F >= 1 && F <= 4 ? k[F - 1] : nullptr;
}

SumGroupsKernel sum_row_groups() { return sum_row_groups_kernel; }

}  // namespace fftconv

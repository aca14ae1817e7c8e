// Matrix-core contraction kernels (contract_kernels.hpp): every workgroup tile shape for each of
// the three passes.
#include <hip/hip_runtime.h>

#include "contract_kernels.hpp"
#include "kernel_tables.hpp"

namespace fftconv {
namespace {

// Layout / conjugation per pass:
//   fprop   A = Xh [S][f]  K contiguous,  B = Wh [fo][f] K contiguous, conj B
//   bprop   A = Gh [S][fo] K contiguous,  B = Wh [fo][f] K outer
//   accGrad A = Gh [S][fo] K outer, conj A,  B = Xh [S][f] K outer
#define GEMM_ENTRY(it, jt, wm, wn, occ) GEMM_ENTRY_SETS(it, jt, wm, wn, occ, 1)
#define GEMM_ENTRY_SETS(it, jt, wm, wn, occ, sets)                                               \
    {GemmTile<it, jt, wm, wn, sets>::MT, GemmTile<it, jt, wm, wn, sets>::NT, wm * wn, occ,       \
     GemmTile<it, jt, wm, wn, sets>::THREADS, GemmTile<it, jt, wm, wn, sets>::LDS_BYTES,         \
     {bin_cgemm_kernel<GemmTile<it, jt, wm, wn, sets>, true, true, false, true>,                 \
      bin_cgemm_kernel<GemmTile<it, jt, wm, wn, sets>, true, false, false, false>,               \
      bin_cgemm_kernel<GemmTile<it, jt, wm, wn, sets>, false, false, true, false>},              \
     bin_cgemm_bprop_accgrad_kernel<GemmTile<it, jt, wm, wn, sets>>}
// (32x32 tiles per wave along M and N, waves along M and N, resident waves per SIMD)
// One 32x32 tile per wave throughout.  Measured inside the full step on MI355X (operands
// coming from HBM, not from a cache warmed by the previous launch), these shapes win over
// larger wave tiles (64x32, 64x64 per wave), over 8-, 12- and 16-wave workgroups and over 1-
// and 2-wave workgroups of the same wave tile at the K of these layers: four resident
// workgroups per CU hide the per-tile prologue, epilogue and barrier waits best.
const GemmEntry kGemmTable[] = {
    GEMM_ENTRY(1, 1, 2, 2, 4),   // 0:  64 x 64
    GEMM_ENTRY(1, 1, 4, 1, 4),   // 1: 128 x 32
    GEMM_ENTRY(1, 1, 2, 3, 4),   // 2:  64 x 96
    GEMM_ENTRY(1, 1, 1, 1, 4),   // 3:  32 x 32
    // the same shapes with two register sets of operand chunks in flight, for HBM-bound products
    GEMM_ENTRY_SETS(1, 1, 2, 2, 3, 2),   // 4:  64 x 64
    GEMM_ENTRY_SETS(1, 1, 4, 1, 3, 2),   // 5: 128 x 32
    GEMM_ENTRY_SETS(1, 1, 2, 3, 3, 2),   // 6:  64 x 96
    GEMM_ENTRY_SETS(1, 1, 1, 1, 3, 2),   // 7:  32 x 32
};
#undef GEMM_ENTRY
#undef GEMM_ENTRY_SETS

}  // namespace

const GemmEntry *gemm_kernel_table() { return kGemmTable; }
int gemm_kernel_count() { return (int)(sizeof(kGemmTable) / sizeof(kGemmTable[0])); }
int gemm_shape_count() { return 4; }

}  // namespace fftconv

// The compiled kernels, grouped in tables that the host code searches.  Each table lives in a
// translation unit of its own (fft_fwd.hip, fft_inv.hip, fft_inv_quad.hip, fft_inv_tiled.hip, fft_fused.hip once
// per number of input maps, contract.hip, skinny.hip) so that the library's parts compile side
// by side; the host code in fftconv.hip instantiates no kernel itself.
#pragma once
#include "contract_args.hpp"
#include "fft_dispatch.hpp"

namespace fftconv {

typedef void (*FwdKernel)(FwdArgs);
typedef void (*InvKernel)(InvArgs);
typedef void (*GemmKernel)(GemmArgs);
typedef void (*GemmPairKernel)(GemmPairArgs);
typedef void (*SkinnyKernel)(SkinnyArgs);
typedef void (*SharedPassKernel)(SharedPassArgs);
typedef void (*SumGroupsKernel)(const cf *, cf *, size_t, int);

// One transform geometry (N, T, NX): launch with `threads` lanes and `lds_bytes` of dynamic LDS.
// The tiled kernels exist for the full-extent geometries (NX == N) of N >= 16 only (smaller
// transforms would be mostly overlap); nullptr otherwise.
struct FwdEntry {
    int N, T, NX, threads, lds_bytes;
    FwdKernel plain, tiled;
};
struct InvEntry {
    int N, T, NX, threads, lds_bytes;
    InvKernel plain, acc;   // overwrite / add to the destination
};
struct InvTiledEntry {
    int N, T, NX;
    InvKernel tiled, tiled_add;   // each window written once / overlapping windows added
};

// Inverse transforms of the extent class N / 4 with every 1-D transform split over four lanes
// (fft_quad_kernels.hpp); N >= 40 only.
struct InvQuadEntry {
    int N, T, threads, lds_bytes;
    InvKernel plain, acc;
};

const FwdEntry *find_fwd_kernels(int N, int T, int NX);        // either list of geometries
const FwdEntry *find_fwd_kernels_small(int N, int T, int NX);  // few maps per workgroup (fft_fwd_small.hip)
const InvEntry *find_inv_kernels_small(int N, int T, int NX);  // (fft_inv_small.hip)
const InvQuadEntry *find_inv_quad_kernels(int N);   // nullptr if N has none
const InvEntry *find_inv_kernels(int N, int T, int NX);
const InvTiledEntry *find_inv_tiled_kernels(int N, int T, int NX);

// Inverse-transform kernels that form their input bins on the fly (fprop of layers with at most
// kMaxFusedMaps input maps): the kernel for geometry (N, T, NX) and F input maps, untiled or
// tiled; nullptr if there is none.
constexpr int kMaxFusedMaps = 4;
InvKernel fused_inverse_kernel(int N, int T, int NX, int F, bool tiled);

// One workgroup tile shape of the matrix-core contraction.
struct GemmEntry {
    int MT, NT, waves, occ, threads, lds_bytes;
    GemmKernel pass[3];   // indexed by FFTCONV_FPROP / BPROP / ACCGRAD
    GemmPairKernel bprop_accgrad;   // both of their products in one launch
};
// Entries i and i + gemm_shape_count() have the same shape (the second half keeps two register
// sets of operand chunks in flight).
const GemmEntry *gemm_kernel_table();
int gemm_kernel_count();
int gemm_shape_count();

// Streaming kernels for layers with at most four input maps, F in [1, 4].
SkinnyKernel skinny_accgrad(int F);
SkinnyKernel skinny_bprop(int F);
SharedPassKernel skinny_bprop_accgrad(int F);
SumGroupsKernel sum_row_groups();

}  // namespace fftconv

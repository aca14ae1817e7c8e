// Argument structures and launch constants of the contraction kernels, shared by the host code
// (which fills them) and the translation units that hold the kernels.
#pragma once
#include "fft_core.hpp"

namespace fftconv {

struct GemmArgs {
    const cf *A;     // left operand spectrum
    const cf *B;     // right operand spectrum
    cf *C;           // result spectrum, [bins][Md][Nd]
    int Md, Nd, Kd;  // per-bin product sizes: C (Md x Nd) = op(A) (Md x Kd) * op(B) (Kd x Nd)
    int bins;
    int tiles_m, tiles_n;
    int xcd_remap;   // 1: renumber workgroups so that each XCD gets contiguous work
    int full_tiles_ok;   // 1: the operand and result matrices of a bin are below 2 GB, so 32-bit byte offsets suffice
};

// bprop's and accGrad's products in one launch (bin_cgemm_bprop_accgrad_kernel): both with the same tile shape.
struct GemmPairArgs {
    GemmArgs bprop, accgrad;
};

struct SkinnyArgs {
    const cf *X;   // accGrad: Xh [bins][M][F];  bprop: Wh [bins][N][F]
    const cf *G;   // Gh  [bins][M][N]
    cf *C;         // accGrad: dWh [bins][N][F];  bprop: dXh [bins][M][F]
    int M, N;      // rows m (samples x tiles), output maps j
    int bins;
    int jblocks;   // accGrad: ceil(N / 64);  bprop: row blocks ceil(M / 64)
};

constexpr int kSkinnyThreads = 256;
constexpr int kSkinnyWaves = kSkinnyThreads / 64;   // K slices a workgroup works on at a time

struct SharedPassArgs {
    const cf *G;   // Gh  [bins][M][N]
    const cf *X;   // Xh  [bins][M][F]
    const cf *W;   // Wh  [bins][N][F]
    cf *DX;        // dXh [bins][M][F]
    cf *DW;        // dWh [bins][N][F]
    cf *DWpart;    // row_groups > 1: partial sums of dWh, [row_groups][bins][N][F]
    int M, N, bins;
    int row_groups;   // ceil(M / kSharedPassMaxRows) workgroups per bin, each on its own rows
};

constexpr int kSharedPassMaxRows = 256;   // rows per workgroup: more, and the partial sums of dXh would crowd the LDS

}  // namespace fftconv

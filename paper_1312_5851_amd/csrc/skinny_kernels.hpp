// Per-bin contraction of accGrad for layers with very few input maps (f <= 4, e.g. RGB
// first layers).
//
// With N = f as small as 3 the complex product of Sec. 2.2 has less than 3 flops per byte: the
// pass is bound by streaming Gh through HBM, and a 32 x 32 matrix-core tile would spend nine
// tenths of its work on padding (measured: 76 us against 46 us here for S=128, f=3, f'=96, N=64).
// This kernel does the few multiply-adds on the vector ALU and is laid out only for coalesced
// streaming: lanes run along the output-map index j, which is contiguous in Gh.
//
//   accGrad dWh[b][j][i] = sum_m conj(Gh[b][m][j]) * Xh[b][m][i]
// m runs over samples (times tiles for a tiled layer).  (fprop and bprop with f <= 4 keep the
// matrix-core kernel: a streaming kernel of the same kind measured no faster for fprop, and the
// large operand of bprop is contiguous along the summed index instead.)
#pragma once
#include <hip/hip_runtime.h>

#include "fft_core.hpp"

namespace fftconv {

struct SkinnyArgs {
    const cf *X;   // Xh  [bins][M][F]
    const cf *G;   // Gh  [bins][M][N]
    cf *C;         // dWh [bins][N][F]
    int M, N;      // rows m (samples x tiles), output maps j
    int bins;
    int jblocks;   // ceil(N / 64)
};

constexpr int kSkinnyThreads = 256;
constexpr int kSkinnyWaves = kSkinnyThreads / 64;   // K slices a workgroup works on at a time

FC_HD cf cmul_conj_b(cf a, cf b) { return mk(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y); }   // a * conj(b)

// A wave works on one row m at a time with its 64 lanes along j, so the row's F values of Xh are
// the same for every lane: they are read through a wave-uniform address (scalar loads) and cost
// no vector-memory instruction; the only vector-memory traffic is the streamed spectrum itself.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)threadIdx.x / 64); }

// grid = bins * jblocks workgroups of kSkinnyThreads threads; the K slices of a workgroup's
// waves are summed through LDS at the end
template <int F>
__global__ __launch_bounds__(kSkinnyThreads) void skinny_accgrad_kernel(SkinnyArgs a)
{
    __shared__ cf part[kSkinnyWaves][64][F];
    const int jl = (int)threadIdx.x % 64, ks = wave_index();
    const int jb = (int)blockIdx.x % a.jblocks, bin = (int)blockIdx.x / a.jblocks;
    const int j = jb * 64 + jl;
    const bool vj = j < a.N;
    const cf *Gb = a.G + (size_t)bin * a.M * a.N + (vj ? j : a.N - 1);
    const cf *Xb = a.X + (size_t)bin * a.M * F;
    cf acc[F];
#pragma unroll
    for (int i = 0; i < F; ++i) acc[i] = mk(0.0f, 0.0f);
    constexpr int U = 8;   // rows in flight per wave
    for (int m0 = ks; m0 < a.M; m0 += U * kSkinnyWaves) {
        cf g[U], x[U][F];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int m = m0 + u * kSkinnyWaves;
            const int mc = m < a.M ? m : a.M - 1;
            g[u] = Gb[(size_t)mc * a.N];
#pragma unroll
            for (int i = 0; i < F; ++i) x[u][i] = Xb[(size_t)mc * F + i];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int m = m0 + u * kSkinnyWaves;
            if (m < a.M) {
#pragma unroll
                for (int i = 0; i < F; ++i) acc[i] = acc[i] + cmul_conj_b(x[u][i], g[u]);   // conj(g) * x
            }
        }
    }
#pragma unroll
    for (int i = 0; i < F; ++i) part[ks][jl][i] = acc[i];
    __syncthreads();
    if (ks == 0 && vj) {
        cf *out = a.C + ((size_t)bin * a.N + j) * F;
#pragma unroll
        for (int i = 0; i < F; ++i) {
            cf s = part[0][jl][i];
#pragma unroll
            for (int q = 1; q < kSkinnyWaves; ++q) s = s + part[q][jl][i];
            out[i] = s;
        }
    }
}

}  // namespace fftconv

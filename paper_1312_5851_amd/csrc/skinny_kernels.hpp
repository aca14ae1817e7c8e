// Per-bin contraction of accGrad and bprop for layers with very few input maps (f <= 4, e.g.
// RGB first layers).
//
// With N = f as small as 3 the complex products of Sec. 2.2 have less than 3 flops per byte: the
// pass is bound by streaming Gh through HBM, and a 32 x 32 matrix-core tile would spend nine
// tenths of its work on padding (measured: accGrad 76 us against 46 us here for S=128, f=3,
// f'=96, N=64).  These kernels do the few multiply-adds on the vector ALU and are laid out only
// for coalesced streaming of Gh, whose rows are contiguous along the output-map index j.
//
//   accGrad dWh[b][j][i] = sum_m conj(Gh[b][m][j]) * Xh[b][m][i]     lanes along j, loop over m
//   bprop   dXh[b][m][i] = sum_j      Gh[b][m][j]  * Wh[b][j][i]     64 x 64 tiles of Gh through LDS,
//                                                                    then lanes along m, loop over j
// m runs over samples (times tiles for a tiled layer).  (fprop with f <= 4 keeps the matrix-core
// kernel: a streaming kernel of the same kind measured no faster.)
#pragma once
#include <hip/hip_runtime.h>

#include "fft_core.hpp"

namespace fftconv {

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

// bprop: grid = bins * ceil(M / 64) workgroups of kSkinnyThreads threads.  A workgroup owns 64
// rows m.  Gh comes in as 64 x 64 tiles with lanes along j (coalesced) and is handed over through
// LDS; then lane = row, each of the four waves sums a quarter of the tile's j range with the
// matching Wh values read as LDS broadcasts; the quarters are added at the end.
template <int F>
__global__ __launch_bounds__(kSkinnyThreads) void skinny_bprop_kernel(SkinnyArgs a)
{
    constexpr int TS = 65;                       // tile row stride (odd: lanes along rows hit distinct banks)
    constexpr int U = 64 / kSkinnyWaves;         // tile rows per wave and load pass
    __shared__ cf tile[64 * TS];
    __shared__ cf wt[64 * F];
    const int tid = (int)threadIdx.x, lane = tid % 64, wv = wave_index();
    const int mb = (int)blockIdx.x % a.jblocks, bin = (int)blockIdx.x / a.jblocks;
    const int m0 = mb * 64;
    const cf *Gb = a.G + (size_t)bin * a.M * a.N;
    const cf *Wb = a.X + (size_t)bin * a.N * F;
    const int nchunks = (a.N + 63) / 64;

    cf regs[U], wreg = mk(0.0f, 0.0f);
    bool ok[U], wok = false;
    auto prefetch = [&](int c) {
        const int j = c * 64 + lane;
        const int jc = j < a.N ? j : a.N - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = m0 + wv + kSkinnyWaves * u;
            ok[u] = row < a.M && j < a.N;
            regs[u] = Gb[(size_t)(row < a.M ? row : a.M - 1) * a.N + jc];   // clamped address, masked at the store
        }
        if (tid < 64 * F) {
            const int jw = c * 64 + tid / F;
            wok = jw < a.N;
            wreg = Wb[(size_t)(wok ? jw : a.N - 1) * F + tid % F];
        }
    };
    cf acc[F];
#pragma unroll
    for (int i = 0; i < F; ++i) acc[i] = mk(0.0f, 0.0f);
    prefetch(0);
    for (int c = 0; c < nchunks; ++c) {
#pragma unroll
        for (int u = 0; u < U; ++u) tile[(wv + kSkinnyWaves * u) * TS + lane] = ok[u] ? regs[u] : mk(0.0f, 0.0f);
        if (tid < 64 * F) wt[tid] = wok ? wreg : mk(0.0f, 0.0f);
        __syncthreads();
        if (c + 1 < nchunks) prefetch(c + 1);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int j = wv * 16 + jj;
            const cf g = tile[lane * TS + j];
#pragma unroll
            for (int i = 0; i < F; ++i) {
                const cf w = wt[j * F + i];
                acc[i] = mk(acc[i].x + (g.x * w.x - g.y * w.y), acc[i].y + (g.x * w.y + g.y * w.x));
            }
        }
        __syncthreads();
    }
    // add the four quarters (the tile is free now)
    cf *part = tile;
#pragma unroll
    for (int i = 0; i < F; ++i) part[(wv * 64 + lane) * F + i] = acc[i];
    __syncthreads();
    if (wv == 0 && m0 + lane < a.M) {
        cf *out = a.C + ((size_t)bin * a.M + m0 + lane) * F;
#pragma unroll
        for (int i = 0; i < F; ++i) {
            cf sum = part[lane * F + i];
#pragma unroll
            for (int q = 1; q < kSkinnyWaves; ++q) sum = sum + part[(q * 64 + lane) * F + i];
            out[i] = sum;
        }
    }
}

}  // namespace fftconv

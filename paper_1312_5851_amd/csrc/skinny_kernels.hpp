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

#include "contract_args.hpp"
#include "fft_core.hpp"

namespace fftconv {

// acc + a * b and acc + conj(a) * b as four fused multiply-adds each (a product formed first and
// added afterwards would take six instructions, and these kernels have little else to issue)
__device__ __forceinline__ cf cmac(cf acc, cf a, cf b)
{
    acc.x = __builtin_fmaf(a.x, b.x, acc.x);
    acc.y = __builtin_fmaf(a.x, b.y, acc.y);
    acc.x = __builtin_fmaf(-a.y, b.y, acc.x);
    acc.y = __builtin_fmaf(a.y, b.x, acc.y);
    return acc;
}
__device__ __forceinline__ cf cmac_conj(cf acc, cf a, cf b)
{
    acc.x = __builtin_fmaf(a.x, b.x, acc.x);
    acc.y = __builtin_fmaf(a.x, b.y, acc.y);
    acc.x = __builtin_fmaf(a.y, b.y, acc.x);
    acc.y = __builtin_fmaf(-a.y, b.x, acc.y);
    return acc;
}

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
                for (int i = 0; i < F; ++i) acc[i] = cmac_conj(acc[i], g[u], x[u][i]);   // conj(g) * x
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
                acc[i] = cmac(acc[i], g, w);
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

// bprop and accGrad in one pass over Gh.  Both products read the whole of Gh, the largest array of
// a layer with few input maps, and nothing else of any size, so computing them together halves
// the HBM traffic of the pair:
//     dXh[b][m][i] = sum_j      Gh[b][m][j]  * Wh[b][j][i]
//     dWh[b][j][i] = sum_m conj(Gh[b][m][j]) * Xh[b][m][i]
// One workgroup per bin (per 256 rows of a bin, if it has more: the partial dWh of the row groups
// are then added by sum_row_groups_kernel) walks Gh[b] in 64 x 64 tiles, column block by column block.  A tile comes
// in with lanes along j and is handed over through LDS; then, for dXh, lane = row and the four
// waves each sum a quarter of the tile's columns; for dWh, lane = column and the four waves each
// sum a quarter of the tile's rows.  dWh of a column block is complete when its last tile is done;
// the partial sums of dXh live in LDS, one slot per (quarter, row), until the end.
template <int F>
constexpr int shared_pass_lds_elems(int M)
{
    return 64 * 65 + 2 * 64 * F + kSkinnyWaves * ((M + 63) / 64) * 64 * F;
}

// grid = bins * row_groups workgroups of kSkinnyThreads threads, shared_pass_lds_elems<F>(M) * 8 bytes of dynamic LDS
template <int F>
__global__ __launch_bounds__(kSkinnyThreads) void skinny_bprop_accgrad_kernel(SharedPassArgs a)
{
    constexpr int TS = 65, U = 64 / kSkinnyWaves;
    extern __shared__ __align__(16) unsigned char shared_raw[];
    cf *tile = reinterpret_cast<cf *>(shared_raw);      // [64][TS]
    cf *wt = tile + 64 * TS;                            // Wh of the column block  [64][F]
    cf *xt = wt + 64 * F;                               // Xh of the row block     [64][F]
    cf *dxacc = xt + 64 * F;                            // [waves][rows padded to 64][F]
    cf *red = tile;                                     // [waves][64][F], used between two column blocks only
    static_assert(kSkinnyWaves * 64 * F <= 64 * TS, "the reduction buffer takes the tile's place");
    const int tid = (int)threadIdx.x, lane = tid % 64, q = wave_index();
    const int bin = (int)blockIdx.x / a.row_groups, grp = (int)blockIdx.x % a.row_groups;
    // this workgroup's rows [m0, m0 + Mr) of the bin
    const int m0 = grp * kSharedPassMaxRows, Mr = a.M - m0 < kSharedPassMaxRows ? a.M - m0 : kSharedPassMaxRows;
    const int nmb = (Mr + 63) / 64, njc = (a.N + 63) / 64, Mp = nmb * 64;
    const cf *Gb = a.G + ((size_t)bin * a.M + m0) * a.N;
    const cf *Xb = a.X + ((size_t)bin * a.M + m0) * F;
    const cf *Wb = a.W + (size_t)bin * a.N * F;

    // lane (row r, quarter q) owns dxacc[q][mb * 64 + r][*] until the final sum
    for (int mb = 0; mb < nmb; ++mb)
#pragma unroll
        for (int i = 0; i < F; ++i) dxacc[((size_t)q * Mp + mb * 64 + lane) * F + i] = mk(0.0f, 0.0f);

    cf regs[U], xreg = mk(0.0f, 0.0f), wreg = mk(0.0f, 0.0f);
    bool ok[U], xok = false, wok = false;
    auto prefetch = [&](int jc, int mb) {
        const int j = jc * 64 + lane;
        const int jcl = j < a.N ? j : a.N - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = mb * 64 + q + kSkinnyWaves * u;
            ok[u] = row < Mr && j < a.N;
            regs[u] = Gb[(size_t)(row < Mr ? row : Mr - 1) * a.N + jcl];   // clamped address, masked at the hand-over
        }
        if (tid < 64 * F) {
            const int m = mb * 64 + tid / F, jw = jc * 64 + tid / F;
            xok = m < Mr;
            wok = jw < a.N;
            xreg = Xb[(size_t)(xok ? m : Mr - 1) * F + tid % F];
            wreg = Wb[(size_t)(wok ? jw : a.N - 1) * F + tid % F];
        }
    };
    prefetch(0, 0);
    for (int jc = 0; jc < njc; ++jc) {
        cf dw[F];
#pragma unroll
        for (int i = 0; i < F; ++i) dw[i] = mk(0.0f, 0.0f);
        for (int mb = 0; mb < nmb; ++mb) {
#pragma unroll
            for (int u = 0; u < U; ++u) tile[(q + kSkinnyWaves * u) * TS + lane] = ok[u] ? regs[u] : mk(0.0f, 0.0f);
            if (tid < 64 * F) {
                xt[tid] = xok ? xreg : mk(0.0f, 0.0f);
                wt[tid] = wok ? wreg : mk(0.0f, 0.0f);
            }
            __syncthreads();
            if (mb + 1 < nmb) prefetch(jc, mb + 1);
            else if (jc + 1 < njc) prefetch(jc + 1, 0);
            // dXh: row = lane, columns q * 16 .. q * 16 + 15 of the tile
            cf pdx[F];
#pragma unroll
            for (int i = 0; i < F; ++i) pdx[i] = mk(0.0f, 0.0f);
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const int j = q * 16 + jj;
                const cf g = tile[lane * TS + j];
#pragma unroll
                for (int i = 0; i < F; ++i) {
                    const cf w = wt[j * F + i];
                    pdx[i] = cmac(pdx[i], g, w);
                }
            }
            cf *slot = dxacc + ((size_t)q * Mp + mb * 64 + lane) * F;
#pragma unroll
            for (int i = 0; i < F; ++i) slot[i] = slot[i] + pdx[i];
            // dWh: column = lane, rows q * 16 .. q * 16 + 15 of the tile
#pragma unroll
            for (int mm = 0; mm < 16; ++mm) {
                const int r = q * 16 + mm;
                const cf g = tile[r * TS + lane];
#pragma unroll
                for (int i = 0; i < F; ++i) {
                    const cf x = xt[r * F + i];
                    dw[i] = cmac_conj(dw[i], g, x);
                }
            }
            __syncthreads();
        }
        // dWh of this column block: add the four quarters
#pragma unroll
        for (int i = 0; i < F; ++i) red[(q * 64 + lane) * F + i] = dw[i];
        __syncthreads();
        if (q == 0 && jc * 64 + lane < a.N) {
            // with several row groups per bin, partial sums [group][bin][j][i] that a second kernel adds up
            cf *out = (a.row_groups > 1 ? a.DWpart + (size_t)grp * a.bins * a.N * F : a.DW) + ((size_t)bin * a.N + jc * 64 + lane) * F;
#pragma unroll
            for (int i = 0; i < F; ++i) {
                cf sum = red[lane * F + i];
#pragma unroll
                for (int w = 1; w < kSkinnyWaves; ++w) sum = sum + red[(w * 64 + lane) * F + i];
                out[i] = sum;
            }
        }
        __syncthreads();
    }
    // dXh: add the four quarters; wave q takes the row blocks q, q + 4, ...
    for (int mb = q; mb < nmb; mb += kSkinnyWaves) {
        const int m = mb * 64 + lane;
        if (m < Mr) {
            cf *out = a.DX + ((size_t)bin * a.M + m0 + m) * F;
#pragma unroll
            for (int i = 0; i < F; ++i) {
                cf sum = dxacc[(size_t)m * F + i];
#pragma unroll
                for (int w = 1; w < kSkinnyWaves; ++w) sum = sum + dxacc[((size_t)w * Mp + m) * F + i];
                out[i] = sum;
            }
        }
    }
}

// dWh = sum over row groups of the partial sums the kernel above leaves, in a fixed order.
static __global__ __launch_bounds__(256) void sum_row_groups_kernel(const cf *part, cf *out, size_t count, int groups)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (size_t)gridDim.x * blockDim.x) {
        cf sum = part[e];
        for (int g = 1; g < groups; ++g) sum = sum + part[(size_t)g * count + e];
        out[e] = sum;
    }
}

}  // namespace fftconv

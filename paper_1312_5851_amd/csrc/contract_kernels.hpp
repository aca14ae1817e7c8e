// Per-frequency-bin complex contraction on the fp32 matrix cores (device only).
//
// For every stored bin b the three passes reduce to one dense complex matrix
// product (paper Sec. 2.2 and Fig. 1: all feature maps are multiplied with all
// kernels as a matrix multiplication in the frequency domain):
//
//   fprop    Yh[b][s][j] = sum_i Xh[b][s][i] * conj(Wh[b][j][i])     (Eq. 1)
//   bprop   dXh[b][s][i] = sum_j Gh[b][s][j] *      Wh[b][j][i]      (Eq. 2)
//   accGrad dWh[b][j][i] = sum_s conj(Gh[b][s][j]) * Xh[b][s][i]     (Eq. 3)
//
// (cross-correlation <-> conjugate of the kernel-side spectrum).  All spectra are
// bin-major, complex interleaved, row-major inside a bin.
//
// A complex product is four real ones, issued as v_mfma_f32_32x32x2_f32:
//   Cre += Are*Bre;  Cre += (-Aim)*Bim;  Cim += Are*Bim;  Cim += Aim*Bre
// i.e. 8*M*N*K real flops per bin.  Conjugation is applied once, while an operand
// tile is written to LDS.
//
// A workgroup of WM x WN waves owns an MT x NT tile of one bin's product and walks
// K in chunks of KT.  Operand tiles are staged through LDS as Ps[k][r] (non-K index
// fastest, complex interleaved), so a 32x2 MFMA fragment is one ds_read_b64 per
// lane: lane l reads Ps[k0 + l/32][r0 + l%32].  The next chunk's global loads are
// issued before the current chunk's MFMAs and land in registers meanwhile.
#pragma once
#include <hip/hip_runtime.h>

#include "fft_core.hpp"

namespace fftconv {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const cf *A;     // left operand spectrum
    const cf *B;     // right operand spectrum
    cf *C;           // result spectrum, [bins][Md][Nd]
    int Md, Nd, Kd;  // per-bin product sizes: C (Md x Nd) = op(A) (Md x Kd) * op(B) (Kd x Nd)
    int bins;
    int tiles_m, tiles_n;
    int xcd_remap;   // 1: renumber workgroups so that each XCD gets contiguous work
};

constexpr int kXcds = 8;   // accelerator complex dies on MI355X, workgroups are dealt to them round-robin
constexpr int kKT = 16;   // complex K elements per chunk (one 128-byte line of a K-contiguous row)

// Loads one operand tile chunk (ROWS non-K indices x KT K indices) from global memory
// into registers and later writes it to LDS as Ps[kk * SP + r].
//   KIN = true : global element (r, k) at base[r * ld + k]   (K contiguous)
//   KIN = false: global element (r, k) at base[k * ld + r]   (non-K index contiguous)
template <int ROWS, int THREADS, bool KIN, bool CONJ>
struct TileLoader {
    static constexpr int ELEMS = ROWS * kKT;
    static constexpr int PER_THREAD = (ELEMS + THREADS - 1) / THREADS;
    static constexpr int SP = ROWS + 2;   // LDS row stride (complex); ROWS % 32 == 0 so SP % 32 == 2

    cf regs[PER_THREAD];

    // element e of the tile handled by this thread in pass p
    __device__ __forceinline__ static void coords(int tid, int p, int &r, int &kk)
    {
        const int e = p * THREADS + tid;
        if (KIN) { kk = e % kKT; r = e / kKT; }
        else     { r = e % ROWS; kk = e / ROWS; }
    }

    __device__ __forceinline__ void load(const cf *base, int ld, int r0, int rmax, int k0, int kmax, int tid)
    {
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p) {
            int r, kk;
            coords(tid, p, r, kk);
            const int gr = r0 + r, gk = k0 + kk;
            const bool ok = (p * THREADS + tid < ELEMS) && gr < rmax && gk < kmax;
            // unconditional load from a clamped (valid) address, masked afterwards: no branch per load
            const int grc = gr < rmax ? gr : rmax - 1, gkc = gk < kmax ? gk : kmax - 1;
            cf v = KIN ? base[(size_t)grc * ld + gkc] : base[(size_t)gkc * ld + grc];
            if (!ok) v = mk(0.0f, 0.0f);
            if (CONJ) v.y = -v.y;
            regs[p] = v;
        }
    }

    __device__ __forceinline__ void store(cf *Ps, int tid) const
    {
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p) {
            int r, kk;
            coords(tid, p, r, kk);
            if (p * THREADS + tid < ELEMS) Ps[kk * SP + r] = regs[p];
        }
    }
};

template <int MT_, int NT_, int WM_, int WN_>
struct GemmTile {
    static constexpr int MT = MT_, NT = NT_, WM = WM_, WN = WN_;
    static constexpr int THREADS = 64 * WM * WN;
    static constexpr int IT = MT / WM / 32;   // 32x32 MFMA tiles per wave along M
    static constexpr int JT = NT / WN / 32;   // ... along N
    static constexpr int SA = MT + 2, SB = NT + 2;
    static constexpr int LDS_BYTES = kKT * (SA + SB) * 8;
    static_assert(MT % (32 * WM) == 0 && NT % (32 * WN) == 0, "wave tiles are multiples of 32x32");
};

// Launch: grid = bins * tiles_m * tiles_n blocks of G::THREADS threads, G::LDS_BYTES dynamic LDS.
template <class G, bool A_KIN, bool B_KIN, bool CONJ_A, bool CONJ_B>
__global__ __launch_bounds__(G::THREADS) void bin_cgemm_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *As = reinterpret_cast<cf *>(lds_raw);
    cf *Bs = As + kKT * G::SA;

    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % G::WM, wn = wave / G::WM;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber
    // them so that every XCD walks a contiguous range of (bin, tile) work: all tiles of
    // a bin then share one L2 and each operand panel is fetched from HBM once.
    const int total = (int)gridDim.x;
    const int xcd = (int)blockIdx.x % kXcds, slot = (int)blockIdx.x / kXcds;
    const int per = total / kXcds, rem = total % kXcds;
    const int work = g.xcd_remap ? xcd * per + (xcd < rem ? xcd : rem) + slot : (int)blockIdx.x;

    const int tiles = g.tiles_m * g.tiles_n;
    const int bin = work / tiles;
    const int t = work % tiles;
    const int i0 = (t % g.tiles_m) * G::MT, j0 = (t / g.tiles_m) * G::NT;

    // leading dimensions follow from the layouts: K-contiguous operands are [rows][Kd],
    // the others are [Kd][rows]
    const int lda = A_KIN ? g.Kd : g.Md;
    const int ldb = B_KIN ? g.Kd : g.Nd;
    const cf *Ab = g.A + (size_t)bin * g.Md * g.Kd;
    const cf *Bb = g.B + (size_t)bin * g.Nd * g.Kd;
    cf *Cb = g.C + (size_t)bin * g.Md * g.Nd;

    TileLoader<G::MT, G::THREADS, A_KIN, CONJ_A> la;
    TileLoader<G::NT, G::THREADS, B_KIN, CONJ_B> lb;

    floatx16 cre[G::IT][G::JT], cim[G::IT][G::JT];
#pragma unroll
    for (int a = 0; a < G::IT; ++a)
#pragma unroll
        for (int b = 0; b < G::JT; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) { cre[a][b][v] = 0.0f; cim[a][b][v] = 0.0f; }

    la.load(Ab, lda, i0, g.Md, 0, g.Kd, tid);
    lb.load(Bb, ldb, j0, g.Nd, 0, g.Kd, tid);

    const int lrow = lane & 31, lk = lane >> 5;
    const cf *Afrag = As + lk * G::SA + wm * (G::IT * 32) + lrow;
    const cf *Bfrag = Bs + lk * G::SB + wn * (G::JT * 32) + lrow;

    for (int k0 = 0; k0 < g.Kd; k0 += kKT) {
        la.store(As, tid);
        lb.store(Bs, tid);
        __syncthreads();
        if (k0 + kKT < g.Kd) {   // next chunk's loads fly during this chunk's MFMAs
            la.load(Ab, lda, i0, g.Md, k0 + kKT, g.Kd, tid);
            lb.load(Bb, ldb, j0, g.Nd, k0 + kKT, g.Kd, tid);
        }
#pragma unroll
        for (int ks = 0; ks < kKT / 2; ++ks) {
            cf af[G::IT], bf[G::JT];
            float nai[G::IT];
#pragma unroll
            for (int a = 0; a < G::IT; ++a) {
                af[a] = Afrag[(2 * ks) * G::SA + a * 32];
                nai[a] = -af[a].y;
            }
#pragma unroll
            for (int b = 0; b < G::JT; ++b) bf[b] = Bfrag[(2 * ks) * G::SB + b * 32];
#pragma unroll
            for (int a = 0; a < G::IT; ++a)
#pragma unroll
                for (int b = 0; b < G::JT; ++b) {
                    cre[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].x, bf[b].x, cre[a][b], 0, 0, 0);
                    cim[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].x, bf[b].y, cim[a][b], 0, 0, 0);
                }
#pragma unroll
            for (int a = 0; a < G::IT; ++a)
#pragma unroll
                for (int b = 0; b < G::JT; ++b) {
                    cre[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(nai[a], bf[b].y, cre[a][b], 0, 0, 0);
                    cim[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].y, bf[b].x, cim[a][b], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int a = 0; a < G::IT; ++a)
#pragma unroll
        for (int b = 0; b < G::JT; ++b) {
            const int col = j0 + wn * (G::JT * 32) + b * 32 + lrow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wm * (G::IT * 32) + a * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (row < g.Md && col < g.Nd)
                    Cb[(size_t)row * g.Nd + col] = mk(cre[a][b][v], cim[a][b][v]);
            }
        }
}

}  // namespace fftconv

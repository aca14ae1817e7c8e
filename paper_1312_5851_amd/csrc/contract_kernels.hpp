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
// Arithmetic.  A complex product needs three real products when sums of the
// operands are formed first (Karatsuba):
//     k1 = ar * br,   k2 = ai * bi,   k3 = (ar + ai) * (br + bi)
//     re = k1 - k2,   im = k3 - k1 - k2
// Each is accumulated over K by v_mfma_f32_32x32x2_f32 in its own fp32 tile, so a
// bin costs 6*M*N*K matrix-core flops instead of the 8*M*N*K of the four-product
// form; the operand sums are two VALU operations per fragment pair, and re/im are
// formed once in the epilogue.  A conjugated operand costs nothing: its sign goes
// into its sum (ar - ai or br - bi) and into the sign of k2 in the epilogue.
//
// Data flow.  A workgroup of WM x WN waves owns an MT x NT tile of one bin and
// walks K in chunks of kKT.  Operand chunks go global -> registers -> LDS, laid
// out Ps[k][r] (non-K index fastest), so the 32x2 operand fragment of an MFMA is
// one ds_read_b64 per lane: lane l reads Ps[k0 + l/32][r0 + l%32].  LDS holds two
// chunks: while chunk c is multiplied, chunk c+1 is written to the other half
// (its global loads were issued SETS chunks earlier, into one of SETS register sets;
// one set by default) and the loads of chunk c+1+SETS are issued; one barrier per chunk.  Fragments are double-buffered in registers so
// the LDS latency of step ks+1 hides behind the MFMAs of step ks.
//
// Vector-ALU instructions and MFMAs of the waves on a SIMD do not overlap (counters:
// no co-execution cycles; a chunk's 24 MFMAs take 1536 cycles, every other vector
// instruction four more), so the K loop carries as few of them as possible.  A tile
// that lies fully inside the matrices with K a multiple of the chunk takes the
// full-tile path: no masks, and every load address is a uniform (scalar) base plus one
// per-thread offset that never changes.  Edge tiles and K tails take the general path.
#pragma once
#include <hip/hip_runtime.h>

#include "contract_args.hpp"
#include "fft_core.hpp"

namespace fftconv {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;   // accelerator complex dies on MI355X; workgroups are dealt to them round-robin
constexpr int kKT = 16;    // complex K elements per chunk (one 128-byte line of a K-contiguous row)

// Moves one operand chunk (ROWS non-K indices x kKT K indices) global -> registers -> LDS.
//   KIN = true : global element (r, k) at base[r * ld + k]   (K contiguous)
//   KIN = false: global element (r, k) at base[k * ld + r]   (non-K index contiguous)
// LDS layout Ps[kk * SP + r].  SP is odd: the 16 lanes that an LDS store of 8-byte
// elements serves together then hit 16 different bank pairs whether they run along r
// (stride 1) or along kk (stride SP).
template <int ROWS, int THREADS, bool KIN>
struct TileLoader {
    static constexpr int ELEMS = ROWS * kKT;
    static constexpr int PER_THREAD = (ELEMS + THREADS - 1) / THREADS;
    static constexpr int SP = ROWS + 1;

    cf regs[PER_THREAD];
    unsigned okmask;   // bit p: element p of this thread lies inside the matrix

    __device__ __forceinline__ static void coords(int tid, int p, int &r, int &kk)
    {
        const int e = p * THREADS + tid;
        if (KIN) { kk = e % kKT; r = e / kKT; }
        else     { r = e % ROWS; kk = e / ROWS; }
    }

    // Issues the loads only.  Nothing here consumes the loaded values, so the loads stay
    // in flight while the caller goes on issuing MFMAs; masking of out-of-range elements
    // happens in store(), when the values are needed.
    __device__ __forceinline__ void load(const cf *base, int ld, int r0, int rmax, int k0, int kmax, int tid)
    {
        static_assert(PER_THREAD <= 32, "okmask holds one bit per element");
        okmask = 0;
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p) {
            int r, kk;
            coords(tid, p, r, kk);
            const int gr = r0 + r, gk = k0 + kk;
            const bool ok = (ELEMS % THREADS == 0 || p * THREADS + tid < ELEMS) && gr < rmax && gk < kmax;
            okmask |= (ok ? 1u : 0u) << p;
            // unconditional load from a clamped (valid) address: no branch per load
            const int grc = gr < rmax ? gr : rmax - 1, gkc = gk < kmax ? gk : kmax - 1;
            regs[p] = KIN ? base[(size_t)grc * ld + gkc] : base[(size_t)gkc * ld + grc];
        }
    }

    __device__ __forceinline__ void store(cf *Ps, int tid) const
    {
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p) {
            int r, kk;
            coords(tid, p, r, kk);
            cf v = regs[p];
            if (!((okmask >> p) & 1u)) v = mk(0.0f, 0.0f);
            if (ELEMS % THREADS == 0 || p * THREADS + tid < ELEMS) Ps[kk * SP + r] = v;
        }
    }
};

// The same for a tile that lies fully inside the matrix, K a multiple of kKT.  Element p of a
// thread is p * PSTEP rows (KIN) or K indices (not KIN) after its element 0, so its address is
// a uniform part (tile origin + chunk + p * PSTEP * ld) plus one per-thread offset that never
// changes.  The loads are buffer loads: the uniform part travels in a scalar register and the
// per-thread offset in one vector register, so a load costs no vector-ALU instruction.  Its LDS
// address is the thread's first one plus a compile-time constant.
typedef float floatx2 __attribute__((ext_vector_type(2)));
constexpr int kBufferWord3 = 0x00020000;   // raw buffer of 32-bit data on gfx9 (DATA_FORMAT = 32)

template <int ROWS, int THREADS, bool KIN>
struct FullTileLoader {
    static constexpr int ELEMS = ROWS * kKT;
    static constexpr int PER_THREAD = (ELEMS + THREADS - 1) / THREADS;
    static constexpr int SP = ROWS + 1;
    static constexpr int PSTEP = KIN ? THREADS / kKT : THREADS / ROWS;
    static constexpr int LDS_PSTEP = KIN ? PSTEP : PSTEP * SP;
    static_assert(KIN ? THREADS % kKT == 0 : THREADS % ROWS == 0, "elements of a thread differ by whole rows / K indices");

    cf regs[PER_THREAD];
    __amdgpu_buffer_rsrc_t rsrc;   // one bin's operand matrix
    unsigned voff;                 // byte offset of element 0 from the chunk's first element
    int lds_off;                   // LDS element index of element 0

    // `matrix`: the bin's operand matrix of `bytes` bytes (below 2 GB), leading dimension ld.
    __device__ __forceinline__ void init(const cf *matrix, unsigned bytes, int ld, int tid)
    {
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<cf *>(matrix), 0, (int)bytes, kBufferWord3);
        const int kk = KIN ? tid % kKT : tid / ROWS, r = KIN ? tid / kKT : tid % ROWS;
        voff = (unsigned)((KIN ? r * ld + kk : kk * ld + r) * 8);
        lds_off = kk * SP + r;
    }

    // `origin`: byte offset (uniform) of the tile's first element of this K chunk inside the matrix.
    __device__ __forceinline__ void load(int origin, int ld, int tid)
    {
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p)
            if (ELEMS % THREADS == 0 || p * THREADS + tid < ELEMS) {
                const floatx2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)voff, origin + p * PSTEP * ld * 8, 0);
                regs[p] = mk(v.x, v.y);
            }
    }

    __device__ __forceinline__ void store(cf *Ps, int tid) const
    {
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p)
            if (ELEMS % THREADS == 0 || p * THREADS + tid < ELEMS) Ps[lds_off + p * LDS_PSTEP] = regs[p];
    }
};

// IT x JT 32x32 MFMA tiles per wave, WM x WN waves per workgroup.  SETS register sets hold
// operand chunks on their way from global memory: a chunk reaches LDS SETS chunks after its
// loads were issued.  One set is enough when the matrix cores are the limit; products with
// little arithmetic per byte (f = 3) are bound by HBM latency instead and run with two.
template <int IT_, int JT_, int WM_, int WN_, int SETS_ = 1>
struct GemmTile {
    static constexpr int IT = IT_, JT = JT_, WM = WM_, WN = WN_, SETS = SETS_;
    static constexpr int MT = 32 * IT * WM, NT = 32 * JT * WN;
    static constexpr int THREADS = 64 * WM * WN;
    static constexpr int SA = MT + 1, SB = NT + 1;
    static constexpr int STAGE = kKT * (SA + SB);       // complex elements of one chunk (A then B)
    static constexpr int LDS_BYTES = 2 * STAGE * 8;     // two chunks
    static constexpr int ACC_REGS = 3 * IT * JT * 16;
    // waves per SIMD the register allocation must allow (the accumulators alone take ACC_REGS of 512), and no
    // more than LDS lets a CU hold anyway: a 128 x 32 tile takes 41.5 KB, so three workgroups of four waves
    // share a CU and a wave may use 168 registers instead of spilling at 128
    static constexpr int BY_LDS = (160 * 1024 / LDS_BYTES) * (WM * WN) / 4;
    static constexpr int BY_REGS =
        SETS > 1 ? 3 : (ACC_REGS <= 48 ? (WM * WN >= 4 ? 4 : 3) : (ACC_REGS <= 96 ? 2 : 1));
    static constexpr int WAVES_PER_SIMD = BY_LDS >= 1 && BY_LDS < BY_REGS ? BY_LDS : BY_REGS;
};

// The K loop of one tile.  la / lb are the two operands' loaders (general or full-tile), one per
// register set; chunk j travels through set j % SETS.  loadA(set, k0) / loadB(set, k0) issue the
// loads of the chunk starting at K index k0 into that set.
template <class G, bool CONJ_A, bool CONJ_B, class LA, class LB, class LoadA, class LoadB>
__device__ __forceinline__ void contract_tile(cf *lds, int tid, int lane, int wm, int wn, int nchunks,
                                              LA (&la)[G::SETS], LB (&lb)[G::SETS], LoadA &&loadA, LoadB &&loadB,
                                              floatx16 (&k1)[G::IT][G::JT], floatx16 (&k2)[G::IT][G::JT],
                                              floatx16 (&k3)[G::IT][G::JT])
{
    constexpr int IT = G::IT, JT = G::JT, KS = kKT / 2, SETS = G::SETS;
    // Prologue: request the first SETS chunks, hand chunk 0 to LDS, refill its set with chunk SETS.
    static_for<0, SETS>([&](auto si) {
        constexpr int set = decltype(si)::value;
        if (set == 0 || set < nchunks) {
            loadA(si, set * kKT);
            loadB(si, set * kKT);
        }
    });
    la[0].store(lds, tid);
    lb[0].store(lds + kKT * G::SA, tid);
    if (SETS < nchunks) {
        loadA(std::integral_constant<int, 0>{}, SETS * kKT);
        loadB(std::integral_constant<int, 0>{}, SETS * kKT);
    }
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    const int a_off = lk * G::SA + wm * (IT * 32) + lrow;
    const int b_off = kKT * G::SA + lk * G::SB + wn * (JT * 32) + lrow;

    // operand sums of the three-product form, with the sign of a conjugated operand folded in
    auto sum_a = [](cf a) { return CONJ_A ? a.x - a.y : a.x + a.y; };       // ar + ai'
    auto sum_b = [](cf b) { return CONJ_B ? b.x - b.y : b.x + b.y; };       // br + bi'

    // One K chunk; P = c % SETS is a compile-time value so that the set handed to LDS in this chunk
    // is a fixed group of registers.  In the first chunk the accumulators start from zero: its first
    // MFMAs take the constant 0 as their addend, which saves clearing 48 registers per tile beforehand.
    auto chunk = [&](auto first_tag, auto set_tag, int c) {
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr int Q = (decltype(set_tag)::value + 1) % SETS;   // set of chunk c + 1
        const std::integral_constant<int, Q> q_tag{};
        const cf *Af = lds + (c & 1) * G::STAGE + a_off;
        const cf *Bf = lds + (c & 1) * G::STAGE + b_off;
        cf af[2][IT], bf[2][JT];
        float as[2][IT], bs[2][JT];
#pragma unroll
        for (int a = 0; a < IT; ++a) {
            af[0][a] = Af[a * 32];
            as[0][a] = sum_a(af[0][a]);
        }
#pragma unroll
        for (int b = 0; b < JT; ++b) {
            bf[0][b] = Bf[b * 32];
            bs[0][b] = sum_b(bf[0][b]);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < KS) {   // fragments of the next step: their LDS latency hides behind this step's MFMAs
#pragma unroll
                for (int a = 0; a < IT; ++a) af[nxt][a] = Af[(2 * (ks + 1)) * G::SA + a * 32];
#pragma unroll
                for (int b = 0; b < JT; ++b) bf[nxt][b] = Bf[(2 * (ks + 1)) * G::SB + b * 32];
            }
            if (ks == KS / 2) {   // mid-chunk: hand the next chunk to LDS, refill its set with chunk c + 1 + SETS
                cf *stage = lds + ((c + 1) & 1) * G::STAGE;
                if (c + 1 < nchunks) {
                    la[Q].store(stage, tid);
                    lb[Q].store(stage + kKT * G::SA, tid);
                }
                if (c + 1 + SETS < nchunks) {
                    loadA(q_tag, (c + 1 + SETS) * kKT);
                    loadB(q_tag, (c + 1 + SETS) * kKT);
                }
            }
            // Order within a step: fragment reads (and staging) first, then this step's MFMAs,
            // then the operand sums of the NEXT step.  Left alone, the scheduler sinks the reads to
            // just before their use (LDS latency back on the critical path), and a sum computed right
            // before the MFMA that consumes it holds up the matrix pipe.
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < IT; ++a)
#pragma unroll
                for (int b = 0; b < JT; ++b) {
                    const floatx16 zero = {};
                    const bool start = FIRST && ks == 0;
                    k1[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][a].x, bf[cur][b].x, start ? zero : k1[a][b], 0, 0, 0);
                    k2[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][a].y, bf[cur][b].y, start ? zero : k2[a][b], 0, 0, 0);
                    k3[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(as[cur][a], bs[cur][b], start ? zero : k3[a][b], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 1 < KS) {
#pragma unroll
                for (int a = 0; a < IT; ++a) as[nxt][a] = sum_a(af[nxt][a]);
#pragma unroll
                for (int b = 0; b < JT; ++b) bs[nxt][b] = sum_b(bf[nxt][b]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };
    chunk(std::true_type{}, std::integral_constant<int, 0>{}, 0);
    for (int c = 1; c < nchunks; c += SETS)
        static_for<0, SETS>([&](auto pi) {
            constexpr int p = decltype(pi)::value;
            if (c + p < nchunks) chunk(std::false_type{}, std::integral_constant<int, (1 + p) % SETS>{}, c + p);
        });
}

// Workgroups are dealt round-robin to the XCDs (each with its own L2).  Renumbering them makes
// every XCD walk a contiguous range of (bin, tile) work: all tiles of a bin then share one L2.
__device__ __forceinline__ int xcd_contiguous_work(int remap)
{
    const int total = (int)gridDim.x;
    const int xcd = (int)blockIdx.x % kXcds, slot = (int)blockIdx.x / kXcds;
    const int per = total / kXcds, rem = total % kXcds;
    return remap ? xcd * per + (xcd < rem ? xcd : rem) + slot : (int)blockIdx.x;
}

// One workgroup's tile t of bin `bin`: C[bin] tile = op(A[bin]) * op(B[bin]).
template <class G, bool A_KIN, bool B_KIN, bool CONJ_A, bool CONJ_B>
__device__ __forceinline__ void cgemm_tile(const GemmArgs &g, int bin, int t, cf *lds)
{
    constexpr int IT = G::IT, JT = G::JT;
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % G::WM, wn = wave / G::WM;
    const int i0 = (t % g.tiles_m) * G::MT, j0 = (t / g.tiles_m) * G::NT;

    // leading dimensions follow from the layouts: K-contiguous operands are [rows][Kd],
    // the others are [Kd][rows]
    const int lda = A_KIN ? g.Kd : g.Md;
    const int ldb = B_KIN ? g.Kd : g.Nd;
    const cf *Ab = g.A + (size_t)bin * g.Md * g.Kd;
    const cf *Bb = g.B + (size_t)bin * g.Nd * g.Kd;
    cf *Cb = g.C + (size_t)bin * g.Md * g.Nd;

    floatx16 k1[IT][JT], k2[IT][JT], k3[IT][JT];   // written first by the MFMAs of the first K chunk

    const int nchunks = (g.Kd + kKT - 1) / kKT;
    // uniform across the workgroup: the tile lies inside both matrices and K has no tail
    const bool full = g.full_tiles_ok && i0 + G::MT <= g.Md && j0 + G::NT <= g.Nd && g.Kd % kKT == 0;
    if (full) {
        FullTileLoader<G::MT, G::THREADS, A_KIN> la[G::SETS];
        FullTileLoader<G::NT, G::THREADS, B_KIN> lb[G::SETS];
        static_for<0, G::SETS>([&](auto si) {
            la[decltype(si)::value].init(Ab, (unsigned)g.Md * (unsigned)g.Kd * 8u, lda, tid);
            lb[decltype(si)::value].init(Bb, (unsigned)g.Nd * (unsigned)g.Kd * 8u, ldb, tid);
        });
        contract_tile<G, CONJ_A, CONJ_B>(
            lds, tid, lane, wm, wn, nchunks, la, lb,
            [&](auto si, int k0) { la[decltype(si)::value].load((A_KIN ? i0 * lda + k0 : k0 * lda + i0) * 8, lda, tid); },
            [&](auto si, int k0) { lb[decltype(si)::value].load((B_KIN ? j0 * ldb + k0 : k0 * ldb + j0) * 8, ldb, tid); },
            k1, k2, k3);
    } else {
        TileLoader<G::MT, G::THREADS, A_KIN> la[G::SETS];
        TileLoader<G::NT, G::THREADS, B_KIN> lb[G::SETS];
        contract_tile<G, CONJ_A, CONJ_B>(
            lds, tid, lane, wm, wn, nchunks, la, lb,
            [&](auto si, int k0) { la[decltype(si)::value].load(Ab, lda, i0, g.Md, k0, g.Kd, tid); },
            [&](auto si, int k0) { lb[decltype(si)::value].load(Bb, ldb, j0, g.Nd, k0, g.Kd, tid); }, k1, k2, k3);
    }

    // 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    // k1 = sum ar br, k2 = sum ai bi (plain imaginary parts), k3 = sum (ar + ai')(br + bi'):
    //   re = k1 - s k2,  im = k3 - k1 - s k2,  s = -1 if exactly one operand is conjugated, else +1.
    constexpr bool ONE_CONJ = CONJ_A != CONJ_B;
    const int lrow = lane & 31, lk = lane >> 5;
    if (full) {
        // buffer stores: the per-lane part of the address is one register, the rest is uniform
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(Cb, 0, (int)((unsigned)g.Md * (unsigned)g.Nd * 8u), kBufferWord3);
        const int voff = ((wm * (IT * 32) + 4 * lk) * g.Nd + wn * (JT * 32) + lrow) * 8;
#pragma unroll
        for (int a = 0; a < IT; ++a)
#pragma unroll
            for (int b = 0; b < JT; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int soff = ((i0 + a * 32 + 8 * (v / 4) + (v % 4)) * g.Nd + j0 + b * 32) * 8;
                    floatx2 out;
                    out.x = ONE_CONJ ? k1[a][b][v] + k2[a][b][v] : k1[a][b][v] - k2[a][b][v];
                    out.y = ONE_CONJ ? (k3[a][b][v] - k1[a][b][v]) + k2[a][b][v] : (k3[a][b][v] - k1[a][b][v]) - k2[a][b][v];
                    __builtin_amdgcn_raw_buffer_store_b64(out, rsrc, voff, soff, 0);
                }
        return;
    }
#pragma unroll
    for (int a = 0; a < IT; ++a)
#pragma unroll
        for (int b = 0; b < JT; ++b) {
            const int col = j0 + wn * (JT * 32) + b * 32 + lrow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wm * (IT * 32) + a * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (row < g.Md && col < g.Nd) {
                    const float re = ONE_CONJ ? k1[a][b][v] + k2[a][b][v] : k1[a][b][v] - k2[a][b][v];
                    const float im = ONE_CONJ ? (k3[a][b][v] - k1[a][b][v]) + k2[a][b][v] : (k3[a][b][v] - k1[a][b][v]) - k2[a][b][v];
                    Cb[(size_t)row * g.Nd + col] = mk(re, im);
                }
            }
        }
}

// Launch: grid = bins * tiles_m * tiles_n blocks of G::THREADS threads, G::LDS_BYTES dynamic LDS.
template <class G, bool A_KIN, bool B_KIN, bool CONJ_A, bool CONJ_B>
__global__ __launch_bounds__(G::THREADS, G::WAVES_PER_SIMD) void bin_cgemm_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int work = xcd_contiguous_work(g.xcd_remap);
    const int tiles = g.tiles_m * g.tiles_n;
    cgemm_tile<G, A_KIN, B_KIN, CONJ_A, CONJ_B>(g, work / tiles, work % tiles, reinterpret_cast<cf *>(lds_raw));
}

// The contractions of bprop and accGrad in one launch (both read the spectrum of dL/dy, Eqs. 2 and 3):
// the work of a bin is its bprop tiles followed by its accGrad tiles, so the workgroups that read
// Gh[bin] for either product run next to each other on one XCD and the second read comes from its
// L2; one launch also has one ramp and one tail instead of two, and the tiles of one product fill the
// last, partly empty round of the other.  Launch: grid = bins * (tiles of bprop + tiles of accGrad).
template <class G>
__global__ __launch_bounds__(G::THREADS, G::WAVES_PER_SIMD) void bin_cgemm_bprop_accgrad_kernel(GemmPairArgs p)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    const int work = xcd_contiguous_work(p.bprop.xcd_remap);
    const int tiles_b = p.bprop.tiles_m * p.bprop.tiles_n, tiles_a = p.accgrad.tiles_m * p.accgrad.tiles_n;
    const int bin = work / (tiles_b + tiles_a), t = work % (tiles_b + tiles_a);
    if (t < tiles_b) cgemm_tile<G, true, false, false, false>(p.bprop, bin, t, lds);
    else cgemm_tile<G, false, false, true, false>(p.accgrad, bin, t - tiles_b, lds);
}

}  // namespace fftconv

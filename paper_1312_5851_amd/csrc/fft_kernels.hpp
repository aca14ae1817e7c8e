// Batched 2-D real-to-complex FFT of zero-padded maps, and the complex-to-real
// inverse fused with cropping (paper Sec. 2.2: transform every map once, crop
// the circular result; Sec. 2.3: a 2-D FFT is two sets of 1-D FFTs).
//
// Spectrum layout ("bin-major"): spec[c * M + m] is stored bin c of map m, complex
// interleaved.  A real map determines only half of its N x N spectrum (Sec. 2.3,
// symmetry of FFTs of real inputs).  Stored are exactly the bins that are not the
// conjugate of another stored bin, B = N*N/2 + 2 of them, in this order:
//     c in [0, N/2]            (ky = 0,   kx = c)
//     c in [N/2+1, N+1]        (ky = N/2, kx = c - (N/2+1))
//     c = N+2 + (ky-1)*N + kx  (ky in [1, N/2-1], kx in [0, N))
// (rows ky = 0 and ky = N/2 are Hermitian in kx, so only kx <= N/2 is kept).
// For a fixed bin the M maps are contiguous, which makes every bin a dense
// row-major matrix for the per-frequency contraction.
//
// One workgroup transforms T consecutive maps so that each bin is written (or
// read) as one contiguous run of T complex numbers.  The work is two phases
// separated by a workgroup barrier:
//
//   forward  A: lane <-> (map pair, column x).  Two real maps are packed as
//               one complex column (re = map a, im = map b), transformed along
//               y in registers, and split back into the two half spectra.
//            B: lane <-> (row ky, map).  Complex transform along x in
//               registers, then the bin-major store with lanes along maps.
//               The purely real rows ky = 0 and ky = N/2 of a map are packed
//               into one complex row ("row 0") and split after the transform.
//   inverse  runs the same two phases backwards and stores only the cropped
//            window, scaled by 1/N^2.
//
// Between the phases the data sits in LDS as lds[r][x][m] (m fastest) with
// strides padded so that both phases touch distinct banks.
//
// Each phase is a plain function of (thread id, block id): the device kernels
// call them around __syncthreads(), and a host build replays them in loops to
// check the index arithmetic without a GPU.
#pragma once
#include "fft_core.hpp"

namespace fftconv {

struct FwdArgs {
    const float *src;   // [M][ext][ext] real maps
    cf *spec;           // [B][M] bin-major spectrum, B = N*N/2 + 2 stored bins
    int M;              // number of maps
    int ext;            // spatial extent of a map (n, k or n'); everything beyond is zero padding
};

struct InvArgs {
    const cf *spec;     // [B][M]
    float *dst;         // [M][crop][crop]
    int M;
    int crop;           // stored window [0,crop)^2
    float scale;        // 1 / N^2
};

template <int N_, int T_, int NX_>
struct TileGeom {
    static constexpr int N = N_;     // transform size
    static constexpr int T = T_;     // maps per workgroup (even)
    static constexpr int NX = NX_;   // columns that can be non-zero (forward) / are needed (inverse)
    static constexpr int ROWS = N / 2;                 // packed row 0 + rows 1..N/2-1
    static constexpr int THREADS = T * ROWS;           // one lane per (row, map) in the x-phase
    static constexpr int SX = T + 1;                   // complex elements between consecutive x
    static constexpr int SR_BASE = NX * SX;
    // row stride: congruent to T modulo 32 complex (= 64 dwords) so that the row groups
    // sharing a half-wave in the x-phase start T complex apart in bank space
    static constexpr int SR = SR_BASE + ((((T - SR_BASE) % 32) + 32) % 32);
    static constexpr int LDS_ELEMS = ROWS * SR;
    static constexpr int LDS_BYTES = LDS_ELEMS * 8;
    static constexpr int YITEMS = (T / 2) * NX;        // work items of the y-phase
    static_assert(T % 2 == 0, "maps are processed in pairs");
    static_assert(NX <= N, "extent class cannot exceed the transform size");
};

// ------------------------------------------------------------------ forward

template <class G>
FC_HD void fwd_phase_y(int tid, int blk, const FwdArgs &a, cf *lds)
{
    constexpr int N = G::N, NX = G::NX;
    const int m0 = blk * G::T;
    for (int item = tid; item < G::YITEMS; item += G::THREADS) {
        const int p = item / NX, x = item % NX;
        const int ma = m0 + 2 * p, mb = ma + 1;
        // Loads are unconditional from clamped (always valid) addresses and masked
        // afterwards, so that they issue back to back; rows beyond the extent are
        // skipped by a wave-uniform branch.
        const bool va = (ma < a.M) && (x < a.ext), vb = (mb < a.M) && (x < a.ext);
        const int xc = x < a.ext ? x : a.ext - 1;
        const int mac = ma < a.M ? ma : a.M - 1, mbc = mb < a.M ? mb : a.M - 1;
        const float *pa = a.src + ((size_t)mac * a.ext) * a.ext + xc;
        const float *pb = a.src + ((size_t)mbc * a.ext) * a.ext + xc;
        float fa[NX], fb[NX];
        static_for<0, NX>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            if (y < a.ext) {
                fa[y] = pa[y * a.ext];
                fb[y] = pb[y * a.ext];
            } else {
                fa[y] = 0.0f;
                fb[y] = 0.0f;
            }
        });
        cf z[N];
        static_for<0, NX>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            z[y] = mk(va ? fa[y] : 0.0f, vb ? fb[y] : 0.0f);
        });
        fft_dif<N, false, ~low_mask(NX)>(z);
        cf *base = lds + x * G::SX + 2 * p;
        {   // packed row 0: (ky = 0, ky = N/2), both real for a real map
            const cf z0 = z[brev<N>(0)], zh = z[brev<N>(N / 2)];
            base[0] = mk(z0.x, zh.x);
            base[1] = mk(z0.y, zh.y);
        }
        static_for<1, N / 2>([&](auto ri) {
            constexpr int r = decltype(ri)::value;
            const cf zk = z[brev<N>(r)], zn = z[brev<N>(N - r)];
            // A = (Z[k] + conj Z[N-k]) / 2,  B = (Z[k] - conj Z[N-k]) / (2i)
            base[r * G::SR + 0] = mk(0.5f * (zk.x + zn.x), 0.5f * (zk.y - zn.y));
            base[r * G::SR + 1] = mk(0.5f * (zk.y + zn.y), 0.5f * (zn.x - zk.x));
        });
    }
}

template <class G>
FC_HD void fwd_phase_x(int tid, int blk, const FwdArgs &a, const cf *lds)
{
    constexpr int N = G::N, NX = G::NX;
    const int r = tid / G::T, m = tid % G::T;
    const int mg = blk * G::T + m;
    cf v[N];
    const cf *base = lds + r * G::SR + m;
    static_for<0, NX>([&](auto xi) {
        constexpr int x = decltype(xi)::value;
        v[x] = base[x * G::SX];
    });
    fft_dif<N, false, ~low_mask(NX)>(v);
    if (mg >= a.M) return;
    cf *out = a.spec + mg;
    const size_t M = (size_t)a.M;
    if (r != 0) {
        static_for<0, N>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            out[((size_t)(N + 2) + (size_t)(r - 1) * N + kx) * M] = v[brev<N>(kx)];
        });
    } else {
        // C = FFT(row0 + i rowH)  ->  row0[k] = (C[k] + conj C[-k]) / 2,  rowH[k] = (C[k] - conj C[-k]) / (2i);
        // both rows are Hermitian in k, only k <= N/2 is stored
        static_for<0, N / 2 + 1>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            const cf c = v[brev<N>(kx)], d = v[brev<N>((N - kx) % N)];
            out[(size_t)kx * M] = mk(0.5f * (c.x + d.x), 0.5f * (c.y - d.y));
            out[(size_t)(N / 2 + 1 + kx) * M] = mk(0.5f * (c.y + d.y), 0.5f * (d.x - c.x));
        });
    }
}

// ------------------------------------------------------------------ inverse

template <class G>
FC_HD void inv_phase_x(int tid, int blk, const InvArgs &a, cf *lds)
{
    constexpr int N = G::N, NX = G::NX;
    const int r = tid / G::T, m = tid % G::T;
    const int mg = blk * G::T + m;
    // Lanes beyond the last map read the last map's bins (valid memory) instead of
    // branching around each load; what they compute is never stored.
    const cf *in = a.spec + (mg < a.M ? mg : a.M - 1);
    const size_t M = (size_t)a.M;
    cf v[N];
    if (r != 0) {
        static_for<0, N>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            v[kx] = in[((size_t)(N + 2) + (size_t)(r - 1) * N + kx) * M];
        });
    } else {
        // rows ky = 0 and ky = N/2 are Hermitian in kx, so their inverse transforms are
        // real: send both through one complex transform as row0 + i rowH, rebuilding the
        // bins kx > N/2 that are not stored from their conjugates
        cf y0[N / 2 + 1], yh[N / 2 + 1];
        static_for<0, N / 2 + 1>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            y0[kx] = in[(size_t)kx * M];
            yh[kx] = in[(size_t)(N / 2 + 1 + kx) * M];
        });
        static_for<0, N / 2 + 1>([&](auto ki) {
            constexpr int kx = decltype(ki)::value;
            v[kx] = mk(y0[kx].x - yh[kx].y, y0[kx].y + yh[kx].x);                 // y0 + i yh
            if constexpr (kx > 0 && kx < N / 2)
                v[N - kx] = mk(y0[kx].x + yh[kx].y, yh[kx].x - y0[kx].y);        // conj y0 + i conj yh
        });
    }
    fft_dif<N, true, 0, first_outputs_mask<N>(NX)>(v);
    cf *base = lds + r * G::SR + m;
    static_for<0, NX>([&](auto xi) {
        constexpr int x = decltype(xi)::value;
        base[x * G::SX] = v[brev<N>(x)];
    });
}

// Stores one cropped output column (rows y < crop of one map at one x), scaled;
// with ACC the old values are all loaded first, then added, then stored.
template <class G, bool ACC, class Get>
FC_HD void store_column(float *col, bool valid, const InvArgs &a, Get &&get)
{
    if (!valid) return;
    float old[G::NX];
    if constexpr (ACC) {
        static_for<0, G::NX>([&](auto yi) {
            constexpr int y = decltype(yi)::value;
            old[y] = (y < a.crop) ? col[y * a.crop] : 0.0f;
        });
    }
    static_for<0, G::NX>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        if (y < a.crop) {
            if constexpr (ACC) col[y * a.crop] = old[y] + get(yi) * a.scale;
            else col[y * a.crop] = get(yi) * a.scale;
        }
    });
}

template <class G, bool ACC>
FC_HD void inv_phase_y(int tid, int blk, const InvArgs &a, const cf *lds)
{
    constexpr int N = G::N, NX = G::NX;
    const int m0 = blk * G::T;
    for (int item = tid; item < G::YITEMS; item += G::THREADS) {
        const int p = item / NX, x = item % NX;
        const int ma = m0 + 2 * p, mb = ma + 1;
        const cf *base = lds + x * G::SX + 2 * p;
        cf z[N];
        {
            const cf ra = base[0], rb = base[1];    // (row 0, row N/2) of map a / map b, all real
            z[0] = mk(ra.x, rb.x);
            z[N / 2] = mk(ra.y, rb.y);
        }
        static_for<1, N / 2>([&](auto ri) {
            constexpr int r = decltype(ri)::value;
            const cf A = base[r * G::SR + 0], B = base[r * G::SR + 1];
            z[r] = mk(A.x - B.y, A.y + B.x);        // A + i B
            z[N - r] = mk(A.x + B.y, B.x - A.y);    // conj A + i conj B
        });
        fft_dif<N, true, 0, first_outputs_mask<N>(NX)>(z);
        if (x >= a.crop) continue;
        store_column<G, ACC>(a.dst + ((size_t)ma * a.crop) * a.crop + x, ma < a.M, a, [&](auto yi) {
            return z[brev<N>(decltype(yi)::value)].x;
        });
        store_column<G, ACC>(a.dst + ((size_t)mb * a.crop) * a.crop + x, mb < a.M, a, [&](auto yi) {
            return z[brev<N>(decltype(yi)::value)].y;
        });
    }
}

#if defined(__HIPCC__)
// Device kernels: the two phases around one workgroup barrier.  Launch with
// G::THREADS threads, ceil(M / G::T) blocks and G::LDS_BYTES of dynamic LDS.
template <class G>
__global__ __launch_bounds__(G::THREADS) void fft2d_r2c_kernel(FwdArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    fwd_phase_y<G>((int)threadIdx.x, (int)blockIdx.x, a, lds);
    __syncthreads();
    fwd_phase_x<G>((int)threadIdx.x, (int)blockIdx.x, a, lds);
}

template <class G, bool ACC>   // ACC: dst += result instead of dst = result
__global__ __launch_bounds__(G::THREADS) void ifft2d_c2r_crop_kernel(InvArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    inv_phase_x<G>((int)threadIdx.x, (int)blockIdx.x, a, lds);
    __syncthreads();
    inv_phase_y<G, ACC>((int)threadIdx.x, (int)blockIdx.x, a, lds);
}
#endif

}  // namespace fftconv

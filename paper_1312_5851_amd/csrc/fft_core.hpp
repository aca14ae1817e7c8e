// In-register complex FFTs of size 2^m, 3 * 2^m, 5 * 2^m or 7 * 2^m with compile-time indexing.
//
// Every array index below is a compile-time constant after template expansion,
// so an N-point transform lives entirely in N complex registers of one lane
// (no scratch memory).  Sizes with a factor 3 (12, 24, 48), 5 (20, 40) or 7 (14, 28, 56) exist
// so that an input need not be padded all the way to the next power of two, the limitation
// the paper points out in Sec. 4.  The same header compiles for gfx950 device code and,
// without HIP, for a host build that replays the kernels' phases on the CPU.
//
// The 1-D transforms are the row / column building blocks of the 2-D
// decomposition described in Sec. 2.3 of the paper (two sets of 1-D FFTs).
// Convention: forward = exp(-2*pi*i*jk/N), unnormalised; inverse = exp(+...),
// also unnormalised (the 1/N^2 of the 2-D inverse is applied once at the
// final store).
#pragma once
#include <cstdint>
#include <type_traits>

#if defined(__HIPCC__)
#define FC_HD __host__ __device__ __forceinline__
#else
#define FC_HD inline __attribute__((always_inline))
#endif

namespace fftconv {

struct alignas(8) cf {
    float x, y;   // real, imaginary
};

FC_HD cf mk(float x, float y) { cf r; r.x = x; r.y = y; return r; }
FC_HD cf operator+(cf a, cf b) { return mk(a.x + b.x, a.y + b.y); }
FC_HD cf operator-(cf a, cf b) { return mk(a.x - b.x, a.y - b.y); }
FC_HD cf conj(cf a) { return mk(a.x, -a.y); }

// Compile-time loop: f(std::integral_constant<int, I>) for I in [B, E).
template <int B, int E, class F>
FC_HD void static_for(F &&f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// cos(2*pi*j/64), j = 0..16, rounded from a double-precision evaluation.
constexpr double kCos64[17] = {
    1.0,
    0.9951847266721969,
    0.9807852804032304,
    0.9569403357322088,
    0.9238795325112867,
    0.881921264348355,
    0.8314696123025452,
    0.773010453362737,
    0.7071067811865476,
    0.6343932841636455,
    0.5555702330196023,
    0.4713967368259978,
    0.38268343236508984,
    0.29028467725446233,
    0.19509032201612833,
    0.09801714032956077,
    0.0,
};

constexpr double cos64(int j)
{
    j &= 63;
    if (j <= 16) return kCos64[j];
    if (j <= 32) return -kCos64[32 - j];
    if (j <= 48) return -kCos64[j - 32];
    return kCos64[64 - j];
}
constexpr double sin64(int j) { return cos64(j + 48); }   // sin(t) = cos(t - pi/2)

constexpr int ilog2(int n) { return n <= 1 ? 0 : 1 + ilog2(n >> 1); }

// N = odd_radix(N) * pow2_part(N) with odd_radix in {1, 3, 5, 7}.
constexpr int odd_radix(int N) { return N % 3 == 0 ? 3 : (N % 5 == 0 ? 5 : (N % 7 == 0 ? 7 : 1)); }
constexpr int pow2_part(int N) { return N / odd_radix(N); }
constexpr bool fft_size_ok(int N) { const int M = pow2_part(N); return M >= 2 && (M & (M - 1)) == 0 && N <= 64; }

// Bit reversal of i within log2(M) bits.
constexpr int bitrev(int i, int M)
{
    int r = 0;
    for (int b = 0; b < ilog2(M); ++b)
        if (i & (1 << b)) r |= 1 << (ilog2(M) - 1 - b);
    return r;
}

// Position at which fft_dif leaves output X[k].  For N = 2^m the bit reversal of k; for
// N = R * M (R = 3, 5 or 7) the radix-R stage sends the outputs k = R q + r to block r, whose
// M-point transform leaves X[R q + r] at bit-reversed q.
template <int N>
constexpr int brev(int k)
{
    constexpr int R = odd_radix(N), M = pow2_part(N);
    return (k % R) * M + bitrev(k / R, M);
}

// cos / sin of 2*pi*p/d for angles that are not multiples of pi/32, evaluated at compile
// time in double precision (series on an angle reduced to at most pi/4).
constexpr double kPi = 3.141592653589793238462643383279502884;
constexpr double series_cos(double x)
{
    double term = 1.0, sum = 1.0;
    for (int i = 1; i <= 14; ++i) { term *= -x * x / ((2 * i - 1) * (2 * i)); sum += term; }
    return sum;
}
constexpr double series_sin(double x)
{
    double term = x, sum = x;
    for (int i = 1; i <= 14; ++i) { term *= -x * x / ((2 * i) * (2 * i + 1)); sum += term; }
    return sum;
}
constexpr double cos_ratio(long p, long d)   // cos(2 pi p / d)
{
    p %= d;
    if (p < 0) p += d;
    if (2 * p > d) p = d - p;                               // angle in [0, pi]
    if (4 * p > d) return -cos_ratio(d - 2 * p, 2 * d);     // cos(t) = -cos(pi - t)
    if (4 * p == d) return 0.0;
    if (8 * p > d) return series_sin(2.0 * kPi * (double)(d - 4 * p) / (double)(4 * d));   // cos(t) = sin(pi/2 - t)
    return series_cos(2.0 * kPi * (double)p / (double)d);
}

// cos / sin of 2*pi*q/N: from the table when the angle is a multiple of 2*pi/64, else computed.
template <int N>
constexpr double cos_n(int q) { return 64 % N == 0 ? cos64(q * (64 / N)) : cos_ratio(q, N); }
template <int N>
constexpr double sin_n(int q) { return 64 % N == 0 ? sin64(q * (64 / N)) : cos_ratio(4L * q - N, 4L * N); }

// Multiply v by exp(-/+ 2*pi*i*Q/N) (minus for forward, plus for inverse) with
// the trivial angles done without multiplications.
template <int N, int Q, bool INV>
FC_HD cf twiddle_mul(cf v)
{
    static_assert(fft_size_ok(N), "transform sizes are 2^m, 3 * 2^m, 5 * 2^m or 7 * 2^m, at most 64");
    constexpr int q = ((Q % N) + N) % N;
    if constexpr (q == 0) {
        return v;
    } else if constexpr (2 * q == N) {
        return mk(-v.x, -v.y);
    } else if constexpr (4 * q == N) {           // -i (forward) or +i (inverse)
        return INV ? mk(-v.y, v.x) : mk(v.y, -v.x);
    } else if constexpr (4 * q == 3 * N) {       // +i (forward) or -i (inverse)
        return INV ? mk(v.y, -v.x) : mk(-v.y, v.x);
    } else {
        constexpr float wr = (float)cos_n<N>(q);
        constexpr float wi = (float)(INV ? sin_n<N>(q) : -sin_n<N>(q));
        if constexpr (8 * q == N || 8 * q == 3 * N || 8 * q == 5 * N || 8 * q == 7 * N) {
            // |wr| == |wi| == sqrt(1/2): two adds and two multiplies
            constexpr float c = (float)kCos64[8];
            constexpr float sr = wr > 0 ? 1.0f : -1.0f, si = wi > 0 ? 1.0f : -1.0f;
            // (x + i y)(sr c + i si c) = c [ (sr x - si y) + i (si x + sr y) ]
            return mk(c * (sr * v.x - si * v.y), c * (si * v.x + sr * v.y));
        } else {
            return mk(v.x * wr - v.y * wi, v.x * wi + v.y * wr);
        }
    }
}

// Known-zero bookkeeping for pruned transforms: bit i of a mask set means
// "element i is known to be exactly zero at compile time".
constexpr uint64_t low_mask(int n) { return n >= 64 ? ~0ull : ((1ull << n) - 1ull); }

// Mask after the radix-R stage of an N = R M point transform (R = 3, 5 or 7): output r of
// butterfly j (position r M + j) is zero iff all R inputs j, j + M, ... are.
template <int N>
constexpr uint64_t odd_stage_mask(uint64_t zm)
{
    constexpr int R = odd_radix(N), M = N / R;
    uint64_t out = 0;
    for (int j = 0; j < M; ++j) {
        bool all = true;
        uint64_t bits = 0;
        for (int q = 0; q < R; ++q) {
            all = all && ((zm >> (j + q * M)) & 1);
            bits |= 1ull << (j + q * M);
        }
        if (all) out |= bits;
    }
    return out;
}

// Mask after one radix-2 decimation-in-frequency stage with half-span h.
template <int N>
constexpr uint64_t dif_stage_mask(uint64_t zm, int h)
{
    uint64_t out = 0;
    for (int s = 0; s < N; s += 2 * h)
        for (int j = 0; j < h; ++j) {
            const bool za = (zm >> (s + j)) & 1, zb = (zm >> (s + j + h)) & 1;
            if (za && zb) out |= (1ull << (s + j)) | (1ull << (s + j + h));
        }
    return out;
}

// Known zeros in front of radix-2 stage `stage` (after the odd-radix stage, if N has one).
template <int N>
constexpr uint64_t dif_mask_before_stage(uint64_t zm, int stage)
{
    if (odd_radix(N) > 1) zm = odd_stage_mask<N>(zm);
    int h = pow2_part(N) / 2;
    for (int s = 0; s < stage; ++s) {
        zm = dif_stage_mask<N>(zm, h);
        h /= 2;
    }
    return zm;
}

// Output pruning: bit i of a "need" mask set means "position i is read after
// the transform" (positions are the ones brev<N> names).  need_after_stage<N>(final, s)
// is the set of positions whose value after radix-2 stage s is still needed by some
// requested output; s = -1 gives what is needed in front of the first radix-2 stage,
// i.e. of the odd-radix stage's outputs.
template <int N>
constexpr uint64_t need_after_stage(uint64_t need_final, int stage)
{
    constexpr int M = pow2_part(N);
    uint64_t need = need_final;
    for (int st = ilog2(M) - 1; st > stage; --st) {
        const int h = M >> (st + 1);
        uint64_t prev = 0;
        for (int s = 0; s < N; s += 2 * h)
            for (int j = 0; j < h; ++j)
                if (((need >> (s + j)) & 1) || ((need >> (s + j + h)) & 1))
                    prev |= (1ull << (s + j)) | (1ull << (s + j + h));
        need = prev;
    }
    return need;
}

// Positions that hold natural-order outputs 0..count-1.
template <int N>
constexpr uint64_t first_outputs_mask(int count)
{
    uint64_t m = 0;
    for (int k = 0; k < count && k < N; ++k) m |= 1ull << brev<N>(k);
    return m;
}

// Radix-3 decimation-in-frequency butterfly j of an N = 3 M point transform, in place on
// a = v[j], b = v[j + M], c = v[j + 2 M]:
//     y_r = (a + w^r b + w^{2r} c) * exp(-/+ 2 pi i r j / N),   w = exp(-/+ 2 pi i / 3)
// ZB / ZC: b / c known to be zero (zero padding fills a map from the high indices down, so a
// known-zero b implies a known-zero c).  N0..N2: which outputs are read later.
template <int N, bool INV, int J, bool ZB, bool ZC, bool N0, bool N1, bool N2>
FC_HD void radix3_butterfly(cf &a, cf &b, cf &c)
{
    static_assert(!ZB || ZC, "zero padding is a suffix");
    constexpr float kHalfSqrt3 = 0.8660254037844386f;
    if constexpr (ZB) {           // only a: y_r = a * twiddle
        if constexpr (N1) b = twiddle_mul<N, J, INV>(a);
        if constexpr (N2) c = twiddle_mul<N, 2 * J, INV>(a);
    } else {
        cf s, d;                  // b + c, b - c
        if constexpr (ZC) { s = b; d = b; }
        else { s = b + c; d = b - c; }
        const cf t = mk(a.x - 0.5f * s.x, a.y - 0.5f * s.y);
        const cf e = mk(kHalfSqrt3 * d.y, -kHalfSqrt3 * d.x);   // -i sqrt(3)/2 (b - c)
        if constexpr (N0) a = a + s;
        if constexpr (N1) b = twiddle_mul<N, J, INV>(INV ? t - e : t + e);
        if constexpr (N2) c = twiddle_mul<N, 2 * J, INV>(INV ? t + e : t - e);
    }
}

// Of the R inputs j, j + M, ... of an odd-radix butterfly: how many leading ones can be
// non-zero, and whether the known zeros form a suffix.
constexpr int leading_nonzero(uint64_t zm, int j, int M, int R)
{
    int nz = 0;
    for (int q = 0; q < R; ++q)
        if (!((zm >> (j + q * M)) & 1)) nz = q + 1;
    return nz;
}
constexpr bool zero_suffix(uint64_t zm, int j, int M, int R)
{
    for (int q = 0; q < leading_nonzero(zm, j, M, R); ++q)
        if ((zm >> (j + q * M)) & 1) return false;
    return true;
}

// Bit r set: output r of the odd-radix butterfly j (position j + r M) is read later.
constexpr unsigned odd_need_bits(uint64_t need, int j, int M, int R)
{
    unsigned bits = 0;
    for (int r = 0; r < R; ++r) bits |= (unsigned)((need >> (j + r * M)) & 1) << r;
    return bits;
}

// Radix-5 decimation-in-frequency butterfly j of an N = 5 M point transform, in place on
// x_q = v[j + q M]:
//     y_r = (sum_q w^{r q} x_q) * exp(-/+ 2 pi i r j / N),   w = exp(-/+ 2 pi i / 5)
// written with the sums and differences of the pairs (x1, x4) and (x2, x3).  NZ: the first NZ
// inputs can be non-zero (zero padding is a suffix).  NEED bit r: output r is read later.
template <int N, bool INV, int J, int NZ, unsigned NEED>
FC_HD void radix5_butterfly(cf &x0, cf &x1, cf &x2, cf &x3, cf &x4)
{
    static_assert(NZ >= 1 && NZ <= 5, "at least the first input is non-zero");
    constexpr float c1 = (float)cos_ratio(1, 5), c2 = (float)cos_ratio(2, 5);     // cos(2 pi/5), cos(4 pi/5)
    constexpr float s1 = (float)cos_ratio(-1, 20), s2 = (float)cos_ratio(3, 20);  // sin(2 pi/5), sin(4 pi/5)
    cf y0, y1, y2, y3, y4;
    if constexpr (NZ == 1) {
        y0 = y1 = y2 = y3 = y4 = x0;
    } else {
        cf sa, da;                 // x1 + x4, x1 - x4
        if constexpr (NZ >= 5) { sa = x1 + x4; da = x1 - x4; }
        else { sa = x1; da = x1; }
        cf t1, t2, u1, u2;
        if constexpr (NZ >= 3) {
            cf sb, db;             // x2 + x3, x2 - x3
            if constexpr (NZ >= 4) { sb = x2 + x3; db = x2 - x3; }
            else { sb = x2; db = x2; }
            y0 = x0 + sa + sb;
            t1 = mk(x0.x + c1 * sa.x + c2 * sb.x, x0.y + c1 * sa.y + c2 * sb.y);
            t2 = mk(x0.x + c2 * sa.x + c1 * sb.x, x0.y + c2 * sa.y + c1 * sb.y);
            u1 = mk(s1 * da.x + s2 * db.x, s1 * da.y + s2 * db.y);
            u2 = mk(s2 * da.x - s1 * db.x, s2 * da.y - s1 * db.y);
        } else {
            y0 = x0 + sa;
            t1 = mk(x0.x + c1 * sa.x, x0.y + c1 * sa.y);
            t2 = mk(x0.x + c2 * sa.x, x0.y + c2 * sa.y);
            u1 = mk(s1 * da.x, s1 * da.y);
            u2 = mk(s2 * da.x, s2 * da.y);
        }
        const cf e1 = mk(u1.y, -u1.x), e2 = mk(u2.y, -u2.x);   // -i u
        y1 = INV ? t1 - e1 : t1 + e1;
        y4 = INV ? t1 + e1 : t1 - e1;
        y2 = INV ? t2 - e2 : t2 + e2;
        y3 = INV ? t2 + e2 : t2 - e2;
    }
    if constexpr (NEED & 1u) x0 = y0;
    if constexpr (NEED & 2u) x1 = twiddle_mul<N, J, INV>(y1);
    if constexpr (NEED & 4u) x2 = twiddle_mul<N, 2 * J, INV>(y2);
    if constexpr (NEED & 8u) x3 = twiddle_mul<N, 3 * J, INV>(y3);
    if constexpr (NEED & 16u) x4 = twiddle_mul<N, 4 * J, INV>(y4);
}

// Radix-7 decimation-in-frequency butterfly j of an N = 7 M point transform, in place on
// x_q = v[j + q M], written like the radix-5 one with the pairs (x1, x6), (x2, x5), (x3, x4):
//     y_0 = x0 + sum_k s_k,   s_k = x_k + x_{7-k},  d_k = x_k - x_{7-k}
//     y_r, y_{7-r} = t_r -/+ i u_r  (forward),   t_r = x0 + sum_k cos(2 pi r k / 7) s_k,
//                                                u_r = sum_k sin(2 pi r k / 7) d_k,   r, k = 1..3
// then the twiddle exp(-/+ 2 pi i r j / N).  NZ and NEED as for radix 5.
template <int N, bool INV, int J, int NZ, unsigned NEED>
FC_HD void radix7_butterfly(cf (&v)[N])
{
    static_assert(NZ >= 1 && NZ <= 7, "at least the first input is non-zero");
    constexpr int M = N / 7;
    cf y[7];
    const cf x0 = v[J];
    if constexpr (NZ == 1) {
        static_for<0, 7>([&](auto ri) { y[decltype(ri)::value] = x0; });
    } else {
        constexpr int P = NZ >= 4 ? 3 : NZ - 1;   // pairs with at least their first member non-zero
        cf s[3], d[3];
        static_for<0, P>([&](auto ki) {
            constexpr int k = decltype(ki)::value + 1;
            if constexpr (7 - k < NZ) {
                s[k - 1] = v[J + k * M] + v[J + (7 - k) * M];
                d[k - 1] = v[J + k * M] - v[J + (7 - k) * M];
            } else {
                s[k - 1] = v[J + k * M];
                d[k - 1] = v[J + k * M];
            }
        });
        y[0] = x0;
        static_for<0, P>([&](auto ki) { y[0] = y[0] + s[decltype(ki)::value]; });
        static_for<1, 4>([&](auto ri) {
            constexpr int r = decltype(ri)::value;
            cf t = x0, u = mk(0.0f, 0.0f);
            static_for<0, P>([&](auto ki) {
                constexpr int k = decltype(ki)::value + 1;
                constexpr float c = (float)cos_ratio(r * k, 7), sn = (float)cos_ratio(4L * (r * k) - 7, 28);
                t = mk(t.x + c * s[k - 1].x, t.y + c * s[k - 1].y);
                if constexpr (k == 1) u = mk(sn * d[0].x, sn * d[0].y);
                else u = mk(u.x + sn * d[k - 1].x, u.y + sn * d[k - 1].y);
            });
            const cf e = mk(u.y, -u.x);   // -i u
            y[r] = INV ? t - e : t + e;
            y[7 - r] = INV ? t + e : t - e;
        });
    }
    static_for<0, 7>([&](auto ri) {
        constexpr int r = decltype(ri)::value;
        if constexpr ((NEED >> r) & 1u) v[J + r * M] = twiddle_mul<N, r * J, INV>(y[r]);
    });
}

// Decimation-in-frequency FFT, in place, natural-order input, outputs left at the
// positions brev<N> names: X[k] = v[brev<N>(k)].  One radix-3, radix-5 or radix-7 stage first
// if N has that factor, then radix-2 stages.
// ZMASK marks inputs known to be zero (their registers are never read), which
// removes the arithmetic a zero-padded map does not need.  NEED marks the
// output positions that will be read; the others are left undefined, which
// removes the arithmetic a cropped result does not need.
template <int N, bool INV, uint64_t ZMASK = 0, uint64_t NEED = ~0ull>
FC_HD void fft_dif(cf (&v)[N])
{
    static_assert(fft_size_ok(N), "transform sizes are 2^m, 3 * 2^m, 5 * 2^m or 7 * 2^m, at most 64");
    constexpr int M = pow2_part(N);
    if constexpr (odd_radix(N) == 5) {
        constexpr uint64_t nd = need_after_stage<N>(NEED, -1);
        static_for<0, M>([&](auto ji) {
            constexpr int j = decltype(ji)::value;
            constexpr int nz = leading_nonzero(ZMASK, j, N / 5, 5);
            static_assert(zero_suffix(ZMASK, j, N / 5, 5), "zero padding is a suffix");
            constexpr unsigned need = (unsigned)(((nd >> j) & 1) | (((nd >> (j + M)) & 1) << 1) | (((nd >> (j + 2 * M)) & 1) << 2) |
                                                 (((nd >> (j + 3 * M)) & 1) << 3) | (((nd >> (j + 4 * M)) & 1) << 4));
            if constexpr (nz > 0)
                radix5_butterfly<N, INV, j, nz, need>(v[j], v[j + M], v[j + 2 * M], v[j + 3 * M], v[j + 4 * M]);
        });
    }
    if constexpr (odd_radix(N) == 7) {
        constexpr uint64_t nd = need_after_stage<N>(NEED, -1);
        static_for<0, M>([&](auto ji) {
            constexpr int j = decltype(ji)::value;
            constexpr int nz = leading_nonzero(ZMASK, j, N / 7, 7);
            static_assert(zero_suffix(ZMASK, j, N / 7, 7), "zero padding is a suffix");
            constexpr unsigned need = odd_need_bits(nd, j, N / 7, 7);
            if constexpr (nz > 0) radix7_butterfly<N, INV, j, nz, need>(v);
        });
    }
    if constexpr (odd_radix(N) == 3) {
        constexpr uint64_t nd = need_after_stage<N>(NEED, -1);
        static_for<0, M>([&](auto ji) {
            constexpr int j = decltype(ji)::value;
            constexpr bool za = (ZMASK >> j) & 1, zb = (ZMASK >> (j + M)) & 1, zc = (ZMASK >> (j + 2 * M)) & 1;
            static_assert(!za || (zb && zc), "zero padding is a suffix");
            if constexpr (!za)
                radix3_butterfly<N, INV, j, zb, zc, (nd >> j) & 1, (nd >> (j + M)) & 1, (nd >> (j + 2 * M)) & 1>(
                    v[j], v[j + M], v[j + 2 * M]);
        });
    }
    static_for<0, ilog2(M)>([&](auto st) {
        constexpr int stage = decltype(st)::value;
        constexpr int h = M >> (stage + 1);
        constexpr uint64_t zm = dif_mask_before_stage<N>(ZMASK, stage);
        constexpr uint64_t nd = need_after_stage<N>(NEED, stage);
        static_for<0, N / 2>([&](auto bi) {
            constexpr int b = decltype(bi)::value;
            constexpr int s = (b / h) * 2 * h, j = b % h;
            constexpr int ia = s + j, ib = s + j + h;
            constexpr bool za = (zm >> ia) & 1, zb = (zm >> ib) & 1;
            constexpr bool na = (nd >> ia) & 1, nb = (nd >> ib) & 1;
            constexpr int Q = j * (N / (2 * h));   // twiddle exp(-/+ 2 pi i j / (2h))
            if constexpr (za && zb) {
                // both zero: outputs are zero and are tracked as such, nothing to do
            } else if constexpr (zb) {
                if constexpr (nb) v[ib] = twiddle_mul<N, Q, INV>(v[ia]);
            } else if constexpr (za) {
                const cf c = v[ib];
                if constexpr (na) v[ia] = c;
                if constexpr (nb) v[ib] = twiddle_mul<N, Q + N / 2, INV>(c);   // -(c) * w
            } else {
                const cf a = v[ia], c = v[ib];
                if constexpr (na) v[ia] = a + c;
                if constexpr (nb) v[ib] = twiddle_mul<N, Q + 0, INV>(a - c);
            }
        });
    });
}

}  // namespace fftconv

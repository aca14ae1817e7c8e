// In-register power-of-two complex FFTs with compile-time indexing.
//
// Every array index below is a compile-time constant after template expansion,
// so an N-point transform lives entirely in N complex registers of one lane
// (no scratch memory).  The same header compiles for gfx950 device code and,
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

// Bit reversal of i within log2(N) bits.
template <int N>
constexpr int brev(int i)
{
    int r = 0;
    for (int b = 0; b < ilog2(N); ++b)
        if (i & (1 << b)) r |= 1 << (ilog2(N) - 1 - b);
    return r;
}

// Multiply v by exp(-/+ 2*pi*i*Q/N) (minus for forward, plus for inverse) with
// the trivial angles done without multiplications.
template <int N, int Q, bool INV>
FC_HD cf twiddle_mul(cf v)
{
    static_assert(N <= 64 && (64 % N) == 0, "twiddle table covers N up to 64");
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
        constexpr float wr = (float)cos64(q * (64 / N));
        constexpr float wi = (float)(INV ? sin64(q * (64 / N)) : -sin64(q * (64 / N)));
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

// Mask after one decimation-in-frequency stage with half-span h.
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

template <int N>
constexpr uint64_t dif_mask_before_stage(uint64_t zm, int stage)
{
    int h = N / 2;
    for (int s = 0; s < stage; ++s) {
        zm = dif_stage_mask<N>(zm, h);
        h /= 2;
    }
    return zm;
}

// Output pruning: bit i of a "need" mask set means "position i is read after
// the transform" (positions are the bit-reversed ones the DIF leaves its
// results in).  need_after_stage<N>(final, s) is the set of positions whose
// value after stage s is still needed by some requested output.
template <int N>
constexpr uint64_t need_after_stage(uint64_t need_final, int stage)
{
    uint64_t need = need_final;
    for (int st = ilog2(N) - 1; st > stage; --st) {
        const int h = N >> (st + 1);
        uint64_t prev = 0;
        for (int s = 0; s < N; s += 2 * h)
            for (int j = 0; j < h; ++j)
                if (((need >> (s + j)) & 1) || ((need >> (s + j + h)) & 1))
                    prev |= (1ull << (s + j)) | (1ull << (s + j + h));
        need = prev;
    }
    return need;
}

// Positions (bit-reversed) that hold natural-order outputs 0..count-1.
template <int N>
constexpr uint64_t first_outputs_mask(int count)
{
    uint64_t m = 0;
    for (int k = 0; k < count && k < N; ++k) m |= 1ull << brev<N>(k);
    return m;
}

// Radix-2 decimation-in-frequency FFT, in place, natural-order input,
// BIT-REVERSED output: X[k] = v[brev<N>(k)].
// ZMASK marks inputs known to be zero (their registers are never read), which
// removes the arithmetic a zero-padded map does not need.  NEED marks the
// output positions that will be read; the others are left undefined, which
// removes the arithmetic a cropped result does not need.
template <int N, bool INV, uint64_t ZMASK = 0, uint64_t NEED = ~0ull>
FC_HD void fft_dif(cf (&v)[N])
{
    static_for<0, ilog2(N)>([&](auto st) {
        constexpr int stage = decltype(st)::value;
        constexpr int h = N >> (stage + 1);
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
                if constexpr (nb) v[ib] = twiddle_mul<N, Q, INV>(a - c);
            }
        });
    });
}

}  // namespace fftconv

// Inverse 2-D transform + crop for small windows (the gradient of the kernels, Eq. 3, cropped to
// k x k with k <= N / 4), with every 1-D transform split over four neighbouring lanes.
//
// The one-lane-per-transform kernels of fft_kernels.hpp keep a whole N-point transform in a lane's
// registers: at N = 64 that is over 200 registers, two waves per SIMD and one workgroup per CU, and
// nothing hides the latency of the loads.  When only the first M = N / 4 outputs of a transform are
// needed (the extent class N / 4), the transform factors as
//
//     out[x] = sum_{q<4} e^{+2 pi i q x / N}  sum_{a<M} V[4a + q] e^{+2 pi i a x / M},   x in [0, M):
//
// lane q of a quad loads every fourth bin, runs an M-point transform in M complex registers,
// multiplies by its twiddle, and the quad's four partial results are added across lanes by two
// DPP adds (quad_perm), after which all four lanes hold out[0 .. M).  A lane then needs 2 M data
// registers instead of 2 N and four times as many lanes work on a tile.
//
// Measured on MI355X against the one-lane kernel (S = 128, f = f' = 256, k = 5): N = 64 326 to 344 us
// against 287 us, N = 48 59 against 55 us, N = 40 48 against 39 us, with the registers capped for two
// workgroups per CU (a few spilled) or not, and with the loads of both rounds issued up front or not.
// The one-lane kernel already moves its bytes at three quarters of the rate of a plain copy; what the
// split adds (a twiddle per value whose factor depends on the lane, the cross-lane sums, four lanes
// running the y-phase's address arithmetic for every output) costs more than the occupancy brings.
// The library therefore uses these kernels only when FFTCONV_QUAD is set in the environment.
//
// Layout, spectrum order and the packing of rows ky = 0 and ky = N/2 are those of fft_kernels.hpp.
// Phase x: lane <-> (row ky of this round, map, q); phase y: lane <-> (map pair, column, q).
// Between them the rows sit in LDS as lds[row][x][map], all rows of the tile at once (only
// M columns per row, so the tile fits).
#pragma once
#include "fft_kernels.hpp"

namespace fftconv {

template <int N_, int T_>
struct QuadGeom {
    static constexpr int N = N_, T = T_;
    static constexpr int M = N / 4;              // points per lane; also the columns / rows kept
    static constexpr int ROWS = N / 2;           // packed row 0 + rows 1 .. N/2 - 1
    static constexpr int ROUNDS = 2;             // the x-phase walks the rows in two halves
    static constexpr int RPR = ROWS / ROUNDS;
    static constexpr int THREADS = RPR * T * 4;  // x-phase lanes of one round
    static constexpr int SX = T + 1;             // complex elements between consecutive x
    static constexpr int SR = M * SX + 3;        // between consecutive rows: the four rows a quad gathers from start in different banks
    static constexpr int LDS_ELEMS = ROWS * SR;
    static constexpr int LDS_BYTES = LDS_ELEMS * 8;
    static constexpr int YITEMS = (T / 2) * M * 4;   // y-phase lanes
    // waves per SIMD the register allocation must allow: two workgroups per CU
    static constexpr int WAVES_PER_SIMD = (THREADS / 64 + 3) / 4;
    static_assert(N % 8 == 0 && fft_size_ok(M) && THREADS <= 1024 && YITEMS <= THREADS, "geometry");
};

// e^{+2 pi i q x / N} v for the lane's q in [0, 4): the three non-trivial factors are compile-time
// constants, picked by q.  (A table of the 4 M twiddles in LDS, read per lane, measured slower: its set-up
// and the extra registers cost more than the two spare products.)
template <int N, int X>
FC_HD cf quad_twiddle(cf v, int q)
{
    if constexpr (X == 0) {
        return v;
    } else {
        const cf t1 = twiddle_mul<N, X, true>(v), t2 = twiddle_mul<N, 2 * X, true>(v), t3 = twiddle_mul<N, 3 * X, true>(v);
        return q == 0 ? v : (q == 1 ? t1 : (q == 2 ? t2 : t3));
    }
}

// x-phase, step 1a: lane (slot, map, q) loads bins kx = 4a + q of its row (natural order in v).
template <class G>
FC_HD void quad_inv_x_load(int tid, int blk, int round, const InvArgs &a, cf (&v)[G::M])
{
    constexpr int N = G::N, M = G::M;
    const int q = tid % 4, m = (tid / 4) % G::T, slot = tid / (4 * G::T);
    const int r = round * G::RPR + slot;
    const int mg = blk * G::T + m;
    const int mc = mg < a.M ? mg : a.M - 1;   // lanes beyond the last map read the last map; nothing of theirs is stored
    const size_t Mt = (size_t)a.bin_stride;
    const cf *src = a.spec + mc;
    if (r != 0) {
        static_for<0, M>([&](auto ai) {
            constexpr int i = decltype(ai)::value;
            v[i] = src[((size_t)(N + 2) + (size_t)(r - 1) * N + 4 * i + q) * Mt];
        });
    } else {
        // rows ky = 0 and ky = N/2, each Hermitian in kx and stored for kx <= N/2, go through one transform as
        // row0 + i rowH; bin kx > N/2 is rebuilt from the conjugates of the stored bins N - kx
        static_for<0, M>([&](auto ai) {
            constexpr int i = decltype(ai)::value;
            const int kx = 4 * i + q;
            const bool direct = kx <= N / 2;
            const int idx = direct ? kx : N - kx;
            const cf y0 = src[(size_t)idx * Mt], yh = src[(size_t)(N / 2 + 1 + idx) * Mt];
            v[i] = direct ? mk(y0.x - yh.y, y0.y + yh.x) : mk(y0.x + yh.y, yh.x - y0.y);
        });
    }
}

// x-phase, step 1b: the lane's M-point transform, twiddled: u[x] is the lane's share of out[x].
template <class G>
FC_HD void quad_inv_x_partial(int tid, cf (&v)[G::M], cf (&u)[G::M])
{
    constexpr int N = G::N, M = G::M;
    const int q = tid % 4;
    fft_dif<M, true>(v);
    static_for<0, M>([&](auto xi) {
        constexpr int x = decltype(xi)::value;
        u[x] = quad_twiddle<N, x>(v[brev<M>(x)], q);
    });
}

// x-phase, step 2: the quad's sums are in u; lane q hands columns x = q, q + 4, ... of its row to LDS.
template <class G>
FC_HD void quad_inv_x_write(int tid, int round, cf *lds, const cf (&u)[G::M])
{
    const int q = tid % 4, m = (tid / 4) % G::T, slot = tid / (4 * G::T);
    cf *base = lds + (round * G::RPR + slot) * G::SR + m;
    static_for<0, G::M>([&](auto xi) {
        constexpr int x = decltype(xi)::value;
        if (x % 4 == q) base[x * G::SX] = u[x];
    });
}

// y-phase, step 1: lane (pair, column, q) collects rows ky = 4a + q of its column (the packed spectrum of the
// map pair, rebuilt as in fft_kernels.hpp) and leaves its twiddled partial transform in z (natural order).
template <class G>
FC_HD void quad_inv_y_partial(int tid, const cf *lds, cf (&z)[G::M])
{
    constexpr int N = G::N, M = G::M;
    const int q = tid % 4, x = (tid / 4) % M, p = tid / (4 * M);
    const cf *base = lds + x * G::SX + 2 * p;
    cf v[M];
    static_for<0, M>([&](auto ai) {
        constexpr int i = decltype(ai)::value;
        const int ky = 4 * i + q;
        if (ky == 0 || ky == N / 2) {
            const cf ra = base[0], rb = base[1];          // (row 0, row N/2) of map a / map b, all real
            v[i] = ky == 0 ? mk(ra.x, rb.x) : mk(ra.y, rb.y);
        } else {
            const bool direct = ky < N / 2;
            const int r = direct ? ky : N - ky;
            const cf A = base[r * G::SR + 0], B = base[r * G::SR + 1];
            v[i] = direct ? mk(A.x - B.y, A.y + B.x)       // A + i B
                          : mk(A.x + B.y, B.x - A.y);      // conj A + i conj B
        }
    });
    fft_dif<M, true>(v);
    static_for<0, M>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        z[y] = quad_twiddle<N, y>(v[brev<M>(y)], q);
    });
}

// y-phase, step 2: the quad's sums are in z (real part: map a, imaginary part: map b); lane q stores
// rows y = q, q + 4, ... of the cropped window, scaled; ACC adds to what is there.
template <class G, bool ACC>
FC_HD void quad_inv_y_store(int tid, int blk, const InvArgs &a, const cf (&z)[G::M])
{
    constexpr int M = G::M;
    const int q = tid % 4, x = (tid / 4) % M, p = tid / (4 * M);
    if (x >= a.crop_x) return;
    const int ma = blk * G::T + 2 * p, mb = ma + 1;
    // output (y, x) goes to window element (y, x), or (crop_y-1-y, crop_x-1-x) if flipped
    const int first = a.flip ? (a.crop_y - 1) * a.crop_x + (a.crop_x - 1 - x) : x;
    const int rstep = a.flip ? -a.crop_x : a.crop_x;
    float *da = a.dst + ((size_t)ma * a.crop_y) * a.crop_x + first;
    float *db = a.dst + ((size_t)mb * a.crop_y) * a.crop_x + first;
    static_for<0, M>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        if (y % 4 == q && y < a.crop_y) {
            if (ma < a.M) da[y * rstep] = (ACC ? da[y * rstep] : 0.0f) + z[y].x * a.scale;
            if (mb < a.M) db[y * rstep] = (ACC ? db[y * rstep] : 0.0f) + z[y].y * a.scale;
        }
    });
}

#if defined(__HIPCC__)
// Sum over the four lanes of a quad, left in all four: two cross-lane adds in the data-parallel
// primitive (DPP) path of the vector ALU, no LDS traffic.  (a + b) + (c + d) in every lane.
__device__ __forceinline__ float quad_allsum(float v)
{
    // quad_perm [1, 0, 3, 2]: each lane adds its neighbour; quad_perm [2, 3, 0, 1]: each pair adds the other pair
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    return v;
}

// Launch with G::THREADS threads, ceil(M / G::T) blocks and G::LDS_BYTES of dynamic LDS.
template <class G, bool ACC>
__global__ __launch_bounds__(G::THREADS, G::WAVES_PER_SIMD) void ifft2d_c2r_crop_quad_kernel(InvArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    cf *lds = reinterpret_cast<cf *>(lds_raw);
    const int tid = (int)threadIdx.x, blk = xcd_contiguous_block();
    // the loads of both rounds are issued before anything waits for them
    cf v[G::ROUNDS][G::M];
    static_for<0, G::ROUNDS>([&](auto ri) { quad_inv_x_load<G>(tid, blk, decltype(ri)::value, a, v[decltype(ri)::value]); });
    static_for<0, G::ROUNDS>([&](auto ri) {
        constexpr int round = decltype(ri)::value;
        cf u[G::M];
        quad_inv_x_partial<G>(tid, v[round], u);
        static_for<0, G::M>([&](auto xi) {
            constexpr int x = decltype(xi)::value;
            u[x] = mk(quad_allsum(u[x].x), quad_allsum(u[x].y));
        });
        quad_inv_x_write<G>(tid, round, lds, u);
    });
    __syncthreads();
    if (tid >= G::YITEMS) return;
    cf z[G::M];
    quad_inv_y_partial<G>(tid, lds, z);
    static_for<0, G::M>([&](auto yi) {
        constexpr int y = decltype(yi)::value;
        z[y] = mk(quad_allsum(z[y].x), quad_allsum(z[y].y));
    });
    quad_inv_y_store<G, ACC>(tid, blk, a, z);
}
#endif

}  // namespace fftconv

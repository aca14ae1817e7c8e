// C-ABI entry points of the fftconv library (declared in include/fftconv.h):
// plan bookkeeping, the spectral cache, kernel selection and launches.
// Host code only enqueues work on the caller's stream; all arithmetic of the
// path runs in the kernels of fft_kernels.hpp and contract_kernels.hpp.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/fftconv.h"
#include "contract_kernels.hpp"
#include "fft_dispatch.hpp"

using namespace fftconv;

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxProfileRecords = 4096;
constexpr int kNumCUs = 256;

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct ProfileRecord {
    int stage;
    hipEvent_t start, stop;
};

// ------------------------------------------------------------------ kernel tables

typedef void (*FwdKernel)(FwdArgs);
typedef void (*InvKernel)(InvArgs);
typedef void (*GemmKernel)(GemmArgs);

struct FftEntry {
    int N, T, NX, threads, lds_bytes;
    FwdKernel fwd;
    InvKernel inv, inv_acc;
};

#define X(n_, t_, nx_)                                                                          \
    {n_, t_, nx_, TileGeom<n_, t_, nx_, rounds_for(n_)>::THREADS, TileGeom<n_, t_, nx_, rounds_for(n_)>::LDS_BYTES, \
     fft2d_r2c_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>>,                                    \
     ifft2d_c2r_crop_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>, false>,                       \
     ifft2d_c2r_crop_kernel<TileGeom<n_, t_, nx_, rounds_for(n_)>, true>},
const FftEntry kFftTable[] = {FFTCONV_FOR_EACH_GEOM(X)};
#undef X

const FftEntry *find_fft(int N, int ext)
{
    const int T = maps_per_block(N), NX = extent_class(N, ext);
    for (const FftEntry &e : kFftTable)
        if (e.N == N && e.T == T && e.NX == NX) return &e;
    return nullptr;
}

struct GemmEntry {
    int MT, NT, wave_tiles, waves, occ, threads, lds_bytes;
    GemmKernel pass[3];   // indexed by FFTCONV_FPROP / BPROP / ACCGRAD
};

// Layout / conjugation per pass (see contract_kernels.hpp):
//   fprop   A = Xh [S][f]  K contiguous,  B = Wh [fo][f] K contiguous, conj B
//   bprop   A = Gh [S][fo] K contiguous,  B = Wh [fo][f] K outer
//   accGrad A = Gh [S][fo] K outer, conj A,  B = Xh [S][f] K outer
#define GEMM_ENTRY(it, jt, wm, wn, occ)                                                       \
    {GemmTile<it, jt, wm, wn>::MT, GemmTile<it, jt, wm, wn>::NT, it * jt, wm * wn, occ,          \
     GemmTile<it, jt, wm, wn>::THREADS, GemmTile<it, jt, wm, wn>::LDS_BYTES,                     \
     {bin_cgemm_kernel<GemmTile<it, jt, wm, wn>, true, true, false, true>,                       \
      bin_cgemm_kernel<GemmTile<it, jt, wm, wn>, true, false, false, false>,                     \
      bin_cgemm_kernel<GemmTile<it, jt, wm, wn>, false, false, true, false>}}
// (32x32 tiles per wave along M and N, waves along M and N, resident waves per SIMD)
const GemmEntry kGemmTable[] = {
    GEMM_ENTRY(2, 1, 2, 2, 3),   //  0: 128 x  64
    GEMM_ENTRY(1, 2, 2, 2, 3),   //  1:  64 x 128
    GEMM_ENTRY(1, 1, 2, 2, 4),   //  2:  64 x  64
    GEMM_ENTRY(2, 1, 1, 3, 3),   //  3:  64 x  96
    GEMM_ENTRY(2, 1, 2, 3, 3),   //  4: 128 x  96
    GEMM_ENTRY(1, 1, 2, 3, 4),   //  5:  64 x  96 (32 x 32 per wave)
    GEMM_ENTRY(1, 1, 1, 1, 4),   //  6:  32 x  32
    GEMM_ENTRY(1, 1, 4, 1, 4),   //  7: 128 x  32
    GEMM_ENTRY(2, 1, 2, 1, 3),   //  8: 128 x  32 (64 x 32 per wave)
    GEMM_ENTRY(2, 2, 2, 2, 1),   //  9: 128 x 128
    GEMM_ENTRY(1, 3, 2, 1, 2),   // 10:  64 x  96 (32 x 96 per wave)
    GEMM_ENTRY(1, 1, 4, 2, 4),   // 11: 128 x  64, 8 waves
    GEMM_ENTRY(1, 1, 2, 4, 4),   // 12:  64 x 128, 8 waves
    GEMM_ENTRY(1, 1, 4, 4, 4),   // 13: 128 x 128, 16 waves
    GEMM_ENTRY(1, 1, 4, 3, 4),   // 14: 128 x  96, 12 waves
};
#undef GEMM_ENTRY
constexpr int kNumGemm = sizeof(kGemmTable) / sizeof(kGemmTable[0]);

// Picks the tile shape.  Measured inside the full step on MI355X (operands coming from HBM,
// not from a cache warmed by the previous launch), the 4-wave shapes with one 32x32 tile per
// wave win over larger wave tiles and over 8- or 16-wave workgroups at these K: more
// independent workgroups per CU hide the per-tile prologue, epilogue and barrier waits.
// So the choice is among those: least padded work first, then the preference order.
int choose_gemm_tile(int Md, int Nd, int /*Kd*/, int /*bins*/)
{
    if (const char *env = std::getenv("FFTCONV_GEMM_TILE")) {
        const int v = std::atoi(env);
        if (v >= 0 && v < kNumGemm) return v;
    }
    static const int preference[] = {2, 7, 5, 6};   // 64x64, 128x32, 64x96, 32x32
    int best = preference[0];
    long best_area = -1;
    for (int i : preference) {
        const GemmEntry &e = kGemmTable[i];
        const long area = (long)((Md + e.MT - 1) / e.MT) * e.MT * ((Nd + e.NT - 1) / e.NT) * e.NT;
        if (best_area < 0 || area < best_area) { best_area = area; best = i; }
    }
    return best;
}

}  // namespace

struct fftconv_plan_s {
    fftconv_desc d;
    int no, N, B;
    long maps_x, maps_w, maps_g, maps_out;
    size_t off_x, off_w, off_g, off_out, ws_bytes;
    unsigned valid;
    void *last_ws;
    int gemm_tile[3];
    unsigned profiling;   // stage mask
    std::vector<ProfileRecord> records;
    std::vector<hipEvent_t> free_events;
};

namespace {

struct StageTimer {
    fftconv_plan_t p;
    hipStream_t stream;
    hipEvent_t stop;
    bool active;
    int status;
    StageTimer(fftconv_plan_t p_, int stage, hipStream_t s) : p(p_), stream(s), stop(nullptr), active(false), status(FFTCONV_OK)
    {
        if (((p->profiling >> stage) & 1u) == 0 || (int)p->records.size() >= kMaxProfileRecords) return;
        hipEvent_t ev[2];
        for (int i = 0; i < 2; ++i) {
            if (!p->free_events.empty()) {
                ev[i] = p->free_events.back();
                p->free_events.pop_back();
            } else if (hipEventCreate(&ev[i]) != hipSuccess) {
                status = FFTCONV_ELAUNCH;
                return;
            }
        }
        if (hipEventRecord(ev[0], stream) != hipSuccess) { status = FFTCONV_ELAUNCH; return; }
        p->records.push_back({stage, ev[0], ev[1]});
        stop = ev[1];
        active = true;
    }
    int finish()
    {
        if (active && hipEventRecord(stop, stream) != hipSuccess) return FFTCONV_ELAUNCH;
        return status;
    }
};

int check_launch() { return hipGetLastError() == hipSuccess ? FFTCONV_OK : FFTCONV_ELAUNCH; }

template <class K>
int allow_lds(K kernel, int bytes)
{
    if (bytes <= 64 * 1024) return FFTCONV_OK;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               bytes) == hipSuccess
               ? FFTCONV_OK
               : FFTCONV_ELAUNCH;
}

int bind_workspace(fftconv_plan_t p, void *ws)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return FFTCONV_EWORKSPACE;
    if (ws != p->last_ws) {
        p->valid = 0;
        p->last_ws = ws;
    }
    return FFTCONV_OK;
}

bool recompute_mode(fftconv_plan_t p) { return (p->d.flags & FFTCONV_RECOMPUTE) != 0; }

// Slot that receives a pass's result spectrum.  With the spectral cache it is the separate
// OUT slot; in the memory-efficient mode it is the one of the three slots the pass does not
// read, which has exactly the result's shape (Y like g, dX like x, dW like w).
int result_slot(fftconv_plan_t p, int pass)
{
    if (!recompute_mode(p)) return FFTCONV_SPEC_OUT;
    switch (pass) {
        case FFTCONV_FPROP: return FFTCONV_SPEC_G;
        case FFTCONV_BPROP: return FFTCONV_SPEC_X;
        default:            return FFTCONV_SPEC_W;
    }
}

cf *slot_ptr(fftconv_plan_t p, void *ws, int slot)
{
    size_t off = 0;
    switch (slot) {
        case FFTCONV_SPEC_X: off = p->off_x; break;
        case FFTCONV_SPEC_W: off = p->off_w; break;
        case FFTCONV_SPEC_G: off = p->off_g; break;
        default: off = p->off_out; break;
    }
    return reinterpret_cast<cf *>(static_cast<unsigned char *>(ws) + off);
}

int launch_forward(fftconv_plan_t p, int slot, const float *src, void *ws, hipStream_t stream)
{
    long M;
    int ext, stage;
    switch (slot) {
        case FFTCONV_SPEC_X: M = p->maps_x; ext = p->d.n; stage = FFTCONV_STAGE_FFT_X; break;
        case FFTCONV_SPEC_W: M = p->maps_w; ext = p->d.k; stage = FFTCONV_STAGE_FFT_W; break;
        case FFTCONV_SPEC_G: M = p->maps_g; ext = p->no; stage = FFTCONV_STAGE_FFT_G; break;
        default: return FFTCONV_EINVAL;
    }
    const FftEntry *e = find_fft(p->N, ext);
    if (!e) return FFTCONV_EUNSUPPORTED;
    if (int rc = allow_lds(e->fwd, e->lds_bytes)) return rc;
    FwdArgs a{src, slot_ptr(p, ws, slot), (int)M, ext};
    const unsigned blocks = (unsigned)((M + e->T - 1) / e->T);
    StageTimer timer(p, stage, stream);
    hipLaunchKernelGGL(e->fwd, dim3(blocks), dim3(e->threads), e->lds_bytes, stream, a);
    if (int rc = check_launch()) return rc;
    if (int rc = timer.finish()) return rc;
    p->valid |= (unsigned)slot;
    return FFTCONV_OK;
}

void pass_dims(fftconv_plan_t p, int pass, int &Md, int &Nd, int &Kd, int &slot_a, int &slot_b)
{
    switch (pass) {
        case FFTCONV_FPROP: Md = p->d.S; Nd = p->d.fo; Kd = p->d.f; slot_a = FFTCONV_SPEC_X; slot_b = FFTCONV_SPEC_W; break;
        case FFTCONV_BPROP: Md = p->d.S; Nd = p->d.f; Kd = p->d.fo; slot_a = FFTCONV_SPEC_G; slot_b = FFTCONV_SPEC_W; break;
        default:            Md = p->d.fo; Nd = p->d.f; Kd = p->d.S; slot_a = FFTCONV_SPEC_G; slot_b = FFTCONV_SPEC_X; break;
    }
}

int launch_contract(fftconv_plan_t p, int pass, void *ws, hipStream_t stream)
{
    int Md, Nd, Kd, sa, sb;
    pass_dims(p, pass, Md, Nd, Kd, sa, sb);
    if ((p->valid & (unsigned)sa) == 0 || (p->valid & (unsigned)sb) == 0) return FFTCONV_ENOTREADY;
    const GemmEntry &e = kGemmTable[p->gemm_tile[pass]];
    GemmArgs g;
    g.A = slot_ptr(p, ws, sa);
    g.B = slot_ptr(p, ws, sb);
    const int sc = result_slot(p, pass);
    g.C = slot_ptr(p, ws, sc);
    g.Md = Md; g.Nd = Nd; g.Kd = Kd;
    g.bins = p->B;
    g.tiles_m = (Md + e.MT - 1) / e.MT;
    g.tiles_n = (Nd + e.NT - 1) / e.NT;
    g.xcd_remap = std::getenv("FFTCONV_NO_XCD_REMAP") ? 0 : 1;
    const long blocks = (long)g.bins * g.tiles_m * g.tiles_n;
    if (blocks <= 0 || blocks > 0x7fffffffL) return FFTCONV_EUNSUPPORTED;
    if (int rc = allow_lds(e.pass[pass], e.lds_bytes)) return rc;
    StageTimer timer(p, FFTCONV_STAGE_CGEMM_FPROP + pass, stream);
    hipLaunchKernelGGL(e.pass[pass], dim3((unsigned)blocks), dim3(e.threads), e.lds_bytes, stream, g);
    if (int rc = check_launch()) return rc;
    if (sc != FFTCONV_SPEC_OUT) p->valid &= ~(unsigned)sc;   // an operand slot now holds a result spectrum
    return timer.finish();
}

int launch_inverse(fftconv_plan_t p, int pass, float *dst, void *ws, hipStream_t stream, int accumulate)
{
    long M;
    int crop;
    switch (pass) {
        case FFTCONV_FPROP: M = p->maps_g; crop = p->no; break;
        case FFTCONV_BPROP: M = p->maps_x; crop = p->d.n; break;
        default:            M = p->maps_w; crop = p->d.k; break;
    }
    const FftEntry *e = find_fft(p->N, crop);
    if (!e) return FFTCONV_EUNSUPPORTED;
    InvKernel kernel = accumulate ? e->inv_acc : e->inv;
    if (int rc = allow_lds(kernel, e->lds_bytes)) return rc;
    InvArgs a{slot_ptr(p, ws, result_slot(p, pass)), dst, (int)M, crop, 1.0f / ((float)p->N * (float)p->N)};
    const unsigned blocks = (unsigned)((M + e->T - 1) / e->T);
    StageTimer timer(p, FFTCONV_STAGE_IFFT_Y + pass, stream);
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(e->threads), e->lds_bytes, stream, a);
    if (int rc = check_launch()) return rc;
    return timer.finish();
}

int run_pass(fftconv_plan_t p, int pass, const float *src_a, const float *src_b, float *dst, void *ws, void *stream,
             int accumulate)
{
    if (!p || !src_a || !src_b || !dst) return FFTCONV_EINVAL;
    if (int rc = bind_workspace(p, ws)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int Md, Nd, Kd, sa, sb;
    pass_dims(p, pass, Md, Nd, Kd, sa, sb);
    if (recompute_mode(p)) p->valid = 0;   // every pass transforms both of its operands
    if ((p->valid & (unsigned)sa) == 0)
        if (int rc = launch_forward(p, sa, src_a, ws, s)) return rc;
    if ((p->valid & (unsigned)sb) == 0)
        if (int rc = launch_forward(p, sb, src_b, ws, s)) return rc;
    if (int rc = launch_contract(p, pass, ws, s)) return rc;
    const int rc = launch_inverse(p, pass, dst, ws, s, accumulate);
    if (recompute_mode(p)) p->valid = 0;
    return rc;
}

}  // namespace

extern "C" {

int fftconv_plan(fftconv_plan_t *out, const fftconv_desc *d)
{
    if (!out || !d) return FFTCONV_EINVAL;
    if (d->S < 1 || d->f < 1 || d->fo < 1 || d->n < 1 || d->k < 1 || d->k > d->n) return FFTCONV_EINVAL;
    if ((d->flags & ~(unsigned)FFTCONV_RECOMPUTE) != 0 || d->n > 64) return FFTCONV_EUNSUPPORTED;
    const long maps_x = (long)d->S * d->f, maps_w = (long)d->fo * d->f, maps_g = (long)d->S * d->fo;
    if (maps_x > 0x7fffffffL || maps_w > 0x7fffffffL || maps_g > 0x7fffffffL) return FFTCONV_EUNSUPPORTED;
    fftconv_plan_s *p = new (std::nothrow) fftconv_plan_s();
    if (!p) return FFTCONV_EINVAL;
    p->d = *d;
    p->no = d->n - d->k + 1;
    p->N = fft_size_for(d->n);
    p->B = p->N * p->N / 2 + 2;
    p->maps_x = maps_x;
    p->maps_w = maps_w;
    p->maps_g = maps_g;
    p->maps_out = maps_x > maps_w ? (maps_x > maps_g ? maps_x : maps_g) : (maps_w > maps_g ? maps_w : maps_g);
    const size_t per_map = (size_t)8 * p->B;
    p->off_x = 0;
    p->off_w = p->off_x + align_up(per_map * maps_x);
    p->off_g = p->off_w + align_up(per_map * maps_w);
    p->off_out = p->off_g + align_up(per_map * maps_g);
    p->ws_bytes = p->off_out + align_up(per_map * p->maps_out);
    if (recompute_mode(p)) {   // three slots only: a pass writes its result into the one it does not read
        p->ws_bytes = p->off_out;
        p->off_out = (size_t)-1;
        p->maps_out = -1;
    }
    p->valid = 0;
    p->last_ws = nullptr;
    p->profiling = 0;
    for (int pass = 0; pass < 3; ++pass) {
        int Md, Nd, Kd, sa, sb;
        pass_dims(p, pass, Md, Nd, Kd, sa, sb);
        p->gemm_tile[pass] = choose_gemm_tile(Md, Nd, Kd, p->B);
    }
    *out = p;
    return FFTCONV_OK;
}

int fftconv_plan_destroy(fftconv_plan_t p)
{
    if (!p) return FFTCONV_EINVAL;
    for (ProfileRecord &r : p->records) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    for (hipEvent_t e : p->free_events) (void)hipEventDestroy(e);
    delete p;
    return FFTCONV_OK;
}

int fftconv_fft_size(fftconv_plan_t p) { return p ? p->N : -1; }
int fftconv_num_bins(fftconv_plan_t p) { return p ? p->B : -1; }
size_t fftconv_workspace_bytes(fftconv_plan_t p) { return p ? p->ws_bytes : 0; }

size_t fftconv_slot_offset(fftconv_plan_t p, int slot)
{
    if (!p) return (size_t)-1;
    switch (slot) {
        case FFTCONV_SPEC_X: return p->off_x;
        case FFTCONV_SPEC_W: return p->off_w;
        case FFTCONV_SPEC_G: return p->off_g;
        case FFTCONV_SPEC_OUT: return p->off_out;
        default: return (size_t)-1;
    }
}

long fftconv_slot_maps(fftconv_plan_t p, int slot)
{
    if (!p) return -1;
    switch (slot) {
        case FFTCONV_SPEC_X: return p->maps_x;
        case FFTCONV_SPEC_W: return p->maps_w;
        case FFTCONV_SPEC_G: return p->maps_g;
        case FFTCONV_SPEC_OUT: return p->maps_out;
        default: return -1;
    }
}

int fftconv_invalidate(fftconv_plan_t p, unsigned slots)
{
    if (!p || (slots & ~(unsigned)(FFTCONV_SPEC_X | FFTCONV_SPEC_W | FFTCONV_SPEC_G)) != 0) return FFTCONV_EINVAL;
    p->valid &= ~slots;
    return FFTCONV_OK;
}

unsigned fftconv_valid_slots(fftconv_plan_t p) { return p ? p->valid : 0; }

int fftconv_fprop(fftconv_plan_t p, const float *x, const float *w, float *y, void *ws, void *stream)
{
    return run_pass(p, FFTCONV_FPROP, x, w, y, ws, stream, 0);
}

int fftconv_bprop(fftconv_plan_t p, const float *g, const float *w, float *dx, void *ws, void *stream)
{
    return run_pass(p, FFTCONV_BPROP, g, w, dx, ws, stream, 0);
}

int fftconv_accgrad(fftconv_plan_t p, const float *g, const float *x, float *dw, void *ws, void *stream, int accumulate)
{
    return run_pass(p, FFTCONV_ACCGRAD, g, x, dw, ws, stream, accumulate);
}

int fftconv_forward_transform(fftconv_plan_t p, int slot, const float *src, void *ws, void *stream)
{
    if (!p || !src) return FFTCONV_EINVAL;
    if (slot != FFTCONV_SPEC_X && slot != FFTCONV_SPEC_W && slot != FFTCONV_SPEC_G) return FFTCONV_EINVAL;
    if (int rc = bind_workspace(p, ws)) return rc;
    return launch_forward(p, slot, src, ws, static_cast<hipStream_t>(stream));
}

int fftconv_contract(fftconv_plan_t p, int pass, void *ws, void *stream)
{
    if (!p || pass < 0 || pass > 2) return FFTCONV_EINVAL;
    if (int rc = bind_workspace(p, ws)) return rc;
    return launch_contract(p, pass, ws, static_cast<hipStream_t>(stream));
}

int fftconv_inverse_transform(fftconv_plan_t p, int pass, float *dst, void *ws, void *stream, int accumulate)
{
    if (!p || !dst || pass < 0 || pass > 2) return FFTCONV_EINVAL;
    if (int rc = bind_workspace(p, ws)) return rc;
    return launch_inverse(p, pass, dst, ws, static_cast<hipStream_t>(stream), accumulate);
}

int fftconv_profile_enable(fftconv_plan_t p, unsigned stage_mask)
{
    if (!p || (stage_mask & ~FFTCONV_PROFILE_ALL) != 0) return FFTCONV_EINVAL;
    p->profiling = stage_mask;
    return FFTCONV_OK;
}

int fftconv_profile_read(fftconv_plan_t p, double *ms_sum, long *launches)
{
    if (!p || !ms_sum || !launches) return FFTCONV_EINVAL;
    int status = FFTCONV_OK;
    for (ProfileRecord &r : p->records) {
        float ms = 0.0f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
            status = FFTCONV_ELAUNCH;
        } else if (r.stage >= 0 && r.stage < FFTCONV_NUM_STAGES) {
            ms_sum[r.stage] += (double)ms;
            launches[r.stage] += 1;
        }
        p->free_events.push_back(r.start);
        p->free_events.push_back(r.stop);
    }
    p->records.clear();
    return status;
}

const char *fftconv_strerror(int status)
{
    switch (status) {
        case FFTCONV_OK: return "ok";
        case FFTCONV_EINVAL: return "invalid argument";
        case FFTCONV_EUNSUPPORTED: return "unsupported layer (n > 64 or unknown flags)";
        case FFTCONV_EWORKSPACE: return "workspace pointer null or not 256-byte aligned";
        case FFTCONV_ELAUNCH: return "HIP launch or event call failed";
        case FFTCONV_ENOTREADY: return "operand spectrum not cached for this workspace";
        default: return "unknown status";
    }
}

size_t fftconv_paper_ram_bytes(int S, int n, int f, int fo)
{
    if (S < 1 || n < 1 || f < 1 || fo < 1) return 0;
    return (size_t)4 * n * (n + 1) * ((size_t)S * f + (size_t)S * fo + (size_t)f * fo);
}

double fftconv_contraction_flops(fftconv_plan_t p)
{
    if (!p) return 0.0;
    return 6.0 * p->d.S * p->d.f * p->d.fo * p->B;
}

}  // extern "C"

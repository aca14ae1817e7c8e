// C-ABI entry points of the fftconv library (declared in include/fftconv.h):
// plan bookkeeping, the spectral cache, kernel selection and launches.
// Host code only enqueues work on the caller's stream; all arithmetic of the
// path runs in the kernels of fft_kernels.hpp, contract_kernels.hpp and
// skinny_kernels.hpp, which are instantiated in translation units of their own
// (kernel_tables.hpp).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/fftconv.h"
#include "kernel_tables.hpp"

using namespace fftconv;

// Workspace of fftconv_pass_static: part of the code object, one copy per GPU.  Host code never
// uses this name as an address; it asks the runtime for the copy's address on the current device
// (static_scratch_ptr below) and passes that to the kernels like any caller-owned workspace.
static __device__ __align__(256) unsigned char scratch[FFTCONV_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxProfileRecords = 4096;
constexpr int kNumCUs = 256;

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct ProfileRecord {
    int stage;
    hipEvent_t start, stop;
};

// ------------------------------------------------------------------ kernel lookup

// Everything a launch of one transform geometry needs: the forward, inverse and tiled kernels of
// (N, T, NX) live in three tables (kernel_tables.hpp).
struct FftEntry {
    int N, T, NX, threads, lds_bytes;
    FwdKernel fwd, fwd_tiled;
    InvKernel inv, inv_acc, inv_tiled, inv_tiled_add;
};

// `maps`: transforms in the launch, or 0 for a launch that must use the usual maps per workgroup (tiled and
// fused kernels exist for those only).
bool find_fft(int N, int ext, long maps, FftEntry &e)
{
    const int T = maps > 0 ? maps_per_block_for(N, maps, true) : maps_per_block(N), NX = extent_class(N, ext);
    const FwdEntry *f = find_fwd_kernels(N, T, NX);
    const InvEntry *i = find_inv_kernels(N, T, NX);
    if (!f || !i) return false;
    const InvTiledEntry *t = find_inv_tiled_kernels(N, T, NX);
    e = FftEntry{N, T, NX, f->threads, f->lds_bytes, f->plain, f->tiled, i->plain, i->acc,
                 t ? t->tiled : nullptr, t ? t->tiled_add : nullptr};
    return true;
}

// Switches for measurements and tests, read from the environment once, when a plan is made.
struct Switches {
    int gemm_tile;   // forced tile shape of the contraction, or -1
    bool no_xcd_remap, no_full_tiles, no_skinny, no_shared_pass, no_fused, no_fused_order, quad, no_small_batch;
};

Switches read_switches()
{
    Switches sw{};
    sw.gemm_tile = -1;
    if (const char *env = std::getenv("FFTCONV_GEMM_TILE")) {
        const int v = std::atoi(env);
        if (v >= 0 && v < gemm_kernel_count()) sw.gemm_tile = v;
    }
    sw.no_xcd_remap = std::getenv("FFTCONV_NO_XCD_REMAP") != nullptr;
    sw.no_full_tiles = std::getenv("FFTCONV_NO_FULL_TILES") != nullptr;
    sw.no_skinny = std::getenv("FFTCONV_NO_SKINNY") != nullptr;
    sw.no_shared_pass = std::getenv("FFTCONV_NO_SHARED_PASS") != nullptr;
    sw.no_fused = std::getenv("FFTCONV_NO_FUSED") != nullptr;
    sw.no_fused_order = std::getenv("FFTCONV_NO_FUSED_ORDER") != nullptr;
    sw.quad = std::getenv("FFTCONV_QUAD") != nullptr;
    sw.no_small_batch = std::getenv("FFTCONV_NO_SMALL_BATCH") != nullptr;
    return sw;
}

// Picks the tile shape: least padded work first, then the order of the table.
int choose_gemm_tile(int Md, int Nd, const Switches &sw)
{
    if (sw.gemm_tile >= 0) return sw.gemm_tile;
    int best = 0;
    long best_area = -1;
    for (int i = 0; i < gemm_shape_count(); ++i) {
        const GemmEntry &e = gemm_kernel_table()[i];
        const long area = (long)((Md + e.MT - 1) / e.MT) * e.MT * ((Nd + e.NT - 1) / e.NT) * e.NT;
        if (best_area < 0 || area < best_area) { best_area = area; best = i; }
    }
    return best;
}

}  // namespace

struct fftconv_plan_s {
    fftconv_desc2d d;
    int noh, now, N, B;
    // Tiling (maps larger than 64 only; otherwise Ly = Lx = 0 and one "tile" per image): tiles
    // are Ly x Lx output blocks, nty x ntx of them for y (and for the blocks of dL/dy and the
    // windows of x), nty2 x ntx2 for dx (and for the windows of dL/dy that bprop reads).
    int Ly, Lx, nty, ntx, nty2, ntx2;
    // Tiled layers with far fewer input than output maps: bprop multiplies the same zero-padded
    // blocks of dL/dy that accGrad transforms (no second transform of dL/dy, no G2 slot) and
    // adds the overlapping N x N windows of the result into dx (overlap-add).
    bool overlap_add;
    long maps_x, maps_w, maps_g, maps_g2, maps_out;   // transforms per slot
    size_t off_x, off_w, off_g, off_g2, off_out, ws_bytes;
    unsigned valid;
    // Layers with few input maps, spectra cached: bprop and accGrad form both of their result
    // spectra in one pass over the spectrum of dL/dy (whichever runs first does), side by side in
    // the OUT slot; `ready` says which of the two is waiting there for its pass (kReady*).
    bool shared_pass_ok;
    size_t off_shared_dw;   // byte offset of dWh inside the OUT slot (dXh is at its start)
    size_t off_shared_part; // ... and of the partial sums of dWh, if a bin's rows are split over several workgroups
    int shared_row_groups;
    unsigned ready;
    void *last_ws;
    int gemm_tile[3];
    int pair_tile;   // tile shape of the joint bprop + accGrad launch
    Switches sw;
    // Set at the first launch: the device the plan runs on (cached spectra and raised LDS limits
    // belong to it), and the kernels whose dynamic-LDS limit has been raised above 64 KB there.
    int device;
    std::vector<const void *> lds_raised;
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
                if (i == 1) p->free_events.push_back(ev[0]);
                status = FFTCONV_ELAUNCH;
                return;
            }
        }
        if (hipEventRecord(ev[0], stream) != hipSuccess) {
            p->free_events.push_back(ev[0]);
            p->free_events.push_back(ev[1]);
            status = FFTCONV_ELAUNCH;
            return;
        }
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

// A kernel needs its dynamic-LDS limit raised once before it may be launched with more than 64 KB;
// the plan remembers for which kernels that has been done on its device (a kernel's LDS size is
// fixed per plan).
template <class K>
int allow_lds(fftconv_plan_t p, K kernel, int bytes)
{
    if (bytes <= 64 * 1024) return FFTCONV_OK;
    const void *fn = reinterpret_cast<const void *>(kernel);
    for (const void *done : p->lds_raised)
        if (done == fn) return FFTCONV_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return FFTCONV_ELAUNCH;
    p->lds_raised.push_back(fn);
    return FFTCONV_OK;
}

int bind_workspace(fftconv_plan_t p, void *ws)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return FFTCONV_EWORKSPACE;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) {   // no GPU: argument checks still answer, any launch will fail
        (void)hipGetLastError();
        device = -1;
    }
    if (device != p->device) {   // first launch, or the caller moved to another GPU: nothing carries over
        p->device = device;
        p->lds_raised.clear();
        p->last_ws = nullptr;
    }
    if (ws != p->last_ws) {
        p->valid = 0;
        p->ready = 0;
        p->last_ws = ws;
    }
    return FFTCONV_OK;
}

bool recompute_mode(fftconv_plan_t p) { return (p->d.flags & FFTCONV_RECOMPUTE) != 0; }

constexpr unsigned kReadyDX = 1u, kReadyDW = 2u;

// A result spectrum waiting in the OUT slot goes stale with the operand spectra it was formed from.
void operands_changed(fftconv_plan_t p, unsigned slots)
{
    if (slots & (FFTCONV_SPEC_G | FFTCONV_SPEC_G2)) p->ready = 0;
    if (slots & FFTCONV_SPEC_X) p->ready &= ~kReadyDW;
    if (slots & FFTCONV_SPEC_W) p->ready &= ~kReadyDX;
}

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
        case FFTCONV_SPEC_G2: off = p->off_g2; break;
        default: off = p->off_out; break;
    }
    return reinterpret_cast<cf *>(static_cast<unsigned char *>(ws) + off);
}

bool tiled(fftconv_plan_t p) { return p->Ly > 0; }

int launch_forward(fftconv_plan_t p, int slot, const float *src, void *ws, hipStream_t stream)
{
    long M;
    int ext_y, ext_x, stage;
    Tiling t{};
    const fftconv_desc2d &d = p->d;
    switch (slot) {
        case FFTCONV_SPEC_X:   // dense N x N windows of x, one per output tile
            M = p->maps_x; ext_y = tiled(p) ? p->N : d.nh; ext_x = tiled(p) ? p->N : d.nw; stage = FFTCONV_STAGE_FFT_X;
            t = Tiling{d.nh, d.nw, d.f, p->ntx, p->nty * p->ntx, p->Ly, p->Lx, 0, 0, p->overlap_add ? 1 : 0};
            break;
        case FFTCONV_SPEC_W:   // kernels are never tiled
            M = p->maps_w; ext_y = d.kh; ext_x = d.kw; stage = FFTCONV_STAGE_FFT_W;
            break;
        case FFTCONV_SPEC_G:   // Ly x Lx blocks of dL/dy
            M = p->maps_g; ext_y = tiled(p) ? p->Ly : p->noh; ext_x = tiled(p) ? p->Lx : p->now; stage = FFTCONV_STAGE_FFT_G;
            t = Tiling{p->noh, p->now, d.fo, p->ntx, p->nty * p->ntx, p->Ly, p->Lx, 0, 0, p->overlap_add ? 1 : 0};
            break;
        case FFTCONV_SPEC_G2:  // N x N windows of dL/dy starting (kh-1, kw-1) before each tile of dx
            if (!tiled(p) || p->overlap_add) return FFTCONV_EINVAL;
            M = p->maps_g2; ext_y = ext_x = p->N; stage = FFTCONV_STAGE_FFT_G;
            t = Tiling{p->noh, p->now, d.fo, p->ntx2, p->nty2 * p->ntx2, p->Ly, p->Lx, -(d.kh - 1), -(d.kw - 1), 0};
            break;
        default: return FFTCONV_EINVAL;
    }
    const bool use_tiles = tiled(p) && slot != FFTCONV_SPEC_W;
    FftEntry entry, *e = &entry;
    if (!find_fft(p->N, use_tiles ? p->N : (ext_y > ext_x ? ext_y : ext_x), use_tiles || p->sw.no_small_batch ? 0 : M, entry) ||
        (use_tiles && !e->fwd_tiled))
        return FFTCONV_EUNSUPPORTED;
    FwdKernel kernel = use_tiles ? e->fwd_tiled : e->fwd;
    if (int rc = allow_lds(p, kernel, e->lds_bytes)) return rc;
    FwdArgs a{src, slot_ptr(p, ws, slot), (int)M, ext_y, ext_x, t};
    // true convolution = correlation with the kernels rotated by 180 degrees: rotate them on the way in
    a.flip = (slot == FFTCONV_SPEC_W && (p->d.flags & FFTCONV_TRUE_CONV)) ? 1 : 0;
    const unsigned blocks = (unsigned)((M + e->T - 1) / e->T);
    StageTimer timer(p, stage, stream);
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(e->threads), e->lds_bytes, stream, a);
    if (int rc = check_launch()) return rc;
    if (int rc = timer.finish()) return rc;
    p->valid |= (unsigned)slot;
    operands_changed(p, (unsigned)slot);
    // in the three-slot workspace the blocks and the windows of dL/dy share one slot
    if (recompute_mode(p) && slot == FFTCONV_SPEC_G) p->valid &= ~(unsigned)FFTCONV_SPEC_G2;
    if (recompute_mode(p) && slot == FFTCONV_SPEC_G2) p->valid &= ~(unsigned)FFTCONV_SPEC_G;
    return FFTCONV_OK;
}

void pass_dims(fftconv_plan_t p, int pass, int &Md, int &Nd, int &Kd, int &slot_a, int &slot_b)
{
    // the tiles of a sample act as extra samples: S * nty * ntx (fprop, accGrad) or S * nty2 * ntx2 (bprop)
    const int St = p->d.S * p->nty * p->ntx, St2 = p->d.S * p->nty2 * p->ntx2;
    switch (pass) {
        case FFTCONV_FPROP: Md = St; Nd = p->d.fo; Kd = p->d.f; slot_a = FFTCONV_SPEC_X; slot_b = FFTCONV_SPEC_W; break;
        case FFTCONV_BPROP:
            Md = St2; Nd = p->d.f; Kd = p->d.fo;
            slot_a = tiled(p) && !p->overlap_add ? FFTCONV_SPEC_G2 : FFTCONV_SPEC_G;
            slot_b = FFTCONV_SPEC_W;
            break;
        default:            Md = p->d.fo; Nd = p->d.f; Kd = St; slot_a = FFTCONV_SPEC_G; slot_b = FFTCONV_SPEC_X; break;
    }
}

// accGrad and bprop of a layer with at most four input maps: streaming kernels on the vector
// ALU instead of matrix-core tiles that would be nine tenths padding.
int launch_skinny(fftconv_plan_t p, int pass, void *ws, hipStream_t stream)
{
    SkinnyArgs a{};
    const int sc = result_slot(p, pass);
    a.C = slot_ptr(p, ws, sc);
    a.N = p->d.fo;
    a.bins = p->B;
    if (pass == FFTCONV_ACCGRAD) {
        a.X = slot_ptr(p, ws, FFTCONV_SPEC_X);
        a.G = slot_ptr(p, ws, FFTCONV_SPEC_G);
        a.M = p->d.S * p->nty * p->ntx;
        a.jblocks = (p->d.fo + 63) / 64;
    } else {
        a.X = slot_ptr(p, ws, FFTCONV_SPEC_W);
        a.G = slot_ptr(p, ws, tiled(p) && !p->overlap_add ? FFTCONV_SPEC_G2 : FFTCONV_SPEC_G);
        a.M = p->d.S * p->nty2 * p->ntx2;
        a.jblocks = (a.M + 63) / 64;
    }
    const long blocks = (long)a.bins * a.jblocks;
    if (blocks <= 0 || blocks > 0x7fffffffL) return FFTCONV_EUNSUPPORTED;
    SkinnyKernel kernel = pass == FFTCONV_ACCGRAD ? skinny_accgrad(p->d.f) : skinny_bprop(p->d.f);
    StageTimer timer(p, FFTCONV_STAGE_CGEMM_FPROP + pass, stream);
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kSkinnyThreads), 0, stream, a);
    if (int rc = check_launch()) return rc;
    if (sc != FFTCONV_SPEC_OUT) p->valid &= ~(unsigned)sc;   // an operand slot now holds the result spectrum
    else p->ready = 0;                                       // whatever waited in the OUT slot is overwritten
    return timer.finish();
}

bool shared_pass(fftconv_plan_t p)
{
    return p->shared_pass_ok && !p->sw.no_shared_pass && (p->d.f > 4 || !p->sw.no_skinny);
}

// Both result spectra of bprop and accGrad from one pass over the spectrum of dL/dy; timed as
// the contraction of the pass that asked for it.
void fill_gemm_args(fftconv_plan_t p, int pass, const GemmEntry &e, void *ws, cf *C, GemmArgs &g)
{
    int Md, Nd, Kd, sa, sb;
    pass_dims(p, pass, Md, Nd, Kd, sa, sb);
    g.A = slot_ptr(p, ws, sa);
    g.B = slot_ptr(p, ws, sb);
    g.C = C;
    g.Md = Md; g.Nd = Nd; g.Kd = Kd;
    g.bins = p->B;
    g.tiles_m = (Md + e.MT - 1) / e.MT;
    g.tiles_n = (Nd + e.NT - 1) / e.NT;
    g.xcd_remap = p->sw.no_xcd_remap ? 0 : 1;
    const long lim = 1L << 28;   // complex elements in 2 GB
    g.full_tiles_ok = ((long)Md * Kd < lim && (long)Nd * Kd < lim && (long)Md * Nd < lim && !p->sw.no_full_tiles) ? 1 : 0;
}

// The same for layers with more than four input maps: the matrix-core contractions of both passes in
// one launch (bin_cgemm_bprop_accgrad_kernel).
int launch_pair_contract(fftconv_plan_t p, int pass, void *ws, hipStream_t stream)
{
    const GemmEntry &e = gemm_kernel_table()[p->pair_tile];
    unsigned char *out = reinterpret_cast<unsigned char *>(slot_ptr(p, ws, FFTCONV_SPEC_OUT));
    GemmPairArgs a;
    fill_gemm_args(p, FFTCONV_BPROP, e, ws, reinterpret_cast<cf *>(out), a.bprop);
    fill_gemm_args(p, FFTCONV_ACCGRAD, e, ws, reinterpret_cast<cf *>(out + p->off_shared_dw), a.accgrad);
    const long blocks = (long)p->B * ((long)a.bprop.tiles_m * a.bprop.tiles_n + (long)a.accgrad.tiles_m * a.accgrad.tiles_n);
    if (blocks <= 0 || blocks > 0x7fffffffL) return FFTCONV_EUNSUPPORTED;
    if (int rc = allow_lds(p, e.bprop_accgrad, e.lds_bytes)) return rc;
    StageTimer timer(p, FFTCONV_STAGE_CGEMM_FPROP + pass, stream);
    hipLaunchKernelGGL(e.bprop_accgrad, dim3((unsigned)blocks), dim3(e.threads), e.lds_bytes, stream, a);
    if (int rc = check_launch()) return rc;
    return timer.finish();
}

int launch_shared_pass(fftconv_plan_t p, int pass, void *ws, hipStream_t stream)
{
    const unsigned need = FFTCONV_SPEC_X | FFTCONV_SPEC_W | FFTCONV_SPEC_G;
    if ((p->valid & need) != need) return FFTCONV_ENOTREADY;
    if (p->d.f > 4) return launch_pair_contract(p, pass, ws, stream);
    SharedPassArgs a{};
    unsigned char *out = reinterpret_cast<unsigned char *>(slot_ptr(p, ws, FFTCONV_SPEC_OUT));
    a.G = slot_ptr(p, ws, FFTCONV_SPEC_G);
    a.X = slot_ptr(p, ws, FFTCONV_SPEC_X);
    a.W = slot_ptr(p, ws, FFTCONV_SPEC_W);
    a.DX = reinterpret_cast<cf *>(out);
    a.DW = reinterpret_cast<cf *>(out + p->off_shared_dw);
    a.DWpart = reinterpret_cast<cf *>(out + p->off_shared_part);
    a.M = p->d.S * p->nty * p->ntx;   // the tiles of a sample are extra samples
    a.N = p->d.fo;
    a.bins = p->B;
    a.row_groups = p->shared_row_groups;
    const int F = p->d.f;
    const int rows = a.M < kSharedPassMaxRows ? a.M : kSharedPassMaxRows;
    const int lds_bytes = (64 * 65 + 2 * 64 * F + kSkinnyWaves * ((rows + 63) / 64) * 64 * F) * 8;
    const long blocks = (long)a.bins * a.row_groups;
    if (blocks > 0x7fffffffL) return FFTCONV_EUNSUPPORTED;
    SharedPassKernel kernel = skinny_bprop_accgrad(F);
    if (int rc = allow_lds(p, kernel, lds_bytes)) return rc;
    StageTimer timer(p, FFTCONV_STAGE_CGEMM_FPROP + pass, stream);
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kSkinnyThreads), lds_bytes, stream, a);
    if (int rc = check_launch()) return rc;
    if (a.row_groups > 1) {
        hipLaunchKernelGGL(sum_row_groups(), dim3(512), dim3(256), 0, stream, a.DWpart, a.DW,
                           (size_t)a.bins * a.N * F, a.row_groups);
        if (int rc = check_launch()) return rc;
    }
    return timer.finish();
}

int launch_contract(fftconv_plan_t p, int pass, void *ws, hipStream_t stream)
{
    int Md, Nd, Kd, sa, sb;
    pass_dims(p, pass, Md, Nd, Kd, sa, sb);
    if ((p->valid & (unsigned)sa) == 0 || (p->valid & (unsigned)sb) == 0) return FFTCONV_ENOTREADY;
    if (p->d.f <= 4 && pass != FFTCONV_FPROP && !p->sw.no_skinny) return launch_skinny(p, pass, ws, stream);
    const GemmEntry &e = gemm_kernel_table()[p->gemm_tile[pass]];
    GemmArgs g;
    const int sc = result_slot(p, pass);
    fill_gemm_args(p, pass, e, ws, slot_ptr(p, ws, sc), g);
    const long blocks = (long)g.bins * g.tiles_m * g.tiles_n;
    if (blocks <= 0 || blocks > 0x7fffffffL) return FFTCONV_EUNSUPPORTED;
    if (int rc = allow_lds(p, e.pass[pass], e.lds_bytes)) return rc;
    StageTimer timer(p, FFTCONV_STAGE_CGEMM_FPROP + pass, stream);
    hipLaunchKernelGGL(e.pass[pass], dim3((unsigned)blocks), dim3(e.threads), e.lds_bytes, stream, g);
    if (int rc = check_launch()) return rc;
    if (sc != FFTCONV_SPEC_OUT) {   // an operand slot now holds a result spectrum
        p->valid &= ~(unsigned)sc;
        if (sc == FFTCONV_SPEC_G) p->valid &= ~(unsigned)FFTCONV_SPEC_G2;   // same place in the three-slot workspace
    } else {
        p->ready = 0;               // whatever waited in the OUT slot is overwritten
    }
    return timer.finish();
}

int launch_inverse(fftconv_plan_t p, int pass, float *dst, void *ws, hipStream_t stream, int accumulate, bool fused = false,
                   size_t spec_offset = 0)
{
    long M;
    InvArgs a{};
    const fftconv_desc2d &d = p->d;
    switch (pass) {
        case FFTCONV_FPROP:   // tiles of y: output rows [0, Ly) and columns [0, Lx) of each transform
            M = p->maps_g; a.crop_y = tiled(p) ? p->Ly : p->noh; a.crop_x = tiled(p) ? p->Lx : p->now;
            a.t = Tiling{p->noh, p->now, d.fo, p->ntx, p->nty * p->ntx, p->Ly, p->Lx, 0, 0, p->overlap_add ? 1 : 0};
            break;
        case FFTCONV_BPROP:   // tiles of dx: rows [kh-1, N), columns [kw-1, N), the part of the circular result free of wrap-around
            M = tiled(p) ? (long)d.S * p->nty2 * p->ntx2 * d.f : p->maps_x;
            a.crop_y = tiled(p) ? p->Ly : d.nh; a.crop_x = tiled(p) ? p->Lx : d.nw;
            a.t = Tiling{d.nh, d.nw, d.f, p->ntx2, p->nty2 * p->ntx2, p->Ly, p->Lx, 0, 0, p->overlap_add ? 1 : 0};
            a.c0_y = d.kh - 1; a.c0_x = d.kw - 1;
            if (p->overlap_add) {   // the whole N x N output of a block's transform, placed at the block's origin
                a.crop_y = a.crop_x = p->N;
                a.c0_y = a.c0_x = 0;
                a.add = 1;
            }
            break;
        default:              // dw is never tiled
            M = p->maps_w; a.crop_y = d.kh; a.crop_x = d.kw;
            break;
    }
    const bool use_tiles = tiled(p) && pass != FFTCONV_ACCGRAD;
    FftEntry entry, *e = &entry;
    if (!find_fft(p->N, use_tiles ? p->N : (a.crop_y > a.crop_x ? a.crop_y : a.crop_x),
                  use_tiles || fused || p->sw.no_small_batch ? 0 : M, entry) ||
        (use_tiles && !e->inv_tiled))
        return FFTCONV_EUNSUPPORTED;
    // the tiled kernels either write every window once or assemble dx from overlapping windows:
    // neither adds to what the caller's tensor held
    if (use_tiles && accumulate) return FFTCONV_EUNSUPPORTED;
    InvKernel kernel = use_tiles ? (a.add ? e->inv_tiled_add : e->inv_tiled) : (accumulate ? e->inv_acc : e->inv);
    if (fused) {
        kernel = fused_inverse_kernel(e->N, e->T, e->NX, d.f, use_tiles);
        if (!kernel) return FFTCONV_EUNSUPPORTED;
        a.xs = slot_ptr(p, ws, FFTCONV_SPEC_X);
        a.wsp = slot_ptr(p, ws, FFTCONV_SPEC_W);
        a.fo = d.fo; a.Mx = (int)p->maps_x; a.Mw = (int)p->maps_w;
        a.groups_per_sample = p->sw.no_fused_order ? 0 : d.fo / e->T;
    }
    // on request (it measured slower, see fft_quad_kernels.hpp): small windows (the extent class N / 4) of the
    // sizes from 40 up with every 1-D transform split over four lanes
    if (!use_tiles && !fused && p->sw.quad && e->NX * 4 == e->N) {
        if (const InvQuadEntry *qe = find_inv_quad_kernels(e->N)) {
            kernel = accumulate ? qe->acc : qe->plain;
            e->T = qe->T;
            e->threads = qe->threads;
            e->lds_bytes = qe->lds_bytes;
        }
    }
    if (int rc = allow_lds(p, kernel, e->lds_bytes)) return rc;
    a.spec = reinterpret_cast<const cf *>(reinterpret_cast<const unsigned char *>(slot_ptr(p, ws, result_slot(p, pass))) +
                                          spec_offset);
    a.dst = dst;
    a.M = (int)M;
    // ... and rotate their gradient on the way out
    a.flip = (pass == FFTCONV_ACCGRAD && (p->d.flags & FFTCONV_TRUE_CONV)) ? 1 : 0;
    a.scale = 1.0f / ((float)p->N * (float)p->N);
    const unsigned blocks = (unsigned)((M + e->T - 1) / e->T);
    StageTimer timer(p, FFTCONV_STAGE_IFFT_Y + pass, stream);
    a.parity = -1;
    a.bin_stride = (int)M;
    if (a.add) {
        // overlap-add: one launch per parity class of tiles (the windows of one class are disjoint), in class
        // order; the first class covering a pixel stores, the later ones add, so dx is never cleared
        for (int parity = 0; parity < 4; ++parity) {
            const int cy = (p->nty2 - parity / 2 + 1) / 2, cx = (p->ntx2 - parity % 2 + 1) / 2;   // tiles of this class per axis
            if (cy < 1 || cx < 1) continue;
            a.parity = parity;
            a.cls_cx = cx;
            a.cls_tiles = cy * cx;
            a.M = d.S * a.cls_tiles * d.f;
            const unsigned class_blocks = (unsigned)((a.M + e->T - 1) / e->T);
            hipLaunchKernelGGL(kernel, dim3(class_blocks), dim3(e->threads), e->lds_bytes, stream, a);
            if (int rc = check_launch()) return rc;
        }
        return timer.finish();
    }
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(e->threads), e->lds_bytes, stream, a);
    if (int rc = check_launch()) return rc;
    return timer.finish();
}

}  // namespace

namespace fftconv {
InvKernel fused_inverse_kernel_f1(int N, int T, int NX, bool tiled);
InvKernel fused_inverse_kernel_f2(int N, int T, int NX, bool tiled);
InvKernel fused_inverse_kernel_f3(int N, int T, int NX, bool tiled);
InvKernel fused_inverse_kernel_f4(int N, int T, int NX, bool tiled);

InvKernel fused_inverse_kernel(int N, int T, int NX, int F, bool tiled)
{
    switch (F) {
        case 1: return fused_inverse_kernel_f1(N, T, NX, tiled);
        case 2: return fused_inverse_kernel_f2(N, T, NX, tiled);
        case 3: return fused_inverse_kernel_f3(N, T, NX, tiled);
        case 4: return fused_inverse_kernel_f4(N, T, NX, tiled);
        default: return nullptr;
    }
}
}  // namespace fftconv

namespace {

// fprop of a layer with at most four input maps: the products are formed inside the inverse
// transform (nullptr: not applicable, or no such kernel for this geometry).
InvKernel fused_fprop_kernel(fftconv_plan_t p, int pass, int accumulate)
{
    if (pass != FFTCONV_FPROP || accumulate || p->d.f > kMaxFusedMaps || p->sw.no_fused) return nullptr;
    const bool use_tiles = tiled(p);
    const int crop_y = use_tiles ? p->Ly : p->noh, crop_x = use_tiles ? p->Lx : p->now;
    FftEntry entry, *e = &entry;
    // the maps of a workgroup must share a sample, whose part of the x spectrum must fit the LDS buffer
    if (!find_fft(p->N, use_tiles ? p->N : (crop_y > crop_x ? crop_y : crop_x), 0, entry) || p->d.fo % e->T != 0 || (long)p->B * p->d.f * 8 > e->lds_bytes) return nullptr;
    return fused_inverse_kernel(e->N, e->T, e->NX, p->d.f, use_tiles);
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
    const bool fused = fused_fprop_kernel(p, pass, accumulate) != nullptr;
    size_t spec_offset = 0;
    if (pass != FFTCONV_FPROP && shared_pass(p)) {
        // bprop and accGrad share one pass over the spectrum of dL/dy when all three spectra are at hand
        const unsigned mine = pass == FFTCONV_BPROP ? kReadyDX : kReadyDW, other = mine ^ (kReadyDX | kReadyDW);
        const unsigned third = pass == FFTCONV_BPROP ? FFTCONV_SPEC_X : FFTCONV_SPEC_W;   // read by the other pass only
        bool from_shared = true;
        if (p->ready & mine) {
            p->ready &= ~mine;                     // formed by the other pass: use it once
        } else if (p->valid & third) {
            if (int rc = launch_shared_pass(p, pass, ws, s)) return rc;
            p->ready = other;
        } else {
            if (int rc = launch_contract(p, pass, ws, s)) return rc;
            from_shared = false;
        }
        if (from_shared && pass == FFTCONV_ACCGRAD) spec_offset = p->off_shared_dw;
    } else if (!fused) {
        if (int rc = launch_contract(p, pass, ws, s)) return rc;
    }
    const int rc = launch_inverse(p, pass, dst, ws, s, accumulate, fused, spec_offset);
    if (recompute_mode(p)) p->valid = 0;
    return rc;
}

}  // namespace

extern "C" {

int fftconv_plan(fftconv_plan_t *out, const fftconv_desc *d)
{
    if (!out || !d) return FFTCONV_EINVAL;
    const fftconv_desc2d d2{d->S, d->f, d->fo, d->n, d->n, d->k, d->k, d->flags};
    return fftconv_plan2d(out, &d2);
}

int fftconv_plan2d(fftconv_plan_t *out, const fftconv_desc2d *d)
{
    if (!out || !d) return FFTCONV_EINVAL;
    if (d->S < 1 || d->f < 1 || d->fo < 1 || d->nh < 1 || d->nw < 1 || d->kh < 1 || d->kw < 1 || d->kh > d->nh ||
        d->kw > d->nw)
        return FFTCONV_EINVAL;
    if ((d->flags & ~(unsigned)(FFTCONV_RECOMPUTE | FFTCONV_TRUE_CONV)) != 0) return FFTCONV_EUNSUPPORTED;
    const int noh = d->nh - d->kh + 1, now = d->nw - d->kw + 1;
    int N = fft_size_for(d->nh > d->nw ? d->nh : d->nw), Ly = 0, Lx = 0, nty = 1, ntx = 1, nty2 = 1, ntx2 = 1;
    // Overlap-add for bprop of a tiled layer when a second transform of dL/dy (f' maps per tile) costs more
    // than clearing dx and reading and writing its larger windows (f maps per tile).  Measured: gains of
    // 21 % of the step for S = 128, f = 3, f' = 96, of 2 and 7 % for f = 96, f' = 256 (n = 96, 128), of 7 %
    // for f = f' = 64.
    const char *ratio_env = std::getenv("FFTCONV_OVERLAP_ADD_RATIO");   // for measurements: overlap-add if f * ratio <= f'
    // (without the spectral cache there is no second transform to save, only fewer blocks than windows to
    //  transform: S = 128, f = 96, f' = 256, n = 96 then loses 8 % of the step, so the bar is higher)
    const long ratio = ratio_env ? std::atol(ratio_env) : ((d->flags & FFTCONV_RECOMPUTE) ? 4 : 1);
    const bool few_input_maps = (long)d->f * ratio <= d->fo && !std::getenv("FFTCONV_NO_OVERLAP_ADD");
    bool overlap_add = false;
    if (N < 0) {
        // Larger than the largest transform: cut into tiles of (N - kh + 1) x (N - kw + 1) outputs
        // (overlap-save).  Pick the tile transform that needs the fewest transformed points over
        // the tiles of y and of dx together.
        static const int sizes[] = {16, 20, 24, 28, 32, 40, 48, 56, 64};
        double best = -1.0, best_filled = 0.0;
        const char *forced = std::getenv("FFTCONV_TILE_SIZE");   // for measurements: only this tile transform
        for (int cand : sizes) {
            const int ly = cand - d->kh + 1, lx = cand - d->kw + 1;
            if (ly < 1 || lx < 1 || (forced && std::atoi(forced) != cand)) continue;
            const long ay = (noh + ly - 1) / ly, ax = (now + lx - 1) / lx;
            long by = (d->nh + ly - 1) / ly, bx = (d->nw + lx - 1) / lx;
            // with overlap-add dx is assembled from the windows of the blocks of dL/dy; the windows of one
            // parity class of tiles must not overlap
            const bool oa = few_input_maps && ly >= d->kh - 1 && lx >= d->kw - 1;
            if (oa) { by = ay; bx = ax; }
            const double cost = (double)(ay * ax + by * bx) * cand * cand;   // transformed points
            // Ties go to the size whose tiles, as rows of the contraction (S * tiles), fill their matrix tiles of 64
            // rows best, then to the larger tile: fewer, longer row segments, so fewer partly written 128-byte
            // lines.  Measured, S = 128, f = 96, f' = 256, n = 96, k = 5: N = 28 and 56 tie on both counts, 5.82 against
            // 5.49 ms per step; S = 32, f = f' = 64, n = 112, k = 3: N = 24 and 40 transform the same points, but 9
            // tiles leave 11 % of the contraction's rows empty where 25 leave 4 %: 0.589 against 0.603 ms.
            const auto fill = [&](long tiles) { const long rows = (long)d->S * tiles; return (double)rows / (double)((rows + 63) / 64 * 64); };
            const double filled = fill(ay * ax) < fill(by * bx) ? fill(ay * ax) : fill(by * bx);
            if (best < 0.0 || cost < best || (cost == best && filled >= best_filled)) {
                best_filled = filled;
                best = cost; N = cand; Ly = ly; Lx = lx; overlap_add = oa;
                nty = (int)ay; ntx = (int)ax; nty2 = (int)by; ntx2 = (int)bx;
            }
        }
        if (N < 0) return FFTCONV_EUNSUPPORTED;   // a kernel side above 64
    }
    const long T = (long)nty * ntx, T2 = (long)nty2 * ntx2;
    const int L = Ly;   // non-zero iff tiled
    const bool lean = (d->flags & FFTCONV_RECOMPUTE) != 0;
    // transforms per slot; in the three-slot workspace the x and g slots also take the results
    // dX and Y and the windows of bprop, whose tile counts can differ
    const long Tmax = T > T2 ? T : T2;
    const long maps_x = (long)d->S * d->f * (lean ? Tmax : T), maps_w = (long)d->fo * d->f;
    const long maps_g = (long)d->S * d->fo * (lean ? Tmax : T),
               maps_g2 = L > 0 && !lean && !overlap_add ? (long)d->S * d->fo * T2 : 0;
    const long out_y = (long)d->S * d->fo * T, out_dx = (long)d->S * d->f * T2;
    const long lim = 0x7fffffffL;
    if (maps_x > lim || maps_w > lim || maps_g > lim || maps_g2 > lim || out_y > lim || out_dx > lim)
        return FFTCONV_EUNSUPPORTED;
    fftconv_plan_s *p = new (std::nothrow) fftconv_plan_s();
    if (!p) return FFTCONV_ENOMEM;
    p->d = *d;
    p->noh = noh;
    p->now = now;
    p->N = N;
    p->B = N * N / 2 + 2;
    p->Ly = Ly;
    p->Lx = Lx;
    p->nty = nty;
    p->ntx = ntx;
    p->nty2 = nty2;
    p->ntx2 = ntx2;
    p->overlap_add = overlap_add;
    p->maps_x = (long)d->S * d->f * T;
    p->maps_w = maps_w;
    p->maps_g = (long)d->S * d->fo * T;
    p->maps_g2 = (long)d->S * d->fo * T2;
    p->maps_out = out_y > out_dx ? (out_y > maps_w ? out_y : maps_w) : (out_dx > maps_w ? out_dx : maps_w);
    // bprop and accGrad of a layer whose two passes read the same transforms of dL/dy (untiled, or tiled with
    // overlap-add) form both of their result spectra in one launch, side by side in the OUT slot: dXh at
    // its start, dWh behind it (256-byte aligned, hence the spare map)
    const bool one_g = !lean && (L == 0 || overlap_add);
    // The joint launch of the matrix-core contractions pays when both result spectra then wait in the 256 MB
    // memory-side cache for their inverse transforms; beyond that the second transform reads a spectrum that
    // has been pushed out meanwhile and loses what the launch gained.  Measured, step with / without it:
    // S = 128, f = f' = 256, n = 16 (102 MB of dXh + dWh) 0.290 / 0.296 ms; f = 256, f' = 384, n = 16 (136 MB)
    // 0.397 / 0.402; f = 96, f' = 256, n = 32 (151 MB) 0.493 / 0.497; f = f' = 256, n = 32 (540 MB) 0.993 / 0.984.
    const bool pair_fits_cache = (double)(out_dx + maps_w) * 8.0 * (N * N / 2 + 2) <= 192.0 * 1024 * 1024;
    const bool pair_ok = one_g && d->f > 4 && pair_fits_cache;
    if (pair_ok && out_dx + maps_w + 1 <= lim && p->maps_out < out_dx + maps_w + 1) p->maps_out = out_dx + maps_w + 1;
    const size_t per_map = (size_t)8 * p->B;
    p->off_x = 0;
    p->off_w = p->off_x + align_up(per_map * maps_x);
    p->off_g = p->off_w + align_up(per_map * maps_w);
    p->off_g2 = p->off_g + align_up(per_map * maps_g);
    p->off_out = p->off_g2 + align_up(per_map * maps_g2);
    p->ws_bytes = p->off_out + align_up(per_map * p->maps_out);
    if (lean) {   // three slots only: a pass writes its result into the one it does not read
        p->ws_bytes = p->off_g2;
        p->off_g2 = p->off_g;   // the windows of bprop take the place of the blocks of dL/dy
        p->off_out = (size_t)-1;
        p->maps_out = -1;
    }
    p->valid = 0;
    p->ready = 0;
    // one pass over the spectrum of dL/dy for bprop and accGrad: few input maps, spectra cached, both passes
    // on the same transforms of dL/dy (untiled, or tiled with overlap-add), and dXh, dWh and the partial
    // sums of dWh fit the OUT slot side by side
    {
        const size_t rows = (size_t)d->S * T, dw_bytes = align_up((size_t)maps_w * p->B * sizeof(cf));
        p->shared_row_groups = (int)((rows + kSharedPassMaxRows - 1) / kSharedPassMaxRows);
        p->off_shared_dw = align_up(rows * d->f * p->B * sizeof(cf));
        p->off_shared_part = p->off_shared_dw + dw_bytes;
        const size_t need = p->off_shared_part + (p->shared_row_groups > 1 ? (size_t)p->shared_row_groups * dw_bytes : 0);
        const size_t room = p->maps_out > 0 ? (size_t)p->maps_out * p->B * sizeof(cf) : 0;
        p->shared_pass_ok = d->f <= 4 ? (one_g && need <= room) : (pair_ok && p->off_shared_part <= room);
    }
    p->last_ws = nullptr;
    p->profiling = 0;
    p->device = -1;
    p->lds_raised.reserve(32);   // more than the kernels one plan launches: no host allocation at launch time
    p->sw = read_switches();
    for (int pass = 0; pass < 3; ++pass) {
        int Md, Nd, Kd, sa, sb;
        pass_dims(p, pass, Md, Nd, Kd, sa, sb);
        p->gemm_tile[pass] = choose_gemm_tile(Md, Nd, p->sw);
    }
    {   // one tile shape for both products of the joint bprop + accGrad launch: least padded work over the two
        int Mb, Nb, Kb, Ma, Na, Ka, sa, sb;
        pass_dims(p, FFTCONV_BPROP, Mb, Nb, Kb, sa, sb);
        pass_dims(p, FFTCONV_ACCGRAD, Ma, Na, Ka, sa, sb);
        p->pair_tile = 0;
        double best_work = -1.0;
        for (int i = 0; i < gemm_shape_count(); ++i) {
            const GemmEntry &e = gemm_kernel_table()[i];
            const auto padded = [&](int M, int Nn) { return (double)((M + e.MT - 1) / e.MT) * e.MT * ((Nn + e.NT - 1) / e.NT) * e.NT; };
            const double work = padded(Mb, Nb) * Kb + padded(Ma, Na) * Ka;
            if (best_work < 0.0 || work < best_work) { best_work = work; p->pair_tile = i; }
        }
        if (p->sw.gemm_tile >= 0) p->pair_tile = p->sw.gemm_tile;
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
        case FFTCONV_SPEC_G2: return tiled(p) && !p->overlap_add ? p->off_g2 : (size_t)-1;
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
        case FFTCONV_SPEC_G2: return tiled(p) && !p->overlap_add ? p->maps_g2 : -1;
        case FFTCONV_SPEC_OUT: return p->maps_out;
        default: return -1;
    }
}

int fftconv_invalidate(fftconv_plan_t p, unsigned slots)
{
    if (!p || (slots & ~(unsigned)(FFTCONV_SPEC_X | FFTCONV_SPEC_W | FFTCONV_SPEC_G)) != 0) return FFTCONV_EINVAL;
    if (slots & FFTCONV_SPEC_G) slots |= FFTCONV_SPEC_G2;   // both are transforms of dL/dy
    p->valid &= ~slots;
    operands_changed(p, slots);
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

// Address of the current device's copy of `scratch`, looked up once per device.
static int static_scratch_ptr(void **out)
{
    constexpr int kMaxDevices = 64;
    static void *ptrs[kMaxDevices];
    static std::mutex lock;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return FFTCONV_ELAUNCH;
    std::lock_guard<std::mutex> guard(lock);
    if (!ptrs[device]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return FFTCONV_ELAUNCH;
        ptrs[device] = ptr;
    }
    *out = ptrs[device];
    return FFTCONV_OK;
}

int fftconv_pass_static(fftconv_plan_t p, int pass, const float *a, const float *b, float *out, void *stream,
                        int accumulate)
{
    if (!p || pass < FFTCONV_FPROP || pass > FFTCONV_ACCGRAD || !a || !b || !out) return FFTCONV_EINVAL;
    if (accumulate && pass != FFTCONV_ACCGRAD) return FFTCONV_EINVAL;
    if (p->ws_bytes > FFTCONV_STATIC_SCRATCH_BYTES) return FFTCONV_ESCRATCH;
    void *ws = nullptr;
    if (int rc = static_scratch_ptr(&ws)) return rc;
    // The array belongs to every plan and call on this GPU: nothing in it is this plan's cache.
    p->last_ws = nullptr;
    const unsigned profiling = p->profiling;
    p->profiling = 0;   // event brackets would create events
    const int rc = run_pass(p, pass, a, b, out, ws, stream, accumulate);
    p->profiling = profiling;
    p->valid = 0;
    p->ready = 0;
    p->last_ws = nullptr;
    return rc;
}

int fftconv_forward_transform(fftconv_plan_t p, int slot, const float *src, void *ws, void *stream)
{
    if (!p || !src) return FFTCONV_EINVAL;
    if (slot != FFTCONV_SPEC_X && slot != FFTCONV_SPEC_W && slot != FFTCONV_SPEC_G && slot != FFTCONV_SPEC_G2)
        return FFTCONV_EINVAL;
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
        case FFTCONV_EUNSUPPORTED: return "unsupported layer (k > 64 with n > 64, too many maps, or unknown flags)";
        case FFTCONV_EWORKSPACE: return "workspace pointer null or not 256-byte aligned";
        case FFTCONV_ELAUNCH: return "HIP launch or event call failed";
        case FFTCONV_ENOTREADY: return "operand spectrum not cached for this workspace";
        case FFTCONV_ENOMEM: return "out of host memory";
        case FFTCONV_ESCRATCH: return "the layer's workspace exceeds the library's static scratch (FFTCONV_STATIC_SCRATCH_BYTES)";
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
    const double tiles = (2.0 * p->nty * p->ntx + (double)p->nty2 * p->ntx2) / 3.0;   // mean over the three passes
    return 6.0 * p->d.S * p->d.f * p->d.fo * p->B * tiles;
}

int fftconv_tiling(fftconv_plan_t p, int tile[2], int tiles_y[2], int tiles_dx[2])
{
    if (!p || !tile || !tiles_y || !tiles_dx) return FFTCONV_EINVAL;
    tile[0] = p->Ly; tile[1] = p->Lx;
    tiles_y[0] = p->nty; tiles_y[1] = p->ntx;
    tiles_dx[0] = p->nty2; tiles_dx[1] = p->ntx2;
    return FFTCONV_OK;
}

}  // extern "C"

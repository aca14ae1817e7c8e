/*
 * fftconv -- the three passes of one convolutional layer computed through FFTs
 * on one MI355X (gfx950), after "Fast Training of Convolutional Networks through
 * FFTs" (Mathieu, Henaff, LeCun; arXiv 1312.5851).
 *
 * Notation (paper Sec. 2.1): S minibatch size, f input maps, fo (= f') output
 * maps, n x n inputs, k x k kernels, no = n - k + 1 (valid output, stride 1).
 * "*" is read as the cross-correlation of neural-network layers (plan flag
 * FFTCONV_TRUE_CONV: as the true convolution).
 *
 * Every pass follows Sec. 2.2: each 2-D map is Fourier-transformed once (zero
 * padded to N x N, N = the smallest of 8, 12, 14, 16, 20, 24, 28, 32, 40, 48, 56, 64 that is >= n;
 * Sec. 4 pads to a power of two, the sizes 3 * 2^m, 5 * 2^m and 7 * 2^m cut its padding waste), the products are
 * accumulated per frequency bin over the summed index, and the result is
 * inverse-transformed and cropped.  The spectra of x, w and dL/dy are kept in a
 * caller-owned workspace and reused by later passes (the option Sec. 2.3 names
 * for avoiding repeated transforms, at the price of memory) until the caller
 * invalidates them.
 *
 * ALL DATA POINTERS ARE DEVICE POINTERS (fp32, contiguous, row-major):
 *   x [S][f ][n ][n ]     w [fo][f][k][k]
 *   y [S][fo][no][no]     g = dL/dy like y,  dx like x,  dw like w
 * The library allocates no device memory and keeps no device pointer beyond a
 * call, except that the cache-valid bits are tied to the workspace address last
 * used (a different address invalidates every slot).  `stream` is a hipStream_t
 * passed as void* (NULL = the default stream).  Calls only enqueue kernels; they
 * never synchronise with the host.  Return values report argument and launch
 * errors; on an argument error nothing is launched.
 *
 * A plan is not thread-safe; use one plan per host thread / stream.  A plan belongs to the
 * GPU that is current at its first launch; when a later call finds another GPU current, the
 * plan starts over there with nothing cached.
 *
 * Environment switches, all read once when a plan is made, for measurements and tests (results
 * are the same up to rounding order): FFTCONV_GEMM_TILE=0..7 forces a tile shape of the contraction kernel;
 * FFTCONV_NO_XCD_REMAP, FFTCONV_NO_FULL_TILES select its plainer block numbering / its guarded
 * loads; FFTCONV_NO_SKINNY sends bprop and accGrad of layers with f <= 4 through the
 * matrix-core kernel instead of the streaming ones, FFTCONV_NO_SHARED_PASS keeps their two
 * products in separate launches instead of one pass over the spectrum of dL/dy; FFTCONV_NO_FUSED makes fprop of such
 * layers store and re-read the product spectrum instead of forming it inside the inverse
 * transform (which needs fo to be a multiple of the 16 to 64 maps a workgroup transforms),
 * FFTCONV_NO_FUSED_ORDER keeps that kernel's plain block order; FFTCONV_QUAD makes the inverse transform of
 * dL/dw for kernels of at most N/4 x N/4 on transforms of 40 points and up split every 1-D transform over four
 * lanes with cross-lane (DPP) sums, a variant that measured slower than the default; FFTCONV_NO_SMALL_BATCH keeps
 * the usual 16 to 64 maps per workgroup of the transform kernels for launches of few maps too (such launches
 * otherwise run with 2 to 16 maps per workgroup, which spreads them over more CUs);
 * FFTCONV_NO_OVERLAP_ADD keeps the second transform of dL/dy for bprop of tiled layers,
 * FFTCONV_TILE_SIZE=N forces the transform size of the tiles, FFTCONV_OVERLAP_ADD_RATIO=r
 * moves the choice of overlap-add to f * r <= fo.
 */
#ifndef FFTCONV_H
#define FFTCONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fftconv_plan_s *fftconv_plan_t;

typedef struct {
    int S, f, fo, n, k;
    unsigned flags; /* bitwise OR of FFTCONV_RECOMPUTE, FFTCONV_TRUE_CONV */
} fftconv_desc;

/* The same layer with a height and a width for maps and kernels (the paper writes square
 * ones only to keep its notation short, Sec. 2.1): x [S][f][nh][nw], w [fo][f][kh][kw],
 * y and dL/dy [S][fo][nh-kh+1][nw-kw+1].  The transform stays square: N covers
 * max(nh, nw). */
typedef struct {
    int S, f, fo, nh, nw, kh, kw;
    unsigned flags; /* bitwise OR of FFTCONV_RECOMPUTE, FFTCONV_TRUE_CONV */
} fftconv_desc2d;

/* Plan flag: the memory-efficient mode all of the paper's own timings assume (Sec. 2.3).
 * No spectrum is reused: every pass transforms both of its operands again, and the
 * workspace shrinks to the three slots x, w, g (8*B*(S*f + fo*f + S*fo) bytes, the
 * count of Sec. 2.3) because a pass writes its result spectrum into the slot it does not
 * read (Y into g's, dX into x's, dW into w's).  One such workspace can serve every layer
 * of a network in turn, sized for the largest.  fftconv_valid_slots is 0 after a pass,
 * and FFTCONV_SPEC_OUT has no offset of its own. */
enum { FFTCONV_RECOMPUTE = 1 };

/* Plan flag: read "*" in Eqs. (1)-(3) as the true convolution, i.e. with the kernel
 * index reversed, y[s,j,p,q] = sum_i sum_ab x[s,i,p+a,q+b] w[j,i,kh-1-a,kw-1-b], instead
 * of the cross-correlation of neural-network layers (the default).  bprop and accGrad
 * stay the adjoints of that fprop.  Costs nothing: the kernels are read, and their
 * gradient is stored, rotated by 180 degrees. */
enum { FFTCONV_TRUE_CONV = 2 };

enum {
    FFTCONV_OK = 0,
    FFTCONV_EINVAL = 1,       /* null pointer, non-positive size, k > n, bad slot/pass */
    FFTCONV_EUNSUPPORTED = 2, /* k > 64 with n > 64, more than 2^31 transforms in a slot, or unknown flag bits */
    FFTCONV_EWORKSPACE = 3,   /* workspace pointer null or not 256-byte aligned */
    FFTCONV_ELAUNCH = 4,      /* the HIP runtime refused a launch or an event call */
    FFTCONV_ENOTREADY = 5,    /* a stage-level call needs a spectrum that is not cached */
    FFTCONV_ENOMEM = 6,       /* host memory for a plan could not be allocated */
    FFTCONV_ESCRATCH = 7      /* fftconv_pass_static: the layer needs more workspace than the static scratch holds */
};

/* Spectral cache slots (bit flags) and the scratch slot holding a pass's result spectrum.
 * FFTCONV_SPEC_G2 exists only for tiled layers (n > 64, see fftconv_tiling) whose bprop
 * transforms windows of dL/dy of its own, which differ from the blocks accGrad transforms. */
enum { FFTCONV_SPEC_X = 1, FFTCONV_SPEC_W = 2, FFTCONV_SPEC_G = 4, FFTCONV_SPEC_OUT = 8, FFTCONV_SPEC_G2 = 16 };

/* Passes: Eq. (1), (2), (3) of Sec. 2.1. */
enum { FFTCONV_FPROP = 0, FFTCONV_BPROP = 1, FFTCONV_ACCGRAD = 2 };

/* Stages timed by the optional profiler, in hot-path order. */
enum {
    FFTCONV_STAGE_FFT_X = 0, FFTCONV_STAGE_FFT_W = 1, FFTCONV_STAGE_FFT_G = 2,
    FFTCONV_STAGE_CGEMM_FPROP = 3, FFTCONV_STAGE_CGEMM_BPROP = 4, FFTCONV_STAGE_CGEMM_ACCGRAD = 5,
    FFTCONV_STAGE_IFFT_Y = 6, FFTCONV_STAGE_IFFT_DX = 7, FFTCONV_STAGE_IFFT_DW = 8,
    FFTCONV_NUM_STAGES = 9
};

/* ---- plan (host only) -------------------------------------------------- */

/* Validates the layer and fixes N, the bin count, the tiling and the workspace layout.
 * Errors: EINVAL for null arguments, sizes < 1 or k > n; EUNSUPPORTED for k > 64 with
 * n > 64, for slots of more than 2^31 transforms, or for unknown flag bits.  *out is
 * written only on success. */
int fftconv_plan(fftconv_plan_t *out, const fftconv_desc *d);
int fftconv_plan2d(fftconv_plan_t *out, const fftconv_desc2d *d);   /* same, rectangular maps / kernels */
int fftconv_plan_destroy(fftconv_plan_t p);

/* Transform size N (2^m, 3 * 2^m, 5 * 2^m or 7 * 2^m, >= n) and number of stored bins B = N*N/2 + 2:
 * the part of the spectrum a real map determines (Sec. 2.3), i.e. every bin that
 * is not the complex conjugate of another stored bin. */
int fftconv_fft_size(fftconv_plan_t p);
int fftconv_num_bins(fftconv_plan_t p);

/* Layers with a map side above 64 are cut into tiles (the paper instead pads the whole map to the next
 * power of two, Sec. 4).  With L = N - k + 1: y and dL/dy are cut into ceil(no / L)^2 blocks
 * of L x L, dx into ceil(n / L)^2.  fprop transforms the N x N window of x under each
 * block of y, multiplies and keeps rows / columns [0, L) of the inverse transform; accGrad
 * multiplies the same windows with the transforms of the zero-padded blocks of dL/dy and
 * sums over samples and tiles; bprop transforms, for each block of dx, the N x N window of
 * dL/dy that starts k - 1 rows and columns before it and keeps rows / columns [k-1, N) of
 * the inverse transform (the part of a circular result that no wrap-around touches).
 * When f <= fo (under FFTCONV_RECOMPUTE: f * 4 <= fo) and L >= k - 1, bprop instead multiplies the blocks of dL/dy that accGrad
 * transforms and adds the whole N x N inverse transform of each at the block's origin into dx
 * (overlap-add, in four launches over tiles whose windows do not overlap): dL/dy is transformed
 * once, there is no FFTCONV_SPEC_G2 slot, and tiles_dx equals tiles_y.  The
 * tiles of a sample act as extra samples for the contraction.  (Rectangular layers: L, the
 * block counts, the window offsets and the kept rows / columns are per axis, with kh and kw.)
 * Each array is (rows, columns): tile = (Ly, Lx), (0, 0) if not tiled; tiles_y and tiles_dx =
 * blocks per axis of y and of dx, (1, 1) if not tiled. */
int fftconv_tiling(fftconv_plan_t p, int tile[2], int tiles_y[2], int tiles_dx[2]);

/* Bytes of device workspace the passes need: the x, w and g spectra (8*B bytes
 * per map for S*f + fo*f + S*fo maps, the count of Sec. 2.3) plus one result
 * slot of 8*B*max(S*fo, S*f, fo*f) bytes (8*B*(S*f + fo*f + 1) if that is more and
 * the layer takes the joint bprop + accGrad launch); each slot 256-byte aligned.
 * With FFTCONV_RECOMPUTE: the three slots only.  Tiled layers hold one transform per
 * tile (fftconv_slot_maps) and, unless bprop uses overlap-add, one more slot, FFTCONV_SPEC_G2. */
size_t fftconv_workspace_bytes(fftconv_plan_t p);

/* Layout of one slot inside the workspace: byte offset and number of maps M.
 * A slot holds spec[c][m] as interleaved (re, im) floats; stored bin c is
 *   (ky = 0, kx = c)                 for c in [0, N/2],
 *   (ky = N/2, kx = c - (N/2+1))     for c in [N/2+1, N+1],
 *   (ky, kx), c = N+2 + (ky-1)*N+kx  for ky in [1, N/2-1], kx in [0, N);
 * m is the map index in the tensor's own order (s*f+i for x, j*f+i for w,
 * s*fo+j for g; tiled layers: (s*tiles+t)*f+i and (s*tiles+t)*fo+j for tile
 * t = ty*tiles_per_row+tx of sample s).  FFTCONV_SPEC_OUT holds the spectrum
 * of the last pass's result at the slot's start, laid out like that result; the
 * one exception is the joint launch for bprop and accGrad (see fftconv_bprop),
 * which leaves dX's spectrum at the start and dW's behind it (256-byte aligned),
 * whichever of the two passes ran.  Returns (size_t)-1 / -1 for a bad slot (and
 * for FFTCONV_SPEC_OUT under FFTCONV_RECOMPUTE). */
size_t fftconv_slot_offset(fftconv_plan_t p, int slot);
long   fftconv_slot_maps(fftconv_plan_t p, int slot);

/* The caller changed the contents of x / w / g: drop their cached spectra
 * (bitwise OR of FFTCONV_SPEC_X/W/G).  This is the only way the library learns
 * that a tensor changed. */
int fftconv_invalidate(fftconv_plan_t p, unsigned slots);
unsigned fftconv_valid_slots(fftconv_plan_t p);

/* ---- the three passes (Sec. 2.1, computed as in Sec. 2.2) --------------- */

/* Eq. (1): y[s,j] = sum_i x[s,i] * w[j,i].  Transforms x and/or w only if their
 * slot is invalid, contracts per bin over i, inverse-transforms and stores the
 * no x no window.  y is overwritten. */
int fftconv_fprop(fftconv_plan_t p, const float *x, const float *w, float *y, void *ws, void *stream);

/* Eq. (2), summed over j: dx[s,i] = sum_j g[s,j] * w[j,i]^T (adjoint of fprop in x).
 * Uses the g and w slots; stores the full n x n window.  dx is overwritten.
 *
 * One launch for the products of bprop and accGrad.  Both read the spectrum of dL/dy.  If the spectra are
 * cached, both passes use the same transforms of dL/dy (untiled layers, or tiled ones whose bprop uses
 * overlap-add) and the slots of x, w and g are all valid, the first of fftconv_bprop / fftconv_accgrad to be
 * called forms the result spectra of both and leaves the other's in FFTCONV_SPEC_OUT; the other pass, called
 * next with the same tensors, only inverse-transforms it.  Layers with f <= 4 do this in one streaming pass
 * over the spectrum of dL/dy; layers with more input maps run both matrix-core contractions in one launch,
 * provided both result spectra together stay below 192 MiB (so that each still sits in the memory-side cache
 * when its inverse transform reads it).  The waiting spectrum is used once, and is dropped when one of its
 * operand slots is invalidated or transformed again or another call writes FFTCONV_SPEC_OUT; results are
 * those of separate calls up to rounding order.
 * FFTCONV_NO_SHARED_PASS in the environment keeps the two products in separate launches. */
int fftconv_bprop(fftconv_plan_t p, const float *g, const float *w, float *dx, void *ws, void *stream);

/* Eq. (3), summed over the minibatch: dw[j,i] = sum_s g[s,j] * x[s,i] (adjoint of
 * fprop in w).  Uses the g and x slots; stores the k x k window.  accumulate = 0
 * overwrites dw, accumulate = 1 adds the gradient to it. */
int fftconv_accgrad(fftconv_plan_t p, const float *g, const float *x, float *dw, void *ws, void *stream,
                    int accumulate);

/* ---- one pass without any allocation ------------------------------------ */

/* For callers that cannot allocate device memory or obtain a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * same pass as fftconv_fprop (pass = FFTCONV_FPROP: a = x, b = w, out = y),
 * fftconv_bprop (FFTCONV_BPROP: a = g, b = w, out = dx) or fftconv_accgrad
 * (FFTCONV_ACCGRAD: a = g, b = x, out = dw; `accumulate` as there, 0 for the other two),
 * run by the same kernels, with the spectral workspace taken from an array of
 * FFTCONV_STATIC_SCRATCH_BYTES that is part of the library's device code: every GPU the
 * library runs on holds one copy of it from the first call there until the process ends.
 * The call allocates nothing, on the device or on the host, and records no events (stage
 * timing is off for its launches).
 *
 * Returns FFTCONV_ESCRATCH, launching nothing, if fftconv_workspace_bytes(p) exceeds
 * FFTCONV_STATIC_SCRATCH_BYTES (plan with FFTCONV_RECOMPUTE to need only three slots).
 * All calls on one GPU, from any plan, share that GPU's array: nothing is cached across
 * calls (both operands are transformed every time, fftconv_valid_slots is 0 afterwards,
 * and the plan's cache bits for a caller-owned workspace are dropped too), the array is
 * left holding the last call's spectra (every call writes all it reads, so nothing needs
 * clearing), and calls that overlap in time on one GPU (two streams, two threads) race on
 * it: serialise them. */
#define FFTCONV_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int fftconv_pass_static(fftconv_plan_t p, int pass, const float *a, const float *b, float *out, void *stream,
                        int accumulate);

/* ---- single stages (same kernels; for stage tests and per-stage timing) - */

/* Forward transform of one tensor into its slot (slot = FFTCONV_SPEC_X, _W, _G, or _G2
 * for a tiled layer that has that slot), unconditionally; marks the slot valid. */
int fftconv_forward_transform(fftconv_plan_t p, int slot, const float *src, void *ws, void *stream);

/* Per-bin contraction of a pass on cached spectra into the OUT slot (under
 * FFTCONV_RECOMPUTE into the slot the pass does not read, which stops being valid).
 * ENOTREADY if an operand slot is not valid for this workspace. */
int fftconv_contract(fftconv_plan_t p, int pass, void *ws, void *stream);

/* Inverse transform + crop of the pass's result spectrum (where fftconv_contract
 * put it) into the pass's result tensor.  accumulate = 1 adds to dst instead of
 * overwriting it; tiled layers (a map side above 64) support that for accGrad only
 * and return EUNSUPPORTED for y and dx, launching nothing. */
int fftconv_inverse_transform(fftconv_plan_t p, int pass, float *dst, void *ws, void *stream, int accumulate);

/* ---- stage timing ------------------------------------------------------- */

/* Launches of the stages selected by `stage_mask` (bit s = stage s of the list above,
 * FFTCONV_PROFILE_ALL = every stage, 0 = none) are bracketed by HIP events on the launch
 * stream (up to 4096 launches between reads; a bracket costs a few microseconds of queue
 * time).  fftconv_profile_read waits for the recorded events, adds each stage's elapsed
 * milliseconds and launch count into the caller's arrays of FFTCONV_NUM_STAGES entries
 * (host memory), and clears the record. */
#define FFTCONV_PROFILE_ALL 0x1ffu
int fftconv_profile_enable(fftconv_plan_t p, unsigned stage_mask);
int fftconv_profile_read(fftconv_plan_t p, double *ms_sum, long *launches);

/* ---- helpers ------------------------------------------------------------ */

const char *fftconv_strerror(int status);

/* The paper's closed form for frequency-domain memory, Sec. 2.3:
 * 4 n (n+1) (S f + S fo + f fo) bytes (it counts n(n+1)/2 complex numbers per
 * map; the workspace query above counts the B = N*N/2 + 2 actually stored). */
size_t fftconv_paper_ram_bytes(int S, int n, int f, int fo);

/* Matrix-core floating-point operations the contraction of one pass issues:
 * 6 * S * f * fo * B (three real multiply-adds per complex product, Karatsuba's
 * form, over the B stored bins), padding of matrix tiles not counted.  For a tiled
 * layer S counts the tiles too, and the value is the mean over the three passes. */
double fftconv_contraction_flops(fftconv_plan_t p);

#ifdef __cplusplus
}
#endif
#endif /* FFTCONV_H */

/*
 * sig.h -- C ABI of libsig: the batched truncated path-signature transform on
 * one AMD MI355X (gfx950), hand-written HIP behind plain pointers and sizes.
 *
 * The operation (paper Section 3.1):
 *   a path is L points in R^d; its K = L - 1 increments are dX_k = X_{k+1} - X_k;
 *   exp^N(v) = (1, v, v(x)v/2!, ..., v^{(x)N}/N!)                         (Eq. 2)
 *   Sig_1 = exp^N(dX_1),  Sig_k = Sig_{k-1} (x) exp^N(dX_k)               (Eq. 3, batched Eq. 5)
 *   (a (x) b)_n = sum_{i+j=n} a_i (x) b_j,  i, j >= 0,  a_0 = b_0 = 1     (Eq. 4)
 *   the output row of a prefix is the concatenation [S_1, ..., S_N]       (Eq. 10)
 * so level 0 (the constant 1) is not stored.  Level n occupies d^n floats
 * starting at offset d + ... + d^{n-1} of a row, flattened row-major with the
 * earliest tensor factor as the slowest index.  A row has
 * D = d + d^2 + ... + d^N floats.
 *
 * Conventions common to all entry points
 *   - every pointer named DEVICE is device memory of the GPU that was current
 *     when the context was created; the caller allocates and frees it and keeps
 *     it alive until the HIP stream has passed the call;
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream), so that this header needs no HIP include.  All work is enqueued
 *     on it and the call returns without synchronising -- with one exception:
 *     a call that needs more context scratch than any earlier call on the
 *     context waits for the device, frees the old buffer and allocates a larger
 *     one (callers that must not allocate or wait size the scratch with one
 *     eager call of the largest shape first, or use sig_compute_noalloc);
 *   - nothing is thrown, printed or aborted across this boundary: every
 *     failure is a return code (enum below) and leaves `out` unspecified;
 *   - a context owns reusable device scratch, so one context serves one stream
 *     at a time; calls on the same stream are ordered by the stream.
 *   - results are deterministic for a fixed plan (no atomics, fixed combine order).
 */
#ifndef SIG_H
#define SIG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sig_ctx sig_ctx; /* opaque: device properties, scratch buffers */

enum sig_status {
    SIG_OK = 0,
    SIG_ERR_INVALID = 1,   /* NULL pointer, B < 0, L < 2, d < 1, depth < 1, flag not 0/1, bad plan */
    SIG_ERR_TOO_LARGE = 2, /* D or an output size overflows int64, or a grid limit is exceeded */
    SIG_ERR_ALLOC = 3,     /* device scratch could not be allocated */
    SIG_ERR_HIP = 4,       /* a HIP call or kernel launch reported an error */
    SIG_ERR_NO_DEVICE = 5, /* no usable HIP device when the context was created */
    SIG_ERR_UNSUPPORTED = 6 /* no kernel is compiled for this (d, depth), or the shape exceeds what it handles */
};

/* Which kernel family runs (see sig_plan). */
enum sig_variant {
    SIG_VARIANT_AUTO = 0,
    /* state of every path lives in HBM (in the output rows themselves) and is read-modified-written
     * once per increment; any (d, depth); the fallback for shapes that neither of the other families takes */
    SIG_VARIANT_HBM_STREAMING = 1,
    /* state lives in registers: each lane owns the words below one prefix of length `prefix_depth`
     * and runs the fused multiply-by-exponential of Eq. 3 over its time chunk; chunks of one path
     * are joined by Eq. 4 products; only for the compiled (d, depth, prefix_depth) combinations */
    SIG_VARIANT_ON_CHIP = 2,
    /* the level-by-level formulation of the paper's Section 3.2 (Eqs. 6-10): one launch per level, each a
     * cumulative sum over time of per-step terms built from the lower levels of every prefix; those live in
     * context scratch of B * (L-1) * (D - d^depth) floats, in both modes (in stream mode the launch of the top level
     * writes whole output rows, the lower levels it has read included); a batch that would need more than 8 GiB is
     * taken in equal slices of paths that share the buffer, one after the other on the caller's stream.
     * d <= 256 (a template parameter up to 10, a run-time value above), depth <= 8.  Built to measure the paper's own design against the fused fold on the same chip (where a
     * fused kernel is compiled, that one is several times faster); sig_plan chooses it for shapes without an on-chip
     * kernel, where its parallelism in time beats the HBM-streaming sweep.  Plan fields used: chunks (time chunks per word and launch, at most 64; 0 = chosen
     * per level) */
    SIG_VARIANT_LEVEL_SCAN = 3
};

/*
 * How one sig_compute call is mapped onto the GPU.  Filled by sig_plan; may be
 * edited and passed to sig_compute_planned (tests and tuning).  Fields:
 *   variant       one of enum sig_variant (never AUTO after sig_plan)
 *   prefix_depth  p: the index space of a row is cut into d^p independent sub-trees
 *   chunks        time chunks of one path folded concurrently inside one workgroup (>= 1)
 *   segments      workgroups per path along time (>= 1); partial signatures of segments are joined by a second
 *                 launch when all rows of a path fit the LDS of a join kernel, else (a power of two of at most 32
 *                 segments) by a pairwise tree of batched Eq. 4 products in device memory, one launch per round
 *   threads       workgroup size (multiple of 64)
 *   tile_steps    increments staged through LDS per tile by the loader (0: chosen by the library)
 *   independent_waves  with chunks == 1: 0 = workgroup-wide tiles of increments (the default, faster in every
 *                 measurement so far); 1 = every wavefront stages its own increments and workgroups walk
 *                 several batches of paths without any barrier (kept for comparison)
 *   stagger_ticks skewed start of the workgroups of a multi-round final-mode launch: 0 = chosen by the
 *                 library, > 0 = delay per residency slot in 100 MHz ticks, < 0 = off
 *   tile_loader   loader of plans with several tiles per chunk: 0 = chosen by the library, 1 = the next tile's
 *                 loads stay in flight in registers while the current tile is consumed, 2 = load, barrier, consume
 *   shared_chain  final mode, one chunk, shapes whose d^prefix_depth lanes per path exceed a workgroup, prefix_depth
 *                 >= 2, (path, segment) pieces short enough for one tile (128 increments for d = 10): a few threads of
 *                 every workgroup evaluate the part of the Horner chains of Eq. 3 that depends on the first
 *                 prefix_depth - 1 letters only, once, and the fold reads it from LDS.  0 = chosen by the library
 *                 (taken for prefix_depth >= 4), 1 = insist (the plan is invalid where the kernel does not apply),
 *                 2 = every lane carries and re-evaluates its own prefix chain
 *   reserved      zero
 */
typedef struct sig_plan_t {
    int32_t variant;
    int32_t prefix_depth;
    int32_t chunks;
    int32_t segments;
    int32_t threads;
    int32_t tile_steps;
    int32_t independent_waves;
    int32_t stagger_ticks;
    int32_t tile_loader;
    int32_t shared_chain;
    int32_t reserved[2];
} sig_plan_t;

/*
 * D = d + d^2 + ... + d^depth (row length of Eq. 10), or -1 if d < 1, depth < 1
 * or the sum does not fit in int64.  Host only.
 */
int64_t sig_size(int d, int depth);

/*
 * Create a context on the current HIP device.  *ctx receives the handle.
 * Returns SIG_ERR_INVALID for ctx == NULL, SIG_ERR_NO_DEVICE when HIP reports
 * no device.  Allocates nothing on the device until the first compute call
 * that needs scratch.
 */
int sig_create(sig_ctx **ctx);

/* Synchronise the device, free the context's scratch and the context.  NULL is a no-op. */
void sig_destroy(sig_ctx *ctx);

/*
 * Signatures of a batch of piecewise-linear paths (Eqs. 2-5, output Eq. 10).
 *   path         DEVICE, float32 [B][L][d], contiguous, read only
 *   B, L, d      batch, points per path (>= 2), channels (>= 1)
 *   depth        truncation level N (>= 1)
 *   stream_flag  0: out is [B][D], the signature of the whole path
 *                1: out is [B][L-1][D]; row k is the signature of points 0..k+1
 *   out          DEVICE, float32, fully overwritten; must not overlap path
 *   hip_stream   hipStream_t as void*
 * B == 0 returns SIG_OK and launches nothing.  L == 1 has no increment and is
 * SIG_ERR_INVALID.  NaN/Inf propagate.  Arithmetic is float32 with FMA.
 */
int sig_compute(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth,
                int stream_flag, float *out, void *hip_stream);

/*
 * sig_compute for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same mapping, same kernels and the same results
 * as sig_compute, but the scratch that some mappings need (partial signatures of time segments that a second
 * launch joins; the lower-level tensors of the level-scan family) is a fixed array of
 * SIG_NOALLOC_SCRATCH_BYTES that is part of the library's code object: every GPU the library runs on holds
 * it from the library's first use until the process ends.  The call allocates and frees nothing and never
 * waits for the device.  A shape whose mapping needs more scratch than that is refused with
 * SIG_ERR_TOO_LARGE and nothing is launched (sig_compute takes such shapes).  All contexts of one GPU share
 * the array: calls that overlap in time on one GPU (different streams, different contexts) race on it;
 * calls ordered by one stream do not.  Nothing in it has to start at zero: every call writes what it reads.
 */
#define SIG_NOALLOC_SCRATCH_BYTES (16 * 1024 * 1024)
int sig_compute_noalloc(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth,
                        int stream_flag, float *out, void *hip_stream);

/*
 * The mapping sig_compute would use for this shape (one remembered by sig_autotune for exactly this shape, else the
 * planner's).  Host only; `ctx` may be NULL (then a 256-CU device is assumed).  Returns SIG_ERR_INVALID /
 * SIG_ERR_TOO_LARGE exactly as sig_compute would for the same shape.
 */
int sig_plan(const sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag,
             sig_plan_t *plan);

/*
 * Optional tuning of the mapping of one shape (the shape grid of the paper's tables, Section 4.1, is where it
 * pays: few paths, where launch and latency effects decide).  Times candidate mappings on the device -- the
 * planner's choice, the level-scan family, the compiled register kernels with neighbouring time cuts, then the
 * fastest of these with smaller workgroups (192, 128, 64 threads) -- on synthetic input of this shape and remembers the fastest in the context: later sig_compute and sig_plan calls
 * with exactly this (B, L, d, depth, stream_flag) use it (64 shapes per context, the oldest is replaced).
 *   chosen, microseconds   HOST, may be NULL: the mapping taken and its measured time per call
 * Unlike the other entry points it allocates temporary device buffers of the input and output size, enqueues a few
 * dozen calls on `hip_stream` and waits for them.  B == 0 is SIG_ERR_INVALID; SIG_ERR_ALLOC if the buffers do not fit.
 */
int sig_autotune(sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag, sig_plan_t *chosen,
                 float *microseconds, void *hip_stream);

/*
 * SIG_OK if sig_compute_planned would accept `plan` for this shape (the same checks, nothing is
 * launched), else the status it would return.  Host only.
 */
int sig_plan_validate(int64_t B, int64_t L, int d, int depth, int stream_flag, const sig_plan_t *plan);

/*
 * What a plan costs on the device, worked out on the host (nothing is launched; a device with 256 compute units is
 * assumed): LDS bytes per workgroup, workgroups of the main launch, and bytes of context scratch the call needs (what
 * sig_compute_noalloc compares with SIG_NOALLOC_SCRATCH_BYTES).  Each pointer may be NULL.  The level-scan family, one
 * launch per level with its own geometry, reports -1 for the first two.  Returns what sig_plan_validate returns.
 */
int sig_plan_footprint(int64_t B, int64_t L, int d, int depth, int stream_flag, const sig_plan_t *plan,
                       int64_t *lds_bytes, int64_t *workgroups, int64_t *scratch_bytes);

/*
 * sig_compute with an explicit mapping.  The plan is validated against the
 * shape and the compiled kernels; an unsupported plan is SIG_ERR_INVALID and
 * nothing is launched.
 */
int sig_compute_planned(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth,
                        int stream_flag, float *out, const sig_plan_t *plan, void *hip_stream);

/*
 * Batched truncated product of Eq. 4 on output rows (level 0 = 1 implied on both sides):
 *   out[b] = a[b] (x) b[b],  a, b, out DEVICE float32 [B][D]; out must not overlap a or b.
 */
int sig_combine(sig_ctx *ctx, const float *a, const float *b, int64_t B, int d, int depth,
                float *out, void *hip_stream);

/*
 * Gradient of a scalar loss with respect to the path.  The signature layer is trained between other
 * layers (paper Section 4.2, Eq. 11), which needs d(loss)/d(path) from d(loss)/d(output); this is the
 * derivative of Eqs. 2-5 (output layout Eq. 10) written out as a reverse sweep over the increments.
 *   path         DEVICE, float32 [B][L][d], the same array sig_compute was given
 *   out          DEVICE, float32, what sig_compute wrote for (path, depth, stream_flag): [B][D] or [B][L-1][D];
 *                read only (the sweep starts from the final signature and undoes one increment at a time)
 *   grad_out     DEVICE, float32, d(loss)/d(out), same shape as out, read only
 *   grad_path    DEVICE, float32 [B][L][d], fully overwritten; must not overlap the inputs
 * Same conventions and status codes as sig_compute (B == 0 returns SIG_OK and launches nothing).  Shapes with a
 * compiled register kernel (see sig_backward_available) whose paths fit its LDS staging take it.
 * Few long paths (fewer workgroups than compute units, from 128 increments on; from 512, and mostly up to 32
 * paths, for shapes with at most 32 lanes per path) and paths too long for that staging are cut into up to 32
 * time segments that are swept by different workgroups: by Eq. 3 a segment can start from the signature of the
 * path up to its end and the gradient with respect to it, which a scan over the segments' own signatures provides.
 * Stream mode is cut the same way at smaller batches (two sweeps per segment and a scan over the segments between
 * them; the upstream gradient is read twice); paths too long for the staging in a batch that fills the chip, or too
 * long even for 32 segments, are walked in tiles of 256 increments by one workgroup; so are, in a batch that fills
 * the chip, paths that fit the staging only a few at a time (kernels with 16 lanes per path or more; those with fewer
 * are cut in time inside the workgroup there, as for few paths, unless the plain sweep still keeps enough lanes busy).
 * Which sweep a call takes never changes its result beyond the rounding order.  Every shape
 * without a register kernel, d <= 256, takes a general sweep, one workgroup per path with its state in LDS or
 * device scratch (much slower); SIG_ERR_UNSUPPORTED only for d > 256.
 * Context scratch (allocated on first use, SIG_ERR_ALLOC if that fails): shapes whose index space is cut into more
 * sub-trees than one workgroup has threads, and paths walked in tiles, keep per-workgroup sums
 * (B * ceil(d^p / 256) * (L-1) * d floats); the
 * sweep cut into W segments keeps those sums and 5 * B * W * D floats of segment rows; the general sweep keeps
 * B * (L-1) * d floats plus, when they exceed 48 KB per path, about 2.5 D floats per path.
 * Deterministic (fixed summation order).  Arithmetic is float32 with FMA.
 */
int sig_backward(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth, int stream_flag,
                 const float *out, const float *grad_out, float *grad_path, void *hip_stream);

/* 1 if sig_backward has a compiled register kernel for (d, depth), 0 if it would take the general sweep.  Host only. */
int sig_backward_available(int d, int depth);

/*
 * How sig_backward would sweep this shape.  Host only; ctx may be NULL (a device with 256 compute units is assumed).
 * Returns the number of time segments the sweep is cut into across workgroups (2 .. 32), 1 for the uncut register
 * sweep, 0 for the general sweep, or minus the SIG_ERR_* status with which sig_backward would reject the arguments.
 */
int sig_backward_segments(const sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag);

/* 1 if an on-chip kernel is compiled for (d, depth, prefix_depth), else 0.  Host only. */
int sig_on_chip_available(int d, int depth, int prefix_depth);

/* Static, NUL-terminated description of a status code. */
const char *sig_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SIG_H */

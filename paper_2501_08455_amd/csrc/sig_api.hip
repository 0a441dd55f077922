// Host side of libsig: argument checking, the planner that maps a shape onto the GPU, scratch
// management and kernel dispatch.  The C ABI is declared and documented in include/sig.h.
#include <cmath>
#include <new>

#include "sig_internal.h"

using namespace sig;

// a mapping measured by sig_autotune for one shape
struct TunedPlan {
    int64_t B, L;
    int d, depth, stream_flag;
    sig_plan_t plan;
};

struct sig_ctx {
    int device;
    int num_cu;
    float *scratch;        // partial signatures of time segments, [B][segments][D]
    size_t scratch_bytes;
    float *fixed_scratch;  // this device's copy of the file-scope array below (sig_compute_noalloc)
    TunedPlan tuned[64];   // filled by sig_autotune, consulted by sig_compute and sig_plan (oldest overwritten)
    int tuned_count;
    int tuned_next;
};

// Scratch of sig_compute_noalloc, the entry point for callers that cannot allocate: part of the code object, so
// every device the library runs on holds its own copy from the first use of the library until the process ends.
// In host code the name only stands for the symbol; its device address is looked up once per context
// (hipGetSymbolAddress in sig_create, with the context's device current) and kept in sig_ctx::fixed_scratch.
constexpr size_t kFixedScratchBytes = (size_t)SIG_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) float fixed_scratch_storage[kFixedScratchBytes / sizeof(float)];

namespace {

constexpr int kDefaultCUs = 256;
constexpr int kThreads = 256;
constexpr int kMinChunkSteps = 8;          // chunks inside a workgroup are at least this long
constexpr int kMinSegmentChunkSteps = 48;  // ... and this long before time is also cut across workgroups

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Argument checks shared by sig_plan and the compute entry points (pointers are checked by the latter).
int check_shape(int64_t B, int64_t L, int d, int depth, int stream_flag, RowShape *rs)
{
    if (B < 0 || L < 2 || d < 1 || depth < 1 || (stream_flag != 0 && stream_flag != 1)) return SIG_ERR_INVALID;
    if (depth > kMaxDepth || d > 8192) return SIG_ERR_TOO_LARGE;
    if (!make_row_shape(d, depth, rs)) return SIG_ERR_TOO_LARGE;
    // sizes in floats must fit in int64 with room to spare: B * L * d and B * (L-1) * D
    const int64_t lim = INT64_MAX / 8;
    if (B > 0) {
        if (L > lim / d || B > lim / (L * d)) return SIG_ERR_TOO_LARGE;
        int64_t rows = stream_flag ? L - 1 : 1;
        if (rs->D > lim / rows || B > lim / (rs->D * rows)) return SIG_ERR_TOO_LARGE;
    }
    return SIG_OK;
}

// LDS of the HBM-streaming kernel for prefix depth p: one tile of increments and two chain buffers
bool streaming_fits(const RowShape &rs, int p)
{
    int tile = 8192 / rs.d;
    if (tile > 64) tile = 64;
    if (tile < 1) tile = 1;
    const int64_t gcap = rs.depth - 1 - p >= 0 ? rs.pow[rs.depth - 1 - p] : 1;
    return ((int64_t)tile * rs.d + 2 * gcap) * (int64_t)sizeof(float) <= kMaxLdsBytes;
}

// Can the partial rows of `segments` time segments be joined by the on-chip join kernels?  The LDS-tree join
// (large lane states) holds all rows of a path at once plus half as many results; the register join stages all rows.
constexpr int kMaxTreeSegments = 32;
bool join_fits_lds(const OnChipKernelInfo *ki, int segments, const RowShape &rs)
{
    const int64_t row = rs.D * (int64_t)sizeof(float);
    // (the same predicate as the kernels' own choice of join: the register join needs a small lane state and a
    // path's lanes inside one workgroup)
    const bool reg_join = ki->state_floats <= 64 && ki->lanes_per_chunk <= 256;
    if (!reg_join && (segments + (segments + 1) / 2) * row > kMaxLdsBytes) return false;
    return segments * row <= kMaxLdsBytes;
}

// Time segments for a join in device memory (a pairwise tree of batched row products, one launch of 5-8 us per
// round): a power of two of at most `wanted`, only from 256 increments on (measured on seven shapes, 1 to 256 paths:
// 1.06-1.96x from there on, mixed below) and while one set of partial rows stays within 8 MB (with 32 MB the larger
// batches lose up to 1.7x).  Returns 1 when it does not pay.
int64_t tree_segments(int64_t wanted, int64_t B, int64_t K, const RowShape &rs)
{
    if (K < 256 || wanted < 4) return 1;
    int64_t W = 1;
    while (W * 2 <= wanted && W * 2 <= kMaxTreeSegments && B * W * 2 * rs.D <= ((int64_t)1 << 21)) W *= 2;
    return W;
}

// Fill the derived launch fields of an on-chip plan (chunk_steps, tile_steps) and check every limit the kernel
// relies on.  Returns false if the plan cannot run.
bool finish_on_chip(const OnChipKernelInfo *ki, int cus, int64_t B, int64_t L, int stream_flag, const sig_plan_t &pl,
                    const RowShape &rs, OnChipArgs *args)
{
    const int Q = ki->lanes_per_chunk;
    const int64_t K = L - 1;
    if (pl.chunks < 1 || pl.segments < 1) return false;
    // only the chunked kernels with a small lane state are built for workgroups above 256 threads
    const int max_threads = (pl.chunks > 1 && ki->state_floats <= 64) ? 512 : 256;
    if (pl.threads < kWave || pl.threads > max_threads || pl.threads % kWave) return false;
    if ((int64_t)pl.chunks * pl.segments > K) return false;  // no more pieces than increments
    if (Q > pl.threads && pl.chunks != 1) return false;
    // slots of Q lanes a workgroup offers: packed in final mode, kept inside wavefronts in stream mode
    const int64_t slots = Q > pl.threads ? 1
                          : (stream_flag && Q <= kWave) ? (int64_t)(pl.threads / kWave) * (kWave / Q)
                                                        : pl.threads / Q;
    if (Q <= pl.threads && pl.chunks > slots) return false;
    if (stream_flag && pl.segments != 1) return false;       // carries across workgroups are not implemented
    // rows of the segments that do not fit the LDS of a join kernel are joined in device memory by a pairwise
    // tree of batched row products: a power of two of them
    if (pl.segments > 1 && !join_fits_lds(ki, pl.segments, rs) &&
        (pl.segments > kMaxTreeSegments || (pl.segments & (pl.segments - 1)) != 0))
        return false;
    if (B * (int64_t)pl.segments > INT32_MAX) return false;
    args->B = B;
    args->L = L;
    args->chunks = pl.chunks;
    args->segments = pl.segments;
    args->threads = pl.threads;
    args->stream_flag = stream_flag;
    args->cooperative = pl.independent_waves != 1 && pl.chunks == 1;
    args->chunk_steps = (int)ceil_div(K, (int64_t)pl.chunks * pl.segments);
    if (ceil_div(K, (int64_t)pl.chunks * pl.segments) > INT32_MAX) return false;
    // groups per workgroup: as many as the threads hold, fewer if their chunk signatures overflow LDS
    int G = Q > pl.threads ? 1 : (int)(slots / pl.chunks);
    if (pl.chunks > 1) {
        // chunk signatures in LDS: half a buffer (final mode, lane state small enough for the register tree),
        // one and a half (final mode, LDS tree) or two (stream mode: the scan's prefixes)
        const int64_t rows = stream_flag ? 2 * pl.chunks
                             : ki->state_floats <= 64 ? (pl.chunks + 1) / 2 : pl.chunks + (pl.chunks + 1) / 2;
        const int64_t per_group = rows * rs.D * (int64_t)sizeof(float);
        int64_t fit = (kMaxLdsBytes - 4096) / per_group;
        if (fit < 1) return false;
        if (G > fit) G = (int)fit;
    }
    // spread the groups over the compute units before packing several into one workgroup
    const int64_t per_cu = ceil_div(B * pl.segments, cus);
    if ((int64_t)G > per_cu) G = (int)per_cu;
    args->groups = G;
    // Tile of staged increments.
    //  - chunked kernels: the whole chunk in one tile if it fits the tile budget, otherwise two tiles
    //    (double buffer) short enough for the budget and for the registers that hold the next tile in
    //    flight (kLoaderStage floats per thread over rows padded to a power of two);
    //  - the fold kernel (chunks == 1): every wavefront stages its own groups; 32 steps per tile unless
    //    the plan asks for fewer (LDS per workgroup is checked below).
    const int64_t ngc = (int64_t)G * pl.chunks;
    const int64_t T = args->chunk_steps;
    int64_t tt = T;
    const bool forced = pl.tile_steps > 0 && pl.tile_steps < T;
    if (forced) tt = pl.tile_steps;
    args->pipe = 0;
    if (pl.chunks == 1 && !args->cooperative) {
        if (!forced && tt > kFoldTileSteps) tt = kFoldTileSteps;
    } else if (forced || ngc * T * ki->d * (int64_t)sizeof(float) > kTileLdsBytes) {
        // Several tiles per chunk.  With four or more wavefronts per SIMD resident the other workgroups hide a
        // tile's load latency and the plain loader (load, barrier, consume) keeps the register count low; with
        // fewer, the next tile is kept in flight in registers while the current one is consumed.
        // plan.tile_loader: 1 forces the register-staged loader, 2 the plain one.
        bool pipe;
        if (pl.tile_loader == 1 || pl.tile_loader == 2) {
            pipe = pl.tile_loader == 1;
        } else {
            const int waves_per_wg = pl.threads / kWave;
            int by_vgpr = 512 / (ki->state_floats + 45);
            if (by_vgpr > 8) by_vgpr = 8;
            if (by_vgpr < 1) by_vgpr = 1;
            const int64_t items = ceil_div(B * pl.segments, G);
            int64_t resident = (int64_t)by_vgpr * 4 / waves_per_wg * cus;
            if (resident > items) resident = items;
            // stream mode is bound by its stores; the plain loader with long tiles measured a few percent faster
            pipe = !stream_flag && resident * waves_per_wg < (int64_t)4 * 4 * cus;
        }
        if (pipe) {
            int64_t by_lds = kTileLdsBytes / (2 * ngc * ki->d * (int64_t)sizeof(float));
            int64_t row_pow2 = 1;
            while (row_pow2 * 2 * ngc <= (int64_t)kLoaderStage * pl.threads) row_pow2 *= 2;
            int64_t by_regs = row_pow2 / ki->d;
            if (tt > by_lds) tt = by_lds;
            if (tt > by_regs) tt = by_regs;
        } else {
            int64_t by_lds = kTileLdsBytes / (ngc * ki->d * (int64_t)sizeof(float));
            if (tt > by_lds) tt = by_lds;
            // Shapes with little arithmetic per byte of path (fewer than 16 flops per byte read: depth 2, small
            // depth 3) are bound by reading the path; short tiles keep the workgroups' LDS small, so that more of
            // them are resident and more loads are in flight (measured with 2 to 5 channels: 10 steps per tile beat
            // 19 by 10-30 %; with 8 channels they lose, with 10 it makes no difference).
            if (!forced && !stream_flag && ki->d <= 6) {
                double fma = 0.0;
                for (int m = 1; m <= rs.depth; ++m) fma += (double)(rs.depth - m + 1) * (double)rs.pow[m];
                if (2.0 * fma / (4.0 * ki->d) < 16.0 && tt > 10) tt = 10;
            }
        }
        if (tt < 1) return false;
        args->pipe = pipe && tt < T;
    }
    // Final mode, one chunk, the lanes of a path in several workgroups, two or more prefix letters, and a (path, segment)
    // short enough to be one tile: the kernel that shares the prefix part of the Horner chains through a table in LDS.
    // Taken by default where three or more prefix levels are shared (d = 10, depth 6, p = 4: 1.06-1.09x from 16 paths of
    // 128 points on; with two shared levels it measured 0.94-1.05x on ten shapes, so those keep the other fold);
    // plan.shared_chain: 1 insists on it (invalid where it does not apply), 2 switches it off.
    args->shared_chain = 0;
    if (pl.shared_chain < 0 || pl.shared_chain > 2) return false;
    if (!stream_flag && pl.chunks == 1 && args->cooperative && ki->p >= 2 && Q > 256 && Q > pl.threads && pl.shared_chain != 2 &&
        (pl.shared_chain == 1 || ki->p >= 4) && !forced && shared_chain_fits(ki->d, rs.depth, ki->p, pl.threads, T)) {
        args->shared_chain = 1;
        args->pipe = 0;
        tt = T;
    } else if (pl.shared_chain == 1) {
        return false;   // asked for, but this shape or plan has no such kernel
    }
    args->tile_steps = (int)tt;
    int shift = 0;
    while (((int64_t)1 << shift) < tt * ki->d) ++shift;
    args->row_shift = shift;
    if (args->pipe && (ngc << shift) > (int64_t)kLoaderStage * pl.threads) return false;
    // straight-copy tile: whole paths (one chunk, one segment), one tile, the workgroup-wide kernel, and a path
    // array long enough that the last full vector pair lies inside it
    // (not with few lanes per path: then a wavefront reads many rows at once, and rows of L * d floats, unlike the
    // (L - 1) * d of the generic tile, tend to start in the same LDS bank)
    args->flat_tile = pl.chunks == 1 && pl.segments == 1 && args->cooperative && tt >= T && L * ki->d >= ki->d + 8 &&
                      (int64_t)G * L * ki->d < (1 << 20) && Q >= 8 && !args->shared_chain;
    int64_t lds = ki->lds_bytes(*args);
    while (pl.chunks == 1 && !args->cooperative && !forced && lds > kMaxLdsBytes / 2 && args->tile_steps > 1) {
        // keep at least two workgroups per 64 KB: shorter tiles
        args->tile_steps /= 2;
        shift = 0;
        while (((int64_t)1 << shift) < (int64_t)args->tile_steps * ki->d) ++shift;
        args->row_shift = shift;
        lds = ki->lds_bytes(*args);
    }
    if (lds > kMaxLdsBytes) return false;
    // workgroups that stay resident at once (persistent kernel): limited by registers (estimated from the
    // lane state), LDS (160 KB per CU) and wavefront slots (8 per SIMD)
    {
        const int waves_per_wg = pl.threads / kWave;
        int waves_per_simd = 512 / (ki->state_floats + 45);
        if (waves_per_simd > 8) waves_per_simd = 8;
        if (waves_per_simd < 1) waves_per_simd = 1;
        int64_t per_cu = (int64_t)waves_per_simd * 4 / waves_per_wg;
        if (per_cu < 1) per_cu = 1;
        const int64_t by_lds_cu = (160 * 1024) / (lds > 0 ? lds : 1);
        if (by_lds_cu >= 1 && per_cu > by_lds_cu) per_cu = by_lds_cu;
        args->resident_workgroups = (int32_t)(per_cu * cus);
        args->num_cus = cus;
        // Skewed start (see the kernel): only when the launch needs more than one round of workgroups, so
        // that the lock-step of loads, arithmetic and stores would repeat.  One workgroup's lifetime is
        // estimated as steps x vector instructions per step (1.25 x the FMAs per lane) x resident wavefronts
        // per SIMD x 2.4 cycles at 2.3 GHz, in 100 MHz ticks; the skew per residency slot is that lifetime
        // divided by the slots of a CU.  plan.stagger_ticks: > 0 sets the ticks, < 0 switches the skew off.
        args->stagger_ticks = 0;
        if (pl.stagger_ticks > 0) {
            args->stagger_ticks = pl.stagger_ticks;
        } else if (pl.stagger_ticks == 0 && !stream_flag && pl.chunks == 1 && args->cooperative && Q <= pl.threads &&
                   !args->flat_tile) {
            const int64_t items = ceil_div(B * pl.segments, G);
            // worth it only where the HBM time is a large part of the arithmetic time (measured: it gains 12 % at
            // 5 KB and 0.19 MFLOP per path, and loses a little from twice that path length on)
            double fma_per_path_step = 0.0;
            for (int m = 1; m <= rs.depth; ++m) fma_per_path_step += (double)(rs.depth - m + 1) * (double)rs.pow[m];
            const double t_hbm = 4.0 * ((double)L * ki->d + (double)rs.D) / 4.58e12;  // at the measured copy rate
            const double t_alu = 2.0 * fma_per_path_step * (double)K / 126e12;      // at the measured FMA rate
            if (items > args->resident_workgroups && per_cu > 1 && t_hbm > 0.6 * t_alu) {
                double fma_per_lane = fma_per_path_step;
                fma_per_lane /= (double)Q;
                const double waves_per_simd_res = (double)per_cu * waves_per_wg / 4.0;
                const double life_us = (double)T * 1.25 * fma_per_lane * waves_per_simd_res * 2.4 / 2300.0;
                double ticks = life_us * 100.0 / (double)per_cu;
                if (ticks > 5000.0) ticks = 5000.0;
                args->stagger_ticks = (int32_t)ticks;
            }
        }
    }
    return true;
}

// Constants of the planner, each fitted to timings on an MI355X (256 compute units, 2.4 GHz).  They decide between
// mappings that all give the same result; sig_autotune replaces them by a measurement for one shape.
namespace tune {
constexpr int kSmallState = 64;          // lane states up to this many floats leave six to eight wavefronts per SIMD
constexpr int kFewLanes = 16;            // kernels with fewer lanes per path write long stretches of a row per lane
constexpr int kHeavyState = 40;          // ... or carry this many floats: the deeper entry then wins on longer paths too
constexpr int kDeepShortPath = 256;      // increments up to which a deeper entry beats the first small-state one
constexpr int kDeepShortPathHeavy = 768; // ... behind a few-lane or heavy entry
constexpr int kDeepShortPathWide = 128;  // ... when the deeper entry has more than 128 lanes per path
constexpr int kDeepBatchFactorFewLanes = 4;   // batch limit of the deeper entry, in units of one wavefront per SIMD
constexpr int kStreamDeepShortPath = 128;   // stream mode, under-filled chip: the entry behind a small state up to this many increments ...
constexpr int kStreamDeepHeavyState = 32;   // ... or at any length behind a small state of more floats than this
constexpr int kStreamFewLanes = 10;      // stream mode: kernels with at most this many lanes per path aim at two wavefronts per SIMD
constexpr int kFinalWavesPerSimd = 8;    // occupancy the final-mode time cut aims for
constexpr int kFewLaneMinChunkSteps = 12;     // chunks of few-lane kernels with states of 31-63 floats
constexpr int kFewLaneMinState = 31;
constexpr double kSegmentCostFactor = 1.7;    // segments of a nearly empty chip: factor * sqrt(state K / (D C))
constexpr double kSegmentOccupancyWaves = 2.0;  // segments on a busy chip: this many wavefronts per SIMD over the chunks' own
constexpr int kMaxLdsJoinSegments = 8;
constexpr int kFillByChunksMinSteps = 200;    // from this many increments on, never fewer chunks than fill the chip (final mode)
}  // namespace tune

// Which compiled prefix depth to use for (d, depth); entries of one (d, depth) are ordered by increasing prefix depth.
//  - final mode: the first entry whose lane state is small (several wavefronts per SIMD, chunk tree in registers);
//    an entry behind it (lighter steps, more lanes) for small batches of short paths, which are bound by the latency of
//    the sequential steps; an entry whose lanes span several workgroups only while the batch cannot fill the chip;
//  - stream mode: bound by the stores, so the deepest entry whose lanes fit a workgroup, but behind a small-state entry
//    only while that one has few lanes per path.
const OnChipKernelInfo *pick_on_chip(int d, int depth, int stream_flag, int64_t B, int64_t K, int cus)
{
    const OnChipKernelInfo *best = nullptr;
    for (int t = 0; on_chip_subtable(t); ++t)
    for (const OnChipKernelInfo *e = on_chip_subtable(t); e->launch; ++e) {
        if (e->d != d || e->depth != depth) continue;
        if (!best) { best = e; continue; }
        const bool spans_workgroups = e->lanes_per_chunk > kThreads && best->lanes_per_chunk <= kThreads;
        if (spans_workgroups && (stream_flag || B * best->lanes_per_chunk >= (int64_t)cus * kWave)) continue;
        const bool best_small = best->p > 0 && best->state_floats <= tune::kSmallState;
        const bool best_few_lanes = best->lanes_per_chunk < tune::kFewLanes;
        // final mode, behind a small-state entry: short paths and a batch below one wavefront per SIMD (four behind a
        // few-lane entry)
        const bool heavy_shallower = best_few_lanes || best->state_floats >= tune::kHeavyState;
        const int64_t short_path = e->lanes_per_chunk > 128 ? tune::kDeepShortPathWide
                                   : heavy_shallower        ? tune::kDeepShortPathHeavy
                                                            : tune::kDeepShortPath;
        const int64_t few_lanes = (int64_t)cus * 4 * kWave * (best_few_lanes ? tune::kDeepBatchFactorFewLanes : 1);
        const bool short_and_few = !stream_flag && best_small && e->lanes_per_chunk < kThreads &&
                                   B * e->lanes_per_chunk * (kThreads / e->lanes_per_chunk) <= few_lanes && K <= short_path;
        // stream mode, behind a small-state entry: only while that one has few lanes per path (the four-lane entry of
        // two channels measured 1.9-4.4x over the two-lane one at 1,024 to 16,384 paths as well as below)
        // ... or the batch leaves the small-state entry at most half a wavefront per SIMD and the deeper one fits a
        // workgroup: more lanes per path and lighter steps then, on short paths (up to 128 increments) and behind the
        // heavier small states (more than 32 floats).  Measured on (4,4), (5,4), (6,4) over 50 ... 1,000 points and
        // 16 ... 4,096 paths: (6,4) up to 256 paths 1.2-2.8x (50 points, 64 paths: 33 -> 13 us), (4,4) with up to 100
        // points 1.06-1.5x; long paths of (4,4) and (5,4) 0.8-0.95x, hence the two conditions.
        const bool stream_underfilled = e->lanes_per_chunk <= kThreads &&
                                        B * best->lanes_per_chunk * 2 <= (int64_t)cus * 4 * kWave &&
                                        (K <= tune::kStreamDeepShortPath || best->state_floats > tune::kStreamDeepHeavyState);
        if (stream_flag && best_small && !best_few_lanes && !stream_underfilled) continue;
        // final mode, behind an entry with two lanes per path (two channels, p = 1): the next one (four lanes, half the
        // state) measured 1.1-1.6x at every batch and length once it fits its small-state budget
        const bool two_lanes = !stream_flag && best_small && best->lanes_per_chunk <= 2 &&
                               e->state_floats <= tune::kSmallState && e->lanes_per_chunk <= 4;
        if (stream_flag || best->state_floats > tune::kSmallState || best->p == 0 || short_and_few || two_lanes) best = e;
    }
    return best;
}

// The level-scan family keeps the levels below the top one of every prefix in scratch: a batch whose tensors would
// exceed 8 GiB is taken in equal slices of paths, one after the other on the caller's stream, which share the
// buffer (a slice of that size fills the chip many times over, so nothing is lost but the memory).
constexpr int64_t kLevelScanSliceFloats = (int64_t)1 << 31;

int64_t level_scan_slice_paths(int64_t B, int64_t L, const RowShape &rs, int stream_flag)
{
    const int64_t per_path = level_scan_scratch_floats(1, L, rs, stream_flag);
    if (B <= 1 || per_path <= 0 || per_path <= kLevelScanSliceFloats / B) return B;
    int64_t paths = kLevelScanSliceFloats / per_path;
    if (paths < 1) paths = 1;
    const int64_t slices = ceil_div(B, paths);
    return ceil_div(B, slices);
}

// the level-scan family takes chunks >= 0 and ignores the other mapping fields
int check_level_scan(int64_t B, int64_t L, const RowShape &rs, int stream_flag, const sig_plan_t &pl)
{
    if (!level_scan_available(rs.d, rs.depth)) return SIG_ERR_INVALID;
    if (pl.chunks < 0) return SIG_ERR_INVALID;
    if (!level_scan_fits(L, rs, stream_flag)) return SIG_ERR_TOO_LARGE;   // also bounds one path's scratch (2^31)
    const int64_t S = level_scan_slice_paths(B, L, rs, stream_flag);
    if (S * rs.pow[rs.depth - 1] > INT32_MAX) return SIG_ERR_TOO_LARGE;
    const int64_t floats = level_scan_scratch_floats(S, L, rs, stream_flag);
    if (floats < 0 || floats > (int64_t)1 << 36) return SIG_ERR_TOO_LARGE;
    return SIG_OK;
}

int plan_auto(const sig_ctx *ctx, int64_t B, int64_t L, int stream_flag, const RowShape &rs, sig_plan_t *pl)
{
    const int cus = ctx ? ctx->num_cu : kDefaultCUs;
    const int64_t K = L - 1;
    const int64_t simd_lanes = (int64_t)cus * 4 * kWave;   // one wavefront on every SIMD
    // lanes that fill the chip: eight wavefronts on every SIMD for the arithmetic-bound final mode, one for stream mode
    // (bound by the stores; cutting time there costs a second fold)
    int64_t want_lanes = simd_lanes * (stream_flag ? 1 : tune::kFinalWavesPerSimd);
    *pl = sig_plan_t{};
    pl->threads = kThreads;

    const OnChipKernelInfo *ki = (B > 0) ? pick_on_chip(rs.d, rs.depth, stream_flag, B, K, cus) : nullptr;
    if (ki) {
        const int Q = ki->lanes_per_chunk;
        const int state = ki->state_floats;
        const bool small_state = state <= tune::kSmallState;
        const bool few_lane_heavy = Q < tune::kFewLanes && state >= tune::kFewLaneMinState;   // few lanes, 31 floats or more each
        // do not cut time to fill wavefront slots that the registers cannot hold (state + 45 registers per lane)
        if (!stream_flag && (!small_state || few_lane_heavy)) {
            int by_vgpr = 512 / (state + 45);
            if (by_vgpr < 1) by_vgpr = 1;
            if (by_vgpr < tune::kFinalWavesPerSimd) want_lanes = simd_lanes * by_vgpr;
        }
        // stream mode, kernels with at most ten lanes per path (each lane stores a long stretch of every row): two
        // wavefronts per SIMD.  Planner against autotuner on 16 shapes x 50 ... 1,000 points x 64 ... 16,384 paths: the tuner
        // doubled the chunks of these kernels almost everywhere (1.2-1.8x at 1,024 and 4,096 paths) and halved or
        // kept those of the kernels with 16 lanes or more (twice the chunks: 0.8-0.9x there).
        if (stream_flag && Q <= tune::kStreamFewLanes) want_lanes = 2 * simd_lanes;
        // (the kernels with up to 63 lanes of at most 16 floats gain 1.05-1.25x from twice the chunks too, but only
        // where the time is cut anyway: an uncut plan keeps its narrow workgroups, which twice the lanes would give up
        // for 0.8-0.9x)
        if (stream_flag && Q > tune::kStreamFewLanes && Q < kWave && state <= 16 && B * Q < simd_lanes)
            want_lanes = 2 * simd_lanes;
        pl->variant = SIG_VARIANT_ON_CHIP;
        pl->prefix_depth = ki->p;
        pl->chunks = 1;
        pl->segments = 1;
        // Workgroups of 512 threads (twice the chunks side by side) for small lane states on batches that would leave
        // the chip at or below a wavefront per SIMD with 256: kernels with more than 64 lanes per path, and the entries
        // behind the first small state once the path is long enough for twice the chunks.
        const int64_t slots256 = Q <= kThreads ? kThreads / Q : 1;
        const bool few = B * Q * slots256 <= simd_lanes;
        const OnChipKernelInfo *shallower = ki->p > 1 ? find_on_chip(rs.d, rs.depth, ki->p - 1) : nullptr;
        const bool deeper = shallower && shallower->state_floats <= tune::kSmallState;
        const bool wide = !stream_flag && small_state && Q < kThreads && few &&
                          (Q > kWave || (deeper && (Q == kWave || K / kMinChunkSteps >= 2 * slots256)));
        const int wg = wide ? 2 * kThreads : kThreads;
        pl->threads = wg;
        if (Q <= kThreads) {
            // cut time into pieces only as far as needed to fill the chip; every cut costs one Eq. 4 product
            int64_t pieces = ceil_div(want_lanes, B * Q);
            // chunks side by side in a workgroup (stream kernels keep a chunk's lanes inside one wavefront), within the
            // LDS their rows take: two buffers in stream mode and for the LDS tree, half of one for the register tree
            int64_t cmax = (stream_flag && Q <= kWave) ? (int64_t)(kThreads / kWave) * (kWave / Q) : wg / Q;
            int64_t clds = (kMaxLdsBytes - kTileLdsBytes) /
                           ((stream_flag || !small_state ? 2 : 1) * rs.D * (int64_t)sizeof(float));
            if (wide) clds *= 2;
            if (cmax > clds) cmax = clds;
            // shortest chunk: eight steps; stream mode (every chunk is folded twice, the sequential steps dominate) four
            // up to 32 floats of state and three up to 16; twelve for the few-lane kernels with heavy states in final mode
            // (their chunk tree multiplies long rows with few lanes)
            const int64_t min_steps = !stream_flag ? ((few_lane_heavy && small_state) ? tune::kFewLaneMinChunkSteps : kMinChunkSteps)
                                      : state <= 16 ? 3 : state <= 32 ? 4 : kMinChunkSteps;
            if (cmax > K / min_steps) cmax = K / min_steps;
            if (cmax < 1) cmax = 1;
            int64_t C = pieces < cmax ? pieces : cmax;
            if (!(stream_flag && Q <= kWave)) {
                // lanes are packed group after group: prefer a nearby chunk count whose groups fill the workgroup
                // (e.g. Q = 25: 6 chunks leave 106 of 256 lanes idle, 5 chunks fit twice)
                // (fewer chunks than it takes to fill the chip only within a fifth of full: (5,4) with 2,000 points at
                // 8,192 paths wants three chunks; one chunk fills its workgroups but leaves three wavefronts per SIMD,
                // 582 us against 422 us with five)
                auto used = [&](int64_t c) { return (wg / (c * Q)) * c * Q; };
                // (where the chunks cannot fill the chip anyway the question does not arise; paths under 200 increments
                // and stream mode, where a cut costs a second fold, measured 0.63-0.98x with the larger count, longer
                // paths in final mode 1.0-1.41x over 41 shapes)
                auto fills = [&](int64_t c) {
                    return stream_flag || K < tune::kFillByChunksMinSteps || C < pieces || c * B * Q * 10 >= want_lanes * 8;
                };
                int64_t best = C;
                for (int64_t c = (C > 2 ? C - 2 : 1); c <= C + 4 && c <= cmax; ++c) {
                    if (c < C && !fills(c)) continue;
                    if (used(c) * 100 > used(best) * 105 || (used(c) * 100 > used(best) * 95 && best > C && c >= C && c < best)) best = c;
                }
                C = best;
            }
            // far from a full chip with short chunks: a power of two just below C saves a round of the chunk tree
            if (!stream_flag && pieces >= 2 * C && C >= 5 && K <= 24 * C) {
                int64_t p2 = 1;
                while (p2 * 2 <= C) p2 *= 2;
                if (p2 < C && 4 * p2 >= 3 * C) C = p2;
            }
            // further workgroups along time (a second launch joins them) only while each chunk keeps a long run
            int64_t W = 1;
            if (!stream_flag) {
                W = (pieces + C / 2) / C;  // rounded: a second launch is not worth a few missing lanes
                int64_t wmax = K / (C * kMinSegmentChunkSteps);
                // nearly empty chip (at most half a wavefront per SIMD): the launch takes about a K / (C W) + b W, minimal
                // at W = factor * sqrt(state K / (D C)); chunks keep at least eight steps; not for fewer than three
                int64_t by_cost = (int64_t)(tune::kSegmentCostFactor * std::sqrt((double)state * (double)K / ((double)rs.D * (double)C)));
                if (by_cost > K / (C * kMinChunkSteps)) by_cost = K / (C * kMinChunkSteps);
                if (by_cost >= 3 && B * Q * C <= simd_lanes / 2 && wmax < by_cost) wmax = by_cost;
                if (W > wmax) W = wmax;
                // busy chip, small lane states: the second launch and the join pay only for long paths
                if (small_state) {
                    const int64_t lanes = B * Q * C;
                    int64_t by_occupancy = (int64_t)(tune::kSegmentOccupancyWaves * (double)simd_lanes / (double)lanes * std::sqrt((double)K / 1000.0) + 0.25);
                    if (by_occupancy < 1) by_occupancy = 1;
                    if (W > by_occupancy) W = by_occupancy;
                }
                const int64_t wanted = W;
                if (W > tune::kMaxLdsJoinSegments) W = tune::kMaxLdsJoinSegments;
                while (W > 1 && !join_fits_lds(ki, (int)W, rs)) --W;
                if (W < 1) W = 1;
                // rows too long for the LDS of a join kernel: a tree in device memory if it allows four times the segments
                const int64_t tree = tree_segments(wanted, B, K, rs);
                if (tree >= 4 && tree >= 4 * W) W = tree;
            }
            pl->chunks = (int)C;
            pl->segments = (int)W;
        } else if (!stream_flag) {
            // the lanes of a path span several workgroups: no chunks, but segments joined in device memory
            int64_t W = ceil_div(want_lanes, B * Q);
            if (W > K / kMinSegmentChunkSteps) W = K / kMinSegmentChunkSteps;
            W = tree_segments(W, B, K, rs);
            if (W >= 4) pl->segments = (int)W;
        }
        // Stream mode with few paths: the on-chip kernels walk K / C steps one after the other (twice when time is
        // cut) and a wavefront stages every row through LDS, while the level-scan family (one launch per level,
        // parallel in time) only pays its launches.  Estimates in microseconds fitted to a measured grid (21
        // shapes, B = 1 .. 8192, L = 100 and 500).  On-chip, per step: 0.1 + 0.01 per state float, plus 0.022 per
        // row-copy iteration of a wavefront (0.1 when the rows are short enough for the per-lane element table);
        // kernels whose lanes store their own state (more than 64 lanes per path): 0.0125 per state float.  The
        // level-scan family: 6.4 + 0.0062 K per level (1 more from 8 paths on) plus its output at 2.36 TB/s (a fit to
        // 248 measured calls, 14 % rms; final mode: 6.5 + 0.008 K per level, 2 more from 8 paths on).  It is
        // taken when the on-chip estimate is 1.3 times larger and the on-chip plan leaves the chip below two
        // wavefronts per SIMD (measured there: up to 15x faster, e.g. d = 8, depth 4, one path of 500 points: 49
        // against 737 us; the estimates err on the side of the on-chip kernels).
        // Final mode: only plans that could not be cut in time at all (large lane states whose rows do not fit LDS
        // for a join, on paths of fewer than 256 increments) can lose, with few paths: K dependent steps
        // of 0.1 + 0.002 us per state float against the level-scan family's launches plus 2.6 x its scratch tensor
        // at 2 TB/s.
        auto prefer_level_scan = [&](const sig_plan_t &chosen) {
            sig_plan_t ls{};
            ls.variant = SIG_VARIANT_LEVEL_SCAN;
            if (check_level_scan(B, L, rs, stream_flag, ls) != SIG_OK) return false;
            if (level_scan_scratch_floats(B, L, rs, stream_flag) > (int64_t)1 << 31) return false;
            const int C = chosen.chunks;
            const double waves = (double)B * Q * C / kWave;
            if (waves > 2.0 * cus * 4) return false;
            const double launches = stream_flag ? rs.depth * (6.4 + 0.0062 * (double)K + (B >= 8 ? 1.0 : 0.0))
                                                : rs.depth * (6.5 + 0.008 * (double)K + (B >= 8 ? 2.0 : 0.0));
            if (!stream_flag) {
                if (C != 1 || chosen.segments != 1) return false;
                const int64_t floats = level_scan_scratch_floats(B, L, rs, 0);
                const double on_chip_final = 6.0 + (double)K * (0.1 + 0.002 * ki->state_floats);
                return on_chip_final > 1.4 * (launches + 2.6 * 4.0 * (double)floats / 2.0e6);
            }
            double rounds = 0;
            for (int c = 1; c < C; c *= 2) rounds += 1.5;
            const double seq = C > 1 ? 2.0 * (double)ceil_div(K, C) + rounds : (double)K;
            double step = 0.0125 * ki->state_floats;
            if (Q <= kWave) {
                const int64_t rowv = rs.D % 4 == 0 ? rs.D / 4 : rs.D;
                const int64_t spw = kWave / Q;
                const int64_t table = ceil_div(spw * rowv, kWave);
                step = 0.1 + 0.01 * ki->state_floats + (table <= 8 ? 0.1 : 0.022 * (double)(spw * ceil_div(rowv, kWave)));
            }
            const double on_chip = 6.0 + seq * step;
            const double out_bytes = 4.0 * (double)B * (double)K * (double)rs.D;
            return on_chip > 1.3 * (launches + out_bytes / 2.36e6);
        };
        auto take_level_scan = [&]() {
            *pl = sig_plan_t{};
            pl->variant = SIG_VARIANT_LEVEL_SCAN;
            pl->threads = kThreads;
            pl->segments = 1;
            return SIG_OK;
        };
        // Stream mode without time cuts: one wavefront per workgroup if its paths then fit one straight-copy tile
        // with room for six workgroups per CU.  A tile boundary costs a stream kernel a drain of its store
        // queue (the loader's wait also waits for every store issued before it); measured 5 % on d = 4, depth 4.
        if (stream_flag && pl->chunks == 1 && pl->segments == 1 && Q <= kWave) {
            sig_plan_t narrow = *pl;
            narrow.threads = kWave;
            OnChipArgs args{};
            if (finish_on_chip(ki, cus, B, L, stream_flag, narrow, rs, &args) && args.flat_tile &&
                ki->lds_bytes(args) <= 26 * 1024) {
                if (prefer_level_scan(narrow)) return take_level_scan();
                *pl = narrow;
                pl->tile_steps = args.tile_steps;
                return SIG_OK;
            }
        }
        // the preferred cut may not fit (LDS for the chunk rows and for the rows staged for emission grows with
        // the row length): fall back to smaller workgroups, then to fewer chunks, before giving up on the family
        const sig_plan_t want = *pl;
        for (int c = want.chunks; c >= 1; c = (c > 1 ? (c + 1) / 2 : 0)) {
            for (int threads = (c == want.chunks ? want.threads : kThreads); threads >= kWave; threads /= 2) {
                *pl = want;
                pl->chunks = c;
                pl->threads = threads;
                if (c != want.chunks) pl->segments = 1;
                OnChipArgs args{};
                if (finish_on_chip(ki, cus, B, L, stream_flag, *pl, rs, &args)) {
                    if (prefer_level_scan(*pl)) return take_level_scan();
                    pl->tile_steps = args.tile_steps;
                    return SIG_OK;
                }
            }
            if (c == 1) break;
        }
        // fall through to the streaming family
        *pl = sig_plan_t{};
        pl->threads = kThreads;
    }
    // No on-chip kernel for this shape.  The level-by-level family is parallel in time and measured 2-25x faster
    // than the state-in-HBM sweep on every such shape (few paths above all), so it is the fallback wherever it
    // applies (d <= 256, depth <= 8) and the scratch tensor of one path stays below 8 GiB (larger batches go in
    // slices); the HBM-streaming family takes the rest.
    if (B > 0) {
        sig_plan_t ls{};
        ls.variant = SIG_VARIANT_LEVEL_SCAN;
        ls.threads = kThreads;
        ls.segments = 1;
        if (check_level_scan(B, L, rs, stream_flag, ls) == SIG_OK &&
            level_scan_scratch_floats(1, L, rs, stream_flag) <= kLevelScanSliceFloats) {
            *pl = ls;
            return SIG_OK;
        }
    }
    pl->variant = SIG_VARIANT_HBM_STREAMING;
    pl->chunks = 1;
    pl->segments = 1;
    pl->tile_steps = 0;
    // cut the index space until the Horner-chain buffers of a sub-tree fit LDS (2 x d^{depth-1-p} floats) and
    // there are enough workgroups, but keep at least one level to the workgroup
    int p = 0;
    const int64_t want_wgs = 4 * (int64_t)cus;
    while (p < rs.depth - 1 && !streaming_fits(rs, p)) ++p;
    while (p < rs.depth - 1 && B * rs.pow[p] < want_wgs && rs.pow[rs.depth - p - 1] >= 4 * kThreads) ++p;
    if (!streaming_fits(rs, p)) return SIG_ERR_TOO_LARGE;
    pl->prefix_depth = p;
    if (B * rs.pow[p] > INT32_MAX) return SIG_ERR_TOO_LARGE;
    return SIG_OK;
}

const sig_plan_t *find_tuned(const sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag)
{
    if (!ctx) return nullptr;
    for (int i = 0; i < ctx->tuned_count; ++i) {
        const TunedPlan &t = ctx->tuned[i];
        if (t.B == B && t.L == L && t.d == d && t.depth == depth && t.stream_flag == stream_flag) return &t.plan;
    }
    return nullptr;
}

// the mapping sig_compute uses: one measured by sig_autotune for exactly this shape, else the planner's
int plan_for(const sig_ctx *ctx, int64_t B, int64_t L, int stream_flag, const RowShape &rs, sig_plan_t *pl)
{
    if (const sig_plan_t *t = find_tuned(ctx, B, L, rs.d, rs.depth, stream_flag)) {
        *pl = *t;
        return SIG_OK;
    }
    return plan_auto(ctx, B, L, stream_flag, rs, pl);
}

int ensure_scratch(sig_ctx *ctx, size_t bytes)
{
    if (bytes <= ctx->scratch_bytes) return SIG_OK;
    if (ctx->scratch) {
        // earlier launches on the caller's stream may still read the old buffer
        if (hipDeviceSynchronize() != hipSuccess) return SIG_ERR_HIP;
        (void)hipFree(ctx->scratch);
        ctx->scratch = nullptr;
        ctx->scratch_bytes = 0;
    }
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return SIG_ERR_ALLOC;
    }
    ctx->scratch = static_cast<float *>(p);
    ctx->scratch_bytes = bytes;
    return SIG_OK;
}

// Scratch of `bytes` for one call: the context's own buffer, grown on demand, or (fixed) the array that is part of
// the code object, which is never grown: a call that needs more is refused.
int get_scratch(sig_ctx *ctx, bool fixed, size_t bytes, float **p)
{
    if (fixed) {
        if (bytes > kFixedScratchBytes) return SIG_ERR_TOO_LARGE;
        *p = ctx->fixed_scratch;
        return SIG_OK;
    }
    const int rc = ensure_scratch(ctx, bytes);
    *p = ctx->scratch;
    return rc;
}

int run_plan(sig_ctx *ctx, const float *path, int64_t B, int64_t L, const RowShape &rs, int stream_flag,
             float *out, const sig_plan_t &pl, hipStream_t st, bool fixed = false)
{
    if (pl.variant == SIG_VARIANT_HBM_STREAMING) {
        if (pl.prefix_depth < 0 || pl.prefix_depth > rs.depth - 1) return SIG_ERR_INVALID;
        if (pl.threads < kWave || pl.threads > 256 || pl.threads % kWave) return SIG_ERR_INVALID;
        if (B * rs.pow[pl.prefix_depth] > INT32_MAX) return SIG_ERR_TOO_LARGE;
        if (!streaming_fits(rs, pl.prefix_depth)) return SIG_ERR_INVALID;
        hipError_t e = launch_hbm_streaming(path, out, B, L, rs, pl.prefix_depth, stream_flag, pl.threads, st);
        return e == hipSuccess ? SIG_OK : SIG_ERR_HIP;
    }
    if (pl.variant == SIG_VARIANT_LEVEL_SCAN) {
        int rc = check_level_scan(B, L, rs, stream_flag, pl);
        if (rc != SIG_OK) return rc;
        const int64_t S = level_scan_slice_paths(B, L, rs, stream_flag);
        const int64_t floats = level_scan_scratch_floats(S, L, rs, stream_flag);
        float *work = nullptr;
        if (floats > 0) {
            rc = get_scratch(ctx, fixed, (size_t)floats * sizeof(float), &work);
            if (rc != SIG_OK) return rc;
        }
        const int64_t out_per_path = stream_flag ? (L - 1) * rs.D : rs.D;
        for (int64_t b0 = 0; b0 < B; b0 += S) {
            const int64_t nb = B - b0 < S ? B - b0 : S;
            hipError_t e = launch_level_scan(path + b0 * L * rs.d, out + b0 * out_per_path, work, nb, L, rs, stream_flag,
                                             pl.chunks, ctx->num_cu, st);
            if (e != hipSuccess) return SIG_ERR_HIP;
        }
        return SIG_OK;
    }
    if (pl.variant != SIG_VARIANT_ON_CHIP) return SIG_ERR_INVALID;
    const OnChipKernelInfo *ki = find_on_chip(rs.d, rs.depth, pl.prefix_depth);
    if (!ki) return SIG_ERR_INVALID;
    OnChipArgs args{};
    if (!finish_on_chip(ki, ctx->num_cu, B, L, stream_flag, pl, rs, &args)) return SIG_ERR_INVALID;
    args.path = path;
    args.out = out;
    args.partial = nullptr;
    const bool lds_join = pl.segments > 1 && join_fits_lds(ki, pl.segments, rs);
    const size_t rows = (size_t)B * pl.segments * rs.D;   // floats of the partial rows
    float *work = nullptr;
    if (pl.segments > 1) {
        // (the tree in device memory ping-pongs between two more buffers of half and a quarter of the rows)
        int rc = get_scratch(ctx, fixed, (lds_join ? rows : rows + rows / 2 + rows / 4 + 4) * sizeof(float), &work);
        if (rc != SIG_OK) return rc;
        args.partial = work;
    }
    hipError_t e = ki->launch(args, st);
    if (e != hipSuccess) return SIG_ERR_HIP;
    if (lds_join) {
        e = ki->join(work, out, B, pl.segments, st);
        if (e != hipSuccess) return SIG_ERR_HIP;
    } else if (pl.segments > 1) {
        // round r joins neighbours: row 2 i (x) row 2 i + 1 of the previous round's rows, the last round into `out`
        const float *in = work;
        float *buf[2] = {work + rows, work + rows + rows / 2};
        int which = 0;
        for (int64_t n = pl.segments; n > 1; n /= 2) {
            float *dst = n == 2 ? out : buf[which];
            e = launch_combine_rows(in, 2 * rs.D, in + rs.D, 2 * rs.D, dst, rs.D, B * (n / 2), rs, st);
            if (e != hipSuccess) return SIG_ERR_HIP;
            in = dst;
            which ^= 1;
        }
    }
    return SIG_OK;
}

}  // namespace

extern "C" {

int64_t sig_size(int d, int depth)
{
    if (d < 1 || depth < 1) return -1;
    int64_t total = 0, p = 1;
    for (int n = 1; n <= depth; ++n) {
        if (p > INT64_MAX / d) return -1;
        p *= d;
        if (total > INT64_MAX - p) return -1;
        total += p;
    }
    return total;
}

int sig_create(sig_ctx **ctx)
{
    if (!ctx) return SIG_ERR_INVALID;
    *ctx = nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return SIG_ERR_NO_DEVICE;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return SIG_ERR_NO_DEVICE;
    }
    sig_ctx *c = new (std::nothrow) sig_ctx;
    if (!c) return SIG_ERR_ALLOC;
    c->device = dev;
    c->num_cu = cus;
    c->scratch = nullptr;
    c->scratch_bytes = 0;
    // the address of this device's copy of the fixed scratch array (the current device is the context's)
    void *fixed = nullptr;
    if (hipGetSymbolAddress(&fixed, HIP_SYMBOL(fixed_scratch_storage)) != hipSuccess || !fixed) {
        (void)hipGetLastError();
        delete c;
        return SIG_ERR_HIP;
    }
    c->fixed_scratch = static_cast<float *>(fixed);
    c->tuned_count = 0;
    c->tuned_next = 0;
    *ctx = c;
    return SIG_OK;
}

void sig_destroy(sig_ctx *ctx)
{
    if (!ctx) return;
    if (ctx->scratch) {
        (void)hipDeviceSynchronize();
        (void)hipFree(ctx->scratch);
    }
    delete ctx;
}

int sig_plan(const sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag, sig_plan_t *plan)
{
    if (!plan) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    return plan_for(ctx, B, L, stream_flag, rs, plan);
}

int sig_plan_validate(int64_t B, int64_t L, int d, int depth, int stream_flag, const sig_plan_t *plan)
{
    if (!plan) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    if (plan->variant == SIG_VARIANT_HBM_STREAMING) {
        if (plan->prefix_depth < 0 || plan->prefix_depth > rs.depth - 1) return SIG_ERR_INVALID;
        if (plan->threads < kWave || plan->threads > 256 || plan->threads % kWave) return SIG_ERR_INVALID;
        if (B * rs.pow[plan->prefix_depth] > INT32_MAX) return SIG_ERR_TOO_LARGE;
        if (!streaming_fits(rs, plan->prefix_depth)) return SIG_ERR_INVALID;
        return SIG_OK;
    }
    if (plan->variant == SIG_VARIANT_LEVEL_SCAN) return check_level_scan(B, L, rs, stream_flag, *plan);
    if (plan->variant != SIG_VARIANT_ON_CHIP) return SIG_ERR_INVALID;
    const OnChipKernelInfo *ki = find_on_chip(rs.d, rs.depth, plan->prefix_depth);
    OnChipArgs args{};
    if (!ki || !finish_on_chip(ki, kDefaultCUs, B, L, stream_flag, *plan, rs, &args)) return SIG_ERR_INVALID;
    return SIG_OK;
}

int sig_plan_footprint(int64_t B, int64_t L, int d, int depth, int stream_flag, const sig_plan_t *plan,
                       int64_t *lds_bytes, int64_t *workgroups, int64_t *scratch_bytes)
{
    if (!plan) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    int64_t lds = 0, wgs = 0, scratch = 0;
    if (plan->variant == SIG_VARIANT_HBM_STREAMING) {
        rc = sig_plan_validate(B, L, d, depth, stream_flag, plan);
        if (rc != SIG_OK) return rc;
        int tile = 8192 / rs.d;
        if (tile > 64) tile = 64;
        if (tile < 1) tile = 1;
        const int64_t gcap = rs.pow[rs.depth - 1 - plan->prefix_depth];
        lds = ((int64_t)tile * rs.d + 2 * gcap) * (int64_t)sizeof(float);
        wgs = B * rs.pow[plan->prefix_depth];
    } else if (plan->variant == SIG_VARIANT_LEVEL_SCAN) {
        rc = check_level_scan(B, L, rs, stream_flag, *plan);
        if (rc != SIG_OK) return rc;
        lds = -1;   // one launch per level, each with its own geometry
        wgs = -1;
        scratch = B > 0 ? level_scan_scratch_floats(level_scan_slice_paths(B, L, rs, stream_flag), L, rs, stream_flag) *
                              (int64_t)sizeof(float)
                        : 0;
    } else if (plan->variant == SIG_VARIANT_ON_CHIP) {
        const OnChipKernelInfo *ki = find_on_chip(rs.d, rs.depth, plan->prefix_depth);
        OnChipArgs args{};
        if (!ki || !finish_on_chip(ki, kDefaultCUs, B, L, stream_flag, *plan, rs, &args)) return SIG_ERR_INVALID;
        lds = ki->lds_bytes(args);
        wgs = B > 0 ? on_chip_workgroups(ki->lanes_per_chunk, args) : 0;
        if (plan->segments > 1) {
            const int64_t rows = B * plan->segments * rs.D;
            scratch = (join_fits_lds(ki, plan->segments, rs) ? rows : rows + rows / 2 + rows / 4 + 4) * (int64_t)sizeof(float);
        }
    } else {
        return SIG_ERR_INVALID;
    }
    if (lds_bytes) *lds_bytes = lds;
    if (workgroups) *workgroups = wgs;
    if (scratch_bytes) *scratch_bytes = scratch;
    return SIG_OK;
}

int sig_compute_planned(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth,
                        int stream_flag, float *out, const sig_plan_t *plan, void *hip_stream)
{
    if (!ctx || !plan) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_OK;
    if (!path || !out) return SIG_ERR_INVALID;
    return run_plan(ctx, path, B, L, rs, stream_flag, out, *plan, static_cast<hipStream_t>(hip_stream));
}

int sig_compute(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth,
                int stream_flag, float *out, void *hip_stream)
{
    if (!ctx) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_OK;
    if (!path || !out) return SIG_ERR_INVALID;
    sig_plan_t pl;
    rc = plan_for(ctx, B, L, stream_flag, rs, &pl);
    if (rc != SIG_OK) return rc;
    return run_plan(ctx, path, B, L, rs, stream_flag, out, pl, static_cast<hipStream_t>(hip_stream));
}

int sig_compute_noalloc(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth,
                        int stream_flag, float *out, void *hip_stream)
{
    if (!ctx) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_OK;
    if (!path || !out) return SIG_ERR_INVALID;
    sig_plan_t pl;
    rc = plan_for(ctx, B, L, stream_flag, rs, &pl);
    if (rc != SIG_OK) return rc;
    return run_plan(ctx, path, B, L, rs, stream_flag, out, pl, static_cast<hipStream_t>(hip_stream), true);
}

int sig_autotune(sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag, sig_plan_t *chosen,
                 float *microseconds, void *hip_stream)
{
    if (!ctx) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_ERR_INVALID;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    sig_plan_t base;
    rc = plan_auto(ctx, B, L, stream_flag, rs, &base);
    if (rc != SIG_OK) return rc;

    // candidates: the planner's choice, the level-scan family, and for the register kernels every compiled prefix
    // depth with the planner's time cut and with half and twice as many chunks
    sig_plan_t cand[24];
    int n = 0;
    cand[n++] = base;
    {
        sig_plan_t ls{};
        ls.variant = SIG_VARIANT_LEVEL_SCAN;
        ls.threads = kThreads;
        ls.segments = 1;
        if (base.variant != SIG_VARIANT_LEVEL_SCAN && check_level_scan(B, L, rs, stream_flag, ls) == SIG_OK &&
            level_scan_scratch_floats(1, L, rs, stream_flag) <= kLevelScanSliceFloats)
            cand[n++] = ls;
    }
    for (int p = 0; p < depth && n < 20; ++p) {
        const OnChipKernelInfo *ki = find_on_chip(d, depth, p);
        if (!ki) continue;
        const int c0 = base.variant == SIG_VARIANT_ON_CHIP ? base.chunks : 8;
        const int w0 = base.variant == SIG_VARIANT_ON_CHIP ? base.segments : 1;
        const int chunk_opts[3] = {c0, c0 > 1 ? c0 / 2 : 2, c0 * 2};
        for (int ci = 0; ci < 3 && n < 20; ++ci) {
            sig_plan_t pl{};
            pl.variant = SIG_VARIANT_ON_CHIP;
            pl.prefix_depth = p;
            pl.chunks = chunk_opts[ci];
            pl.segments = stream_flag ? 1 : w0;
            pl.threads = kThreads;
            OnChipArgs args{};
            if (pl.chunks < 1 || !finish_on_chip(ki, ctx->num_cu, B, L, stream_flag, pl, rs, &args)) continue;
            bool dup = false;
            for (int i = 0; i < n; ++i)
                dup = dup || (cand[i].variant == pl.variant && cand[i].prefix_depth == p && cand[i].chunks == pl.chunks &&
                              cand[i].segments == pl.segments && cand[i].threads == pl.threads);
            if (!dup) cand[n++] = pl;
        }
    }

    // synthetic input (zeros: no kernel's timing depends on the values) and an output buffer of the real size
    const size_t path_bytes = (size_t)B * (size_t)L * (size_t)d * sizeof(float);
    const size_t out_bytes = (size_t)B * (size_t)(stream_flag ? L - 1 : 1) * (size_t)rs.D * sizeof(float);
    float *path = nullptr, *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int status = SIG_OK;
    if (hipMalloc(reinterpret_cast<void **>(&path), path_bytes) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&out), out_bytes) != hipSuccess) {
        (void)hipGetLastError();
        status = SIG_ERR_ALLOC;
    } else if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess ||
               hipMemsetAsync(path, 0, path_bytes, st) != hipSuccess) {
        status = SIG_ERR_HIP;
    }
    int best = -1;
    float best_us = 0.0f;
    // times one candidate; returns false if the kernels refuse it (skipped) or a HIP call failed (status set)
    auto time_plan = [&](const sig_plan_t &pl, float *us_out) {
        int r = SIG_OK;
        for (int w = 0; w < 2 && r == SIG_OK; ++w) r = run_plan(ctx, path, B, L, rs, stream_flag, out, pl, st);
        if (r != SIG_OK) return false;
        // five calls, and forty more if they took under a quarter of a millisecond (short calls time noisily)
        float us = 0.0f;
        for (int pass = 0, reps = 5; pass < 2; ++pass, reps = 40) {
            if (hipEventRecord(e0, st) != hipSuccess) { status = SIG_ERR_HIP; return false; }
            for (int k = 0; k < reps && r == SIG_OK; ++k) r = run_plan(ctx, path, B, L, rs, stream_flag, out, pl, st);
            if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { status = SIG_ERR_HIP; return false; }
            float ms = 0.0f;
            if (r != SIG_OK || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return false;
            us = ms * 1000.0f / reps;
            if (ms > 0.25f) break;
        }
        *us_out = us;
        return true;
    };
    float first_us = 0.0f;
    bool first_ok = false;
    for (int i = 0; i < n && status == SIG_OK; ++i) {
        float us = 0.0f;
        if (!time_plan(cand[i], &us)) continue;
        if (i == 0) { first_us = us; first_ok = true; }
        // the planner's own choice (candidate 0) is kept unless another mapping is at least 3 % faster
        if (best < 0 || us < 0.97f * best_us) { best = i; best_us = us; }
    }
    // the first candidate was timed right after the allocations, when calls have been seen to run several times
    // slower for a while: before another mapping replaces the planner's choice, time that choice once more
    if (status == SIG_OK && best > 0 && first_ok) {
        float again = 0.0f;
        if (time_plan(cand[0], &again)) {
            if (again < first_us) first_us = again;
            if (!(best_us < 0.97f * first_us)) { best = 0; best_us = first_us; }
        }
    }
    // second stage: the winner with smaller workgroups.  With a few workgroups per compute unit the number of paths a
    // workgroup takes decides how evenly they spread (measured 5-20 % either way on batches of 2,048 to 8,192 paths, with
    // no rule that the planner could follow), so the measurement decides.
    if (status == SIG_OK && best >= 0 && cand[best].variant == SIG_VARIANT_ON_CHIP) {
        const OnChipKernelInfo *ki = find_on_chip(d, depth, cand[best].prefix_depth);
        const int sizes[3] = {192, 128, 64};
        for (int si = 0; si < 3 && ki && status == SIG_OK && n < (int)(sizeof(cand) / sizeof(cand[0])); ++si) {
            sig_plan_t pl = cand[best];
            if (sizes[si] >= pl.threads) continue;
            pl.threads = sizes[si];
            pl.tile_steps = 0;
            OnChipArgs args{};
            if (!finish_on_chip(ki, ctx->num_cu, B, L, stream_flag, pl, rs, &args)) continue;
            float us = 0.0f;
            if (!time_plan(pl, &us)) continue;
            if (us < 0.97f * best_us) {
                cand[n] = pl;
                best = n++;
                best_us = us;
            }
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (path || out) (void)hipStreamSynchronize(st);
    if (path) (void)hipFree(path);
    if (out) (void)hipFree(out);
    if (status != SIG_OK) return status;
    if (best < 0) return SIG_ERR_HIP;

    TunedPlan entry{B, L, d, depth, stream_flag, cand[best]};
    int slot = -1;
    for (int i = 0; i < ctx->tuned_count; ++i) {
        const TunedPlan &t = ctx->tuned[i];
        if (t.B == B && t.L == L && t.d == d && t.depth == depth && t.stream_flag == stream_flag) slot = i;
    }
    if (slot < 0) {
        const int cap = (int)(sizeof(ctx->tuned) / sizeof(ctx->tuned[0]));
        if (ctx->tuned_count < cap) slot = ctx->tuned_count++;
        else { slot = ctx->tuned_next; ctx->tuned_next = (ctx->tuned_next + 1) % cap; }
    }
    ctx->tuned[slot] = entry;
    if (chosen) *chosen = cand[best];
    if (microseconds) *microseconds = best_us;
    return SIG_OK;
}

int sig_combine(sig_ctx *ctx, const float *a, const float *b, int64_t B, int d, int depth,
                float *out, void *hip_stream)
{
    if (!ctx || B < 0 || d < 1 || depth < 1) return SIG_ERR_INVALID;
    RowShape rs;
    if (depth > kMaxDepth || !make_row_shape(d, depth, &rs)) return SIG_ERR_TOO_LARGE;
    if (B == 0) return SIG_OK;
    if (!a || !b || !out) return SIG_ERR_INVALID;
    hipError_t e = launch_combine_rows(a, rs.D, b, rs.D, out, rs.D, B, rs, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int sig_backward(sig_ctx *ctx, const float *path, int64_t B, int64_t L, int d, int depth, int stream_flag,
                 const float *out, const float *grad_out, float *grad_path, void *hip_stream)
{
    if (!ctx) return SIG_ERR_INVALID;
    RowShape rs;
    int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_OK;
    if (!path || !out || !grad_out || !grad_path) return SIG_ERR_INVALID;
    const bool fits = backward_available(d, depth) && backward_fits(d, depth, L);
    if (backward_available(d, depth)) {
        // few long paths (or paths too long for the LDS of the uncut sweep): the sweep cut in time across workgroups
        const int segs = backward_segments(d, depth, B, L, ctx->num_cu, fits, stream_flag);
        if (segs > 1) {
            const int64_t need = backward_segmented_scratch_floats(d, depth, B, L, segs);
            if (need <= 0 || need > (int64_t)1 << 36) return SIG_ERR_TOO_LARGE;
            rc = ensure_scratch(ctx, (size_t)need * sizeof(float));
            if (rc != SIG_OK) return rc;
            hipError_t es = launch_backward_segmented(path, out, grad_out, grad_path, ctx->scratch, B, L, d, depth, stream_flag,
                                                      segs, ctx->num_cu, (hipStream_t)hip_stream);
            return es == hipSuccess ? SIG_OK : SIG_ERR_HIP;
        }
    }
    if (!fits && !(backward_available(d, depth) && backward_tiles_fit(d, depth))) {
        // no register kernel for this shape: the general sweep
        if (!backward_general_available(d) || B > INT32_MAX) return SIG_ERR_UNSUPPORTED;
        const int64_t need = backward_general_scratch_floats(B, L, rs);
        if (need <= 0 || need > (int64_t)1 << 36) return SIG_ERR_TOO_LARGE;
        rc = ensure_scratch(ctx, (size_t)need * sizeof(float));
        if (rc != SIG_OK) return rc;
        hipError_t eg = launch_backward_general(path, out, grad_out, grad_path, ctx->scratch, B, L, rs, stream_flag,
                                                (hipStream_t)hip_stream);
        return eg == hipSuccess ? SIG_OK : SIG_ERR_HIP;
    }
    const int64_t floats = backward_scratch_floats(d, depth, B, L);
    if (floats > 0) {
        rc = ensure_scratch(ctx, (size_t)floats * sizeof(float));
        if (rc != SIG_OK) return rc;
    }
    hipError_t e = launch_backward(path, out, grad_out, grad_path, floats > 0 ? ctx->scratch : nullptr, B, L, d, depth,
                                   stream_flag, ctx->num_cu, (hipStream_t)hip_stream);
    return e == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int sig_backward_segments(const sig_ctx *ctx, int64_t B, int64_t L, int d, int depth, int stream_flag)
{
    RowShape rs;
    const int rc = check_shape(B, L, d, depth, stream_flag, &rs);
    if (rc != SIG_OK) return -rc;
    if (!backward_available(d, depth)) return backward_general_available(d) ? 0 : -SIG_ERR_UNSUPPORTED;
    const bool fits = backward_fits(d, depth, L);
    if (B > 0) {
        const int segs = backward_segments(d, depth, B, L, ctx ? ctx->num_cu : kDefaultCUs, fits, stream_flag);
        if (segs > 1) return segs;
    }
    return fits || backward_tiles_fit(d, depth) ? 1 : 0;
}

int sig_backward_available(int d, int depth)
{
    return backward_available(d, depth) ? 1 : 0;
}

int sig_on_chip_available(int d, int depth, int prefix_depth)
{
    return find_on_chip(d, depth, prefix_depth) ? 1 : 0;
}

const char *sig_strerror(int status)
{
    switch (status) {
    case SIG_OK: return "ok";
    case SIG_ERR_INVALID: return "invalid argument or plan";
    case SIG_ERR_TOO_LARGE: return "shape too large for the supported index range";
    case SIG_ERR_ALLOC: return "allocation of scratch memory failed";
    case SIG_ERR_HIP: return "a HIP call or kernel launch failed";
    case SIG_ERR_NO_DEVICE: return "no usable HIP device";
    case SIG_ERR_UNSUPPORTED: return "no kernel is compiled for this shape";
    default: return "unknown status";
    }
}

}  // extern "C"

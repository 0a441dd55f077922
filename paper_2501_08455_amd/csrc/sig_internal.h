// Internal declarations shared by the host API and the kernel translation units of libsig.
// Nothing here is part of the C ABI (that is include/sig.h).
#ifndef SIG_INTERNAL_H
#define SIG_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sig.h"

namespace sig {

constexpr int kMaxDepth = 30;        // d^depth must also fit in int32
constexpr int kWave = 64;
constexpr int kMaxLdsBytes = 64 * 1024;  // per-workgroup LDS this library asks for at most
constexpr int kCuLdsBytes = 160 * 1024;  // LDS of one compute unit, shared by its resident workgroups
constexpr int kTileLdsBytes = 19968;     // LDS the increment tile(s) of one workgroup may take (8 workgroups share 160 KB)
constexpr int kFoldTileSteps = 32;       // increments a wavefront of the fold kernel stages at a time
constexpr int kLoaderStage = 8;          // floats of the next tile one thread holds in registers when tiles are pipelined

// Offsets of the levels inside an output row (Eq. 10: level 0 dropped): level n starts at
// d + ... + d^{n-1} and holds d^n floats.
struct RowShape {
    int d;
    int depth;
    int64_t D;                      // row length
    int64_t pow[kMaxDepth + 2];     // pow[n] = d^n
    int64_t off[kMaxDepth + 2];     // off[n] = start of level n (n >= 1), off[depth + 1] = D
};

// returns false if d^depth or D overflow the supported range
bool make_row_shape(int d, int depth, RowShape *rs);

// ---------------------------------------------------------------- HBM-streaming family (any d, depth)
// One workgroup per (path, sub-tree of prefix depth p); the state is the output row itself.
hipError_t launch_hbm_streaming(const float *path, float *out, int64_t B, int64_t L, const RowShape &rs,
                                int p, int stream_flag, int threads, hipStream_t st);

// out[b] = a[b] (x) b[b] on rows of D floats (Eq. 4 with implied level 0 = 1); strides in floats.
hipError_t launch_combine_rows(const float *a, int64_t a_stride, const float *b, int64_t b_stride,
                               float *out, int64_t out_stride, int64_t B, const RowShape &rs,
                               hipStream_t st);

// ---------------------------------------------------------------- level-scan family (d <= 256, depth <= 8)
// The level-by-level formulation of the paper's Section 3.2: one launch per level, each a cumulative sum over time
// of per-step terms built from the lower levels of every prefix, which live in `scratch` (level_scan_scratch_floats
// floats in both modes, one dense [B][L-1][d^m] tensor per level m < depth).
bool level_scan_available(int d, int depth);
int64_t level_scan_scratch_floats(int64_t B, int64_t L, const RowShape &rs, int stream_flag);
// false if the rows of one path cannot be addressed with 32-bit offsets
bool level_scan_fits(int64_t L, const RowShape &rs, int stream_flag);
// time chunks of one (path, parent word) at `level`; forced > 0 overrides the choice (clamped to the path)
int level_scan_chunks(int64_t B, int64_t L, const RowShape &rs, int level, int forced, int cus);
hipError_t launch_level_scan(const float *path, float *out, float *scratch, int64_t B, int64_t L, const RowShape &rs,
                             int stream_flag, int forced_chunks, int cus, hipStream_t st);

// ---------------------------------------------------------------- gradient with respect to the path (compiled (d, depth) only)
bool backward_available(int d, int depth);
// false if even one path per workgroup does not fit the LDS of the uncut sweep (the increments of a whole path are
// staged at once); such paths are walked in tiles by launch_backward (sequential in time, needs scratch)
bool backward_fits(int d, int depth, int64_t L);
// whether a tile of the tiled sweep fits LDS (true for every compiled shape; checked before launching)
bool backward_tiles_fit(int d, int depth);
// device scratch the launch needs (shapes whose lanes per path span several workgroups keep per-slice sums), in floats
int64_t backward_scratch_floats(int d, int depth, int64_t B, int64_t L);
hipError_t launch_backward(const float *path, const float *sig, const float *grad_out, float *grad_path, float *scratch,
                           int64_t B, int64_t L, int d, int depth, int stream_flag, int cus, hipStream_t st);

// d(loss)/dX from per-slice sums of d(loss)/d(increment), part = [B][slices][L-1][d]
hipError_t launch_backward_finish(const float *part, float *grad_path, int64_t B, int64_t L, int d, int slices,
                                  hipStream_t st);

// ---------------------------------------------------------------- gradient cut in time across workgroups
// Time segments the sweep should be cut into (<= 1: do not cut); uncut_fits = backward_fits(d, depth, L)
int backward_segments(int d, int depth, int64_t B, int64_t L, int cus, bool uncut_fits, int stream_flag);
int64_t backward_segmented_scratch_floats(int d, int depth, int64_t B, int64_t L, int segs);
hipError_t launch_backward_segmented(const float *path, const float *sig, const float *grad_out, float *grad_path,
                                     float *scratch, int64_t B, int64_t L, int d, int depth, int stream_flag, int segs,
                                     int cus, hipStream_t st);

// ---------------------------------------------------------------- gradient, any (d <= 256, depth): one workgroup per path
bool backward_general_available(int d);
int64_t backward_general_scratch_floats(int64_t B, int64_t L, const RowShape &rs);
hipError_t launch_backward_general(const float *path, const float *sig, const float *grad_out, float *grad_path,
                                   float *scratch, int64_t B, int64_t L, const RowShape &rs, int stream_flag,
                                   hipStream_t st);

// ---------------------------------------------------------------- on-chip family (compiled (d, depth, p) only)
struct OnChipArgs {
    const float *path;   // [B][L][d]
    float *out;          // final: [B][D]; stream: [B][K][D]
    float *partial;      // [B][segments][D] scratch when segments > 1, else unused
    int64_t B;
    int64_t L;
    int32_t chunks;      // C: time chunks per (path, segment) folded side by side in one workgroup
    int32_t segments;    // W: workgroups per path along time
    int32_t chunk_steps; // T: increments per chunk; segments * chunks * T >= L - 1
    int32_t tile_steps;  // TT: increments per LDS tile
    int32_t threads;     // workgroup size
    int32_t groups;      // (path, segment) pairs per workgroup (1 when a chunk's lanes span several workgroups)
    int32_t row_shift;   // log2 of the padded length of one chunk's stretch of a tile (tile_steps * d floats)
    int32_t resident_workgroups;  // workgroups the device keeps resident at once (persistent kernels); 0: no limit
    int32_t stagger_ticks;  // start delay (100 MHz ticks) per residency slot of the first wave of workgroups; 0: none
    int32_t num_cus;        // compute units of the device
    int32_t cooperative;  // chunks == 1 only: 1 = workgroup-wide tiles with barriers instead of independent wavefronts
    int32_t pipe;         // several tiles per chunk: 1 = the next tile's loads stay in flight in registers while the current
                          // one is consumed (hides the load latency inside one workgroup), 0 = load, barrier, consume
                          // (fewer registers; the other resident workgroups hide the latency)
    int32_t flat_tile;    // 1: the workgroup's paths are whole and adjacent in memory and fit one tile: the tile is a
                          // straight copy of that range (rows of L * d floats), differenced on the way
    int32_t stream_flag;
    int32_t shared_chain; // 1: final mode, one chunk, lanes of a path spanning several workgroups, prefix depth >= 2: the
                          // prefix part of the Horner chains comes from a table in LDS that a few lanes of the workgroup
                          // fill once (the whole (path, segment) is one tile: tile_steps = chunk_steps)
};

// The fold that shares the prefix part of the Horner chains (sig_shared_chain_kernel) takes the `steps` increments of a
// (path, segment) as one tile.  LDS floats of a workgroup: the increments [steps][d], the table [steps][nq][depth - p + 1]
// with nq the prefixes of length p - 1 the words of one workgroup can have, the chunk totals of the table's running sums
// (one float per thread and level at most), and the totals of the words at the segment's end.
constexpr int64_t shared_chain_round4(int64_t x) { return (x + 3) / 4 * 4; }
constexpr int64_t shared_chain_prefixes(int d, int threads) { return (threads - 1) / d + 2; }
constexpr int64_t shared_chain_lds_floats(int d, int depth, int p, int threads, int64_t steps)
{
    const int64_t nq = shared_chain_prefixes(d, threads);
    return shared_chain_round4(steps * d) + shared_chain_round4(steps * nq * (depth - p + 1)) + (p - 1) * shared_chain_round4(threads) +
           shared_chain_round4((p - 1) * nq);
}
// whether a segment of `steps` increments fits: 52 KB of LDS (three workgroups per compute unit), a table builder per
// prefix among the threads, and at most 16 steps per builder (prefixes take a power of two of thread slots, the chunks of
// steps the rest)
constexpr bool shared_chain_fits(int d, int depth, int p, int threads, int64_t steps)
{
    const int64_t nq = shared_chain_prefixes(d, threads);
    int64_t slots = 1;
    while (slots < nq) slots *= 2;
    return steps >= 1 && slots <= threads && (threads / slots) * 16 >= steps &&
           shared_chain_lds_floats(d, depth, p, threads, steps) * (int64_t)sizeof(float) <= 52 * 1024;
}

struct OnChipKernelInfo {
    int d, depth, p;
    int lanes_per_chunk;                       // Q = d^p
    int state_floats;                          // registers of state per lane
    int row_floats;                            // LDS floats per staged increment (= d)
    hipError_t (*launch)(const OnChipArgs &, hipStream_t);
    // LDS bytes the launch needs for these arguments (for validation before launching)
    int64_t (*lds_bytes)(const OnChipArgs &);
    // out[b] = product over the `segments` partial rows of path b (second launch when segments > 1)
    hipError_t (*join)(const float *partial, float *out, int64_t B, int segments, hipStream_t);
};

// Work items of an on-chip launch with Q = d^p lanes per (path, chunk): one per slice of a path's lanes when they exceed
// a workgroup, else one per `groups` (path, segment) pairs.  <= 0: invalid arguments.
inline int64_t on_chip_work_items(int Q, const OnChipArgs &A)
{
    const int64_t ngroups = A.B * A.segments;
    if (Q > A.threads) {
        if (A.chunks != 1 || A.groups != 1) return -1;
        return ngroups * ((Q + A.threads - 1) / A.threads);
    }
    if (A.groups < 1) return -1;
    return (ngroups + A.groups - 1) / A.groups;
}
// Workgroups launched: one per work item, except that the kernels with independent wavefronts launch no more workgroups
// than stay resident and let each walk the same number of items.
inline int64_t on_chip_workgroups(int Q, const OnChipArgs &A)
{
    int64_t grid = on_chip_work_items(Q, A);
    if (A.chunks == 1 && !A.cooperative && grid > 0) {
        int64_t resident = A.resident_workgroups > 0 ? A.resident_workgroups : grid;
        if (resident > grid) resident = grid;
        const int64_t rounds = (grid + resident - 1) / resident;
        grid = (grid + rounds - 1) / rounds;
    }
    return grid;
}

// table of compiled on-chip kernels; terminated by an entry with launch == nullptr
// The compiled kernels live in several translation units (so that they build in parallel); sub-table i ends
// with an entry whose launch pointer is null, and on_chip_subtable(i) is null past the last sub-table.  Entries
// of one (d, depth) are adjacent and ordered by increasing prefix depth.
const OnChipKernelInfo *on_chip_subtable(int i);
const OnChipKernelInfo *on_chip_table_base();      // sub-tables 0 .. 5, one translation unit each
const OnChipKernelInfo *on_chip_table_depth2();
const OnChipKernelInfo *on_chip_table_depth3();
const OnChipKernelInfo *on_chip_table_depth4();
const OnChipKernelInfo *on_chip_table_depth56();
const OnChipKernelInfo *on_chip_table_odd();
const OnChipKernelInfo *find_on_chip(int d, int depth, int p);

}  // namespace sig
#endif

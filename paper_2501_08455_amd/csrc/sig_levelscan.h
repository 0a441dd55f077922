// Kernels of the level-scan family and their launch tables, shared by the two translation units that instantiate them
// (sig_levelscan.hip: the launches that write one level; sig_levelscan_rows.hip: the stream mode's top-level launch,
// which writes whole output rows).  The method is described at the top of sig_levelscan.hip.
#ifndef SIG_LEVELSCAN_H_
#define SIG_LEVELSCAN_H_

#include "sig_internal.h"

namespace sig {
namespace levelscan {


constexpr int kLsThreads = 256;
constexpr int kLsTileFloats = 12288; // most LDS floats the increment tile of one workgroup may take
constexpr int kLsBatch = 4;          // steps whose lower-level loads are in flight together (deeper did not measure faster)
constexpr int kLsMaxChunks = 64;     // so that a tile of one batch pair per (path, chunk) always fits
constexpr int kLsMaxD = 256;         // up to 10 channels are template parameters, more are a run-time value
constexpr int kLsMaxLevel = 8;

struct LevelScanArgs {
    const float *path;               // [B][L][d]
    const float *lo[kLsMaxLevel];    // lo[m], m = 1 .. n-1: level m of prefix (b, j) at lo[m] + (b * K + j) * lo_stride[m]
    int32_t lo_stride[kLsMaxLevel];  // K * lo_stride[m] fits 31 bits (checked by the host)
    float *hi;                       // level n of prefix (b, j) goes to hi + (b * K + j) * hi_stride; null: not stored
    float *fin;                      // level n of the whole path goes to fin + b * fin_stride; null: not stored
    float *cat;                      // stream mode, top level: level m < n of prefix (b, j) is copied to
    int32_t cat_off[kLsMaxLevel];    //   cat + (b * K + j) * hi_stride + cat_off[m]; null: no copies
    int64_t hi_stride, fin_stride;
    int64_t B, L;
    int32_t d;           // channels (the kernels for d <= 10 have it as a template parameter as well)
    int32_t items;       // work items of one path: parent words P = d^{n-1}, times the blocks of children per parent
    int32_t pw;          // items per workgroup and chunk
    int32_t wblocks;     // ceil(items / pw)
    int32_t chunks;      // C
    int32_t groups;      // G paths per workgroup; G * C * pw <= blockDim.x
    int32_t chunk_steps; // T = ceil(K / C)
    int32_t tile_steps;  // TT <= T; a tile holds TT rounded up to whole batches of steps, G * C * that * d <= kLsTileFloats
    int32_t sub_shift;   // the loader gives 2^sub_shift adjacent threads to one (path, chunk) stretch of a tile
};

struct No { static constexpr bool value = false; };   // compile-time switches of the sweep
struct Yes { static constexpr bool value = true; };

// VEC floats per store instruction (the host picks the widest the alignment of the rows allows)
template <int d, int VEC>
__device__ __forceinline__ void store_children(float *dst, const float (&acc)[d])
{
    static_assert(d % VEC == 0, "store width must divide the number of children");
    if constexpr (VEC == 4) {
#pragma unroll
        for (int q = 0; q < d / 4; ++q)
            *reinterpret_cast<float4 *>(dst + 4 * q) = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    } else if constexpr (VEC == 2) {
#pragma unroll
        for (int q = 0; q < d / 2; ++q) *reinterpret_cast<float2 *>(dst + 2 * q) = make_float2(acc[2 * q], acc[2 * q + 1]);
    } else {
#pragma unroll
        for (int a = 0; a < d; ++a) dst[a] = acc[a];
    }
}

// run-time d: a lane holds kWideBlock children starting at child `first`; children past the last one repeat it
// (same value to the same address), so that every lane issues the same stores
constexpr int kWideBlock = 4;
__device__ __forceinline__ void store_block(float *parent_row, int first, int d, const float (&acc)[kWideBlock])
{
#pragma unroll
    for (int a = 0; a < kWideBlock; ++a) {
        const int ch = first + a < d ? first + a : d - 1;
        parent_row[ch] = acc[a];
    }
}

// DT > 0: d = DT at compile time, a lane owns all d children of its parent word.  DT == 0: d at run time (more than
// 10 channels), a lane owns a block of kWideBlock children, the lanes of one parent are adjacent and recompute its chain.
// CAT: the launch of the top level in stream mode, which also copies the lower levels into the output rows (a kernel of
// its own: compiled into the others, the copies cost the deep levels four registers and with them a wavefront per SIMD)
template <int DT, int n, int VEC, bool CAT>
__global__ __launch_bounds__(kLsThreads) void sig_level_scan_kernel(LevelScanArgs A)
{
    static_assert(n >= 2, "level 1 has its own kernel");
    constexpr int M = n - 1;  // lower levels on the chain
    constexpr int DB = DT > 0 ? DT : kWideBlock;             // children a lane owns
    const int d = DT > 0 ? DT : A.d;
    const int NB = DT > 0 ? 1 : (d + DB - 1) / DB;           // lanes per parent word
    extern __shared__ float ls_smem[];
    const int tid = threadIdx.x;
    const int PW = A.pw, C = A.chunks, G = A.groups, T = A.chunk_steps, TT = A.tile_steps;
    const int TP = (TT + 2 * kLsBatch - 1) / (2 * kLsBatch) * (2 * kLsBatch);  // stretch of a tile, whole batches
    float *tile = ls_smem;                        // [G * C][TP * d]
    float *tot = ls_smem + G * C * TP * d;        // [G][C][pw][DB], used when C > 1

    const int64_t K = A.L - 1;
    const int wl = tid % PW;
    const int c = (tid / PW) % C;
    const int g = tid / (PW * C);
    const int64_t b0 = (int64_t)(blockIdx.x / A.wblocks) * G;
    const int64_t b = b0 + g;
    const int item = (int)(blockIdx.x % A.wblocks) * PW + wl;
    const bool lane_ok = g < G && b < A.B && item < A.items;
    const int w = DT > 0 ? item : item / NB;                 // parent word
    const int first_child = DT > 0 ? 0 : (item - w * NB) * DB;

    // Addresses are a workgroup-uniform base plus a 32-bit lane offset (the host checks that the rows of the
    // workgroup's paths stay below 2^30 floats and the strides below 2^24, so offsets are one 24-bit multiply-add).
    // prefixes of the parent word: w_{1:m} as a number in base d addresses level m; let[m-1] = w_m
    const int K32 = (int)K;
    const float *base[M];
    uint32_t lane_off[M];
    int stride[M], let[M];
    float rc[M];
    {
        int rest = lane_ok ? w : 0;
#pragma unroll
        for (int m = M; m >= 1; --m) {
            stride[m - 1] = A.lo_stride[m];
            base[m - 1] = A.lo[m] + b0 * K * A.lo_stride[m];
            lane_off[m - 1] = (uint32_t)(lane_ok ? g : 0) * (uint32_t)(K32 * A.lo_stride[m]) + (uint32_t)rest;
            let[m - 1] = rest % d;
            rest /= d;
            rc[m - 1] = 1.0f / (float)(n - m + 1);
        }
    }
    const int j_begin = c * T;
    const int j_end = (j_begin + T < K32) ? j_begin + T : K32;   // may be <= j_begin for trailing chunks
    const int hi_stride = (int)A.hi_stride;
    // Copies of the lower levels into the output rows: a lane writes the values it has loaded for its chain.  Of the
    // lanes that share a prefix of their parent words, which all hold its value, the first one writes it (a store
    // instruction whose lanes hit one address several times measured 30 % slower over the whole launch); a row the
    // fetch was clamped to is written once more with what was read from it.
    float *cat_base = nullptr;
    uint32_t cat_lane[CAT ? M : 1];
    bool cat_own[CAT ? M : 1];
    if constexpr (CAT) {
        cat_base = A.cat + b0 * K * A.hi_stride;
        int rest = lane_ok ? w : 0;
        bool first_of_prefix = lane_ok && first_child == 0;
#pragma unroll
        for (int m = M; m >= 1; --m) {
            cat_lane[m - 1] = (uint32_t)(lane_ok ? g : 0) * (uint32_t)(K32 * hi_stride) + (uint32_t)A.cat_off[m] + (uint32_t)rest;
            cat_own[m - 1] = first_of_prefix;
            first_of_prefix = first_of_prefix && rest % d == 0;
            rest /= d;
        }
    }
    float *hi_base = A.hi ? A.hi + b0 * K * A.hi_stride : nullptr;
    const uint32_t hi_off = (uint32_t)(lane_ok ? g : 0) * (uint32_t)(K32 * hi_stride) + (uint32_t)(lane_ok ? w : 0) * d;
    const float *my_tile = tile + (size_t)((g < G ? g : 0) * C + c) * TP * d;
    const int tiles = (T + TT - 1) / TT;

    // children of this lane inside an increment (run-time d: clamped to the last channel)
    int child[DB];
#pragma unroll
    for (int a = 0; a < DB; ++a) child[a] = first_child + a < d ? first_child + a : d - 1;
    float acc[DB];
#pragma unroll
    for (int a = 0; a < DB; ++a) acc[a] = 0.0f;
    auto store_acc = [&](float *parent_row) {
        if constexpr (DT > 0) store_children<DB, VEC>(parent_row, acc);
        else store_block(parent_row, first_child, d, acc);
    };

    // differenced increments of tile i: the stretch of every (path, chunk) of the workgroup is a straight run of
    // the path, taken by 2^sub_shift adjacent threads; the rest of the stretch (past the end of a chunk, and the
    // padding up to a whole number of batches) is zero
    auto load_tile = [&](int i) {
        const int sub = tid >> A.sub_shift, lane_in = tid & ((1 << A.sub_shift) - 1);
        const int per_pass = blockDim.x >> A.sub_shift;
        for (int pair = sub; pair < G * C; pair += per_pass) {
            const int cc = pair % C;
            const int64_t bb = b0 + pair / C;
            const int64_t j0 = (int64_t)cc * T + (int64_t)i * TT;
            int64_t jend = (int64_t)(cc + 1) * T;
            if (jend > K) jend = K;
            int64_t steps = jend - j0;
            if (steps > TT) steps = TT;
            const int len = (bb < A.B && steps > 0) ? (int)steps * d : 0;
            const float *x = A.path + (bb < A.B ? (bb * A.L + j0) * d : 0);
            float *dst = tile + (size_t)pair * TP * d;
            for (int e = lane_in; e < TP * d; e += 1 << A.sub_shift) dst[e] = e < len ? x[e + d] - x[e] : 0.0f;
        }
    };

    // Lower-level coefficients of the prefix before step jt + t.  Always loaded, from a row clamped into the path, so
    // that no load sits in a divergent branch (the wait counters then let a batch stay in flight behind the one
    // being consumed); steps outside the chunk are masked when the values are used.
    const int last_row = K32 >= 2 ? K32 - 2 : 0;
    auto fetch = [&](int jt, int t, float (&s)[M]) {
        int jj = jt + t - 1;
        jj = jj < 0 ? 0 : jj;
        jj = jj > last_row ? last_row : jj;
#pragma unroll
        for (int m = 0; m < M; ++m) s[m] = base[m][lane_off[m] + __umul24((uint32_t)jj, (uint32_t)stride[m])];
    };
    // n_on: steps of this tile that belong to the lane's chunk; `first` is set when the tile starts at the first
    // step of the path, whose prefix is the empty path (all lower levels zero).  A step outside the chunk adds
    // nothing; when levels are stored it stores the unchanged sum once more over the row of the chunk's last step, so
    // that every step issues the same memory operations and the wait counters stay exact.
    const bool has_work = lane_ok && j_begin < j_end;
    auto step = [&](int jt, int t, int n_on, bool first, const float (&s)[M], auto emit_c, auto cat_c) {
        if constexpr (decltype(cat_c)::value) {
            int jj = jt + t - 1;      // the row `fetch` read s from
            jj = jj < 0 ? 0 : jj;
            jj = jj > last_row ? last_row : jj;
#pragma unroll
            for (int m = 0; m < M; ++m)
                if (cat_own[m]) cat_base[cat_lane[m] + __umul24((uint32_t)jj, (uint32_t)hi_stride)] = s[m];
        }
        const float *dx = my_tile + t * d;
        float h = 1.0f;
#pragma unroll
        for (int m = 0; m < M; ++m) h = fmaf(h, dx[let[m]] * rc[m], first ? 0.0f : s[m]);
        h = t < n_on ? h : 0.0f;
#pragma unroll
        for (int a = 0; a < DB; ++a) acc[a] = fmaf(h, dx[DT > 0 ? a : child[a]], acc[a]);
        if constexpr (decltype(emit_c)::value) {
            int row = jt + t;
            row = row < j_end ? row : j_end - 1;
            store_acc(hi_base + (hi_off + __umul24((uint32_t)row, (uint32_t)hi_stride)));
        }
    };

    auto sweep = [&](auto emit_c, auto cat_c, bool reload) {
        for (int i = 0; i < tiles; ++i) {
            if (reload) {
                __syncthreads();   // the previous tile has been consumed
                load_tile(i);
                __syncthreads();
            }
            if (!has_work) continue;
            const int jt = j_begin + i * TT;
            int n_on = j_end - jt;
            n_on = n_on > TT ? TT : n_on;
            float ping[kLsBatch][M], pong[kLsBatch][M];
#pragma unroll
            for (int u = 0; u < kLsBatch; ++u) fetch(jt, u, ping[u]);
            for (int t0 = 0; t0 < TP; t0 += 2 * kLsBatch) {
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u) fetch(jt, t0 + kLsBatch + u, pong[u]);
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u) step(jt, t0 + u, n_on, u == 0 && jt + t0 == 0, ping[u], emit_c, cat_c);
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u) fetch(jt, t0 + 2 * kLsBatch + u, ping[u]);
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u) step(jt, t0 + kLsBatch + u, n_on, false, pong[u], emit_c, cat_c);
            }
        }
    };
    const bool one_tile = tiles == 1;
    if (one_tile) {
        load_tile(0);
        __syncthreads();
    }
    if (C > 1) {
        sweep(No{}, No{}, !one_tile);
        float *mine = tot + (size_t)tid * DB;
        if (tid < G * C * PW) {
#pragma unroll
            for (int a = 0; a < DB; ++a) mine[a] = acc[a];
        }
        __syncthreads();
        // Without per-step stores the sum of all chunks is the result and the lane of chunk 0 writes it; otherwise
        // a lane starts its second pass from the sum of the chunks before its own, earliest first.
        if (!A.hi) {
            if (lane_ok && c == 0 && A.fin) {
#pragma unroll
                for (int a = 0; a < DB; ++a) acc[a] = 0.0f;
                for (int cc = 0; cc < C; ++cc) {
                    const float *part = tot + (size_t)((g * C + cc) * PW + wl) * DB;
#pragma unroll
                    for (int a = 0; a < DB; ++a) acc[a] += part[a];
                }
                store_acc(A.fin + b * A.fin_stride + (int64_t)w * d);
            }
            return;
        }
#pragma unroll
        for (int a = 0; a < DB; ++a) acc[a] = 0.0f;
        if (lane_ok) {
            for (int cc = 0; cc < c; ++cc) {
                const float *part = tot + (size_t)((g * C + cc) * PW + wl) * DB;
#pragma unroll
                for (int a = 0; a < DB; ++a) acc[a] += part[a];
            }
        }
    }
    if constexpr (CAT) {
        sweep(Yes{}, Yes{}, !one_tile);     // (the host sets cat only together with hi)
    } else {
        if (A.hi) sweep(Yes{}, No{}, !one_tile);
        else sweep(No{}, No{}, !one_tile);
    }
    // the chunk that holds the last step also holds the level of the whole path
    if (lane_ok && A.fin && j_begin < K32 && j_end == K32) store_acc(A.fin + b * A.fin_stride + (int64_t)w * d);
    // ... and copies the lower levels of the last row, which no step reads
    if constexpr (CAT) {
        if (lane_ok && j_begin < K32 && j_end == K32) {
#pragma unroll
            for (int m = 0; m < M; ++m)
                if (cat_own[m])
                    cat_base[cat_lane[m] + __umul24((uint32_t)(K32 - 1), (uint32_t)hi_stride)] =
                        base[m][lane_off[m] + __umul24((uint32_t)(K32 - 1), (uint32_t)stride[m])];
        }
    }
}

template <int d, int n, bool CAT>
hipError_t launch_one(const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    constexpr int kNatural = d == 0 ? 1 : (d % 4 == 0 ? 4 : (d % 2 == 0 ? 2 : 1));
    if ((A.cat != nullptr) != CAT || (CAT && !A.hi)) return hipErrorInvalidValue;
    if (kNatural > 1 && vec >= kNatural)
        hipLaunchKernelGGL((sig_level_scan_kernel<d, n, kNatural, CAT>), dim3(blocks), dim3(threads), lds, st, A);
    else
        hipLaunchKernelGGL((sig_level_scan_kernel<d, n, 1, CAT>), dim3(blocks), dim3(threads), lds, st, A);
    return hipGetLastError();
}

template <int d, bool CAT>
hipError_t launch_level(int n, const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    switch (n) {
    case 2: return launch_one<d, 2, CAT>(A, vec, blocks, threads, lds, st);
    case 3: return launch_one<d, 3, CAT>(A, vec, blocks, threads, lds, st);
    case 4: return launch_one<d, 4, CAT>(A, vec, blocks, threads, lds, st);
    case 5: return launch_one<d, 5, CAT>(A, vec, blocks, threads, lds, st);
    case 6: return launch_one<d, 6, CAT>(A, vec, blocks, threads, lds, st);
    case 7: return launch_one<d, 7, CAT>(A, vec, blocks, threads, lds, st);
    case 8: return launch_one<d, 8, CAT>(A, vec, blocks, threads, lds, st);
    default: return hipErrorInvalidValue;
    }
}

template <bool CAT>
hipError_t launch_level_d(int d, int n, const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    switch (d) {
    case 1: return launch_level<1, CAT>(n, A, vec, blocks, threads, lds, st);
    case 2: return launch_level<2, CAT>(n, A, vec, blocks, threads, lds, st);
    case 3: return launch_level<3, CAT>(n, A, vec, blocks, threads, lds, st);
    case 4: return launch_level<4, CAT>(n, A, vec, blocks, threads, lds, st);
    case 5: return launch_level<5, CAT>(n, A, vec, blocks, threads, lds, st);
    case 6: return launch_level<6, CAT>(n, A, vec, blocks, threads, lds, st);
    case 7: return launch_level<7, CAT>(n, A, vec, blocks, threads, lds, st);
    case 8: return launch_level<8, CAT>(n, A, vec, blocks, threads, lds, st);
    case 9: return launch_level<9, CAT>(n, A, vec, blocks, threads, lds, st);
    case 10: return launch_level<10, CAT>(n, A, vec, blocks, threads, lds, st);
    default: return launch_level<0, CAT>(n, A, 1, blocks, threads, lds, st);   // run-time d
    }
}


// the stream mode's top-level launch (defined in sig_levelscan_rows.hip)
hipError_t launch_rows_level(int d, int n, const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st);

}  // namespace levelscan
}  // namespace sig

#endif  // SIG_LEVELSCAN_H_

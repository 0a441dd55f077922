// Level-scan family: the level-by-level formulation of the paper's Section 3.2 (Eqs. 6-10), one launch per level.
//
// Section 3.2 replaces the fold over time by one cumulative sum per level: level n of every prefix signature is
// the running sum over the steps of a per-step term that needs only the LOWER levels of the prefix before the
// step.  In the reading that agrees with Eq. 3 (S on the left, exclusive prefix, tensor powers over factorials):
//     S_n(j) = sum_{i <= j} T_n(i),    T_n(i) = sum_{m=0}^{n-1} S_m(i-1) (x) dX_i^{(x)(n-m)} / (n-m)!.
// For one word w.a (parent w of length n-1, last letter a) the inner sum is a Horner chain along the prefixes
// of w, exactly the chain of the fused step:
//     g_0 = 1,  g_m = S_m(i-1)[w_{1:m}] + g_{m-1} * dX_i[w_m] / (n-m+1)   (m = 1 .. n-1),   T_n(i)[w.a] = g_{n-1} * dX_i[a],
// so a term costs n-1 loads of lower-level coefficients, n-1+d FMAs and touches no other word.  The lower levels
// of every prefix must therefore be in memory (the intermediates of shape (B, L-1, d^m) the paper names as its
// memory cost): one dense scratch tensor per level below the top one, [B][L-1][d^m], as in the paper.  In stream
// mode the launch of the top level also writes the lower levels it reads into the output rows (the concatenation
// of Eq. 10), so that every byte of a row is written by one launch and every lower level is read from a dense
// tensor: when the lower levels lived inside the rows, a 16-byte read at the start of a 1,360-byte row cost a
// whole 64-byte fetch, and the launches fetched 2.7 times what they used.
//
// Mapping.  Level 1 is the running sum of the increments, which telescopes to X_{j+1} - X_0: one elementwise
// launch.  Launch n >= 2 computes level n from levels 1 .. n-1.  A lane owns one parent word w (its d children are
// adjacent floats of the level) and one time chunk; lanes of a wavefront take consecutive parents, so the loads of
// S_{n-1}(i-1)[w] and the stores of S_n(i)[w.*] of a wavefront are contiguous.  The increments of the workgroup's
// paths are differenced on the way into an LDS tile; a lane reads dX_i[.] (the same address across the lanes
// of a path: a broadcast) and dX_i[w_m] (a gather inside d adjacent floats) from there.  Time is parallel as in the
// paper: the terms of different steps are independent, and the cumulative sum is a two-pass scan of plain vector
// additions over the C time chunks of a workgroup (pass 1: chunk totals into LDS; exclusive prefix in a fixed order;
// pass 2: recompute the terms from the carry-in and store every step).  The top level of the final mode needs no
// second pass.  C falls to 1 once B * d^{n-1} alone fills the chip.
//
// Traffic per path and step in floats: level n reads the n-1 lower levels at its parents' prefixes (d^{n-1} +
// d^{n-2} + ... distinct floats, twice when C > 1) and writes d^n; over all levels that is about
// 2 * (D - d^N) * (1 + 1 / (d - 1)) moved through scratch, plus the D floats of a row written once in stream mode.
#include "sig_internal.h"

namespace sig {

namespace {

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

// Level 1: S_1(j) = X_{j+1} - X_0, one thread per float of the level.
__global__ __launch_bounds__(kLsThreads) void sig_level_one_kernel(const float *path, float *hi, int64_t hi_stride,
                                                                   float *fin, int64_t fin_stride, int64_t B,
                                                                   int64_t L, int d)
{
    const int64_t K = L - 1;
    const int64_t per_path = K * d;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= B * per_path) return;
    const int64_t b = e / per_path;
    const int64_t r = e - b * per_path;
    const int64_t j = r / d;
    const int a = (int)(r - j * d);
    const float *x = path + b * L * d;
    const float v = x[d + r] - x[a];
    if (hi) hi[(b * K + j) * hi_stride + a] = v;
    if (fin && j == K - 1) fin[b * fin_stride + a] = v;
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

template <int d, int n>
hipError_t launch_one(const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    constexpr int kNatural = d == 0 ? 1 : (d % 4 == 0 ? 4 : (d % 2 == 0 ? 2 : 1));
    if (A.cat && !A.hi) return hipErrorInvalidValue;
    const bool wide = kNatural > 1 && vec >= kNatural;
    if (A.cat) {
        if (wide) hipLaunchKernelGGL((sig_level_scan_kernel<d, n, kNatural, true>), dim3(blocks), dim3(threads), lds, st, A);
        else hipLaunchKernelGGL((sig_level_scan_kernel<d, n, 1, true>), dim3(blocks), dim3(threads), lds, st, A);
    } else {
        if (wide) hipLaunchKernelGGL((sig_level_scan_kernel<d, n, kNatural, false>), dim3(blocks), dim3(threads), lds, st, A);
        else hipLaunchKernelGGL((sig_level_scan_kernel<d, n, 1, false>), dim3(blocks), dim3(threads), lds, st, A);
    }
    return hipGetLastError();
}

template <int d>
hipError_t launch_level(int n, const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    switch (n) {
    case 2: return launch_one<d, 2>(A, vec, blocks, threads, lds, st);
    case 3: return launch_one<d, 3>(A, vec, blocks, threads, lds, st);
    case 4: return launch_one<d, 4>(A, vec, blocks, threads, lds, st);
    case 5: return launch_one<d, 5>(A, vec, blocks, threads, lds, st);
    case 6: return launch_one<d, 6>(A, vec, blocks, threads, lds, st);
    case 7: return launch_one<d, 7>(A, vec, blocks, threads, lds, st);
    case 8: return launch_one<d, 8>(A, vec, blocks, threads, lds, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_level_d(int d, int n, const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    switch (d) {
    case 1: return launch_level<1>(n, A, vec, blocks, threads, lds, st);
    case 2: return launch_level<2>(n, A, vec, blocks, threads, lds, st);
    case 3: return launch_level<3>(n, A, vec, blocks, threads, lds, st);
    case 4: return launch_level<4>(n, A, vec, blocks, threads, lds, st);
    case 5: return launch_level<5>(n, A, vec, blocks, threads, lds, st);
    case 6: return launch_level<6>(n, A, vec, blocks, threads, lds, st);
    case 7: return launch_level<7>(n, A, vec, blocks, threads, lds, st);
    case 8: return launch_level<8>(n, A, vec, blocks, threads, lds, st);
    case 9: return launch_level<9>(n, A, vec, blocks, threads, lds, st);
    case 10: return launch_level<10>(n, A, vec, blocks, threads, lds, st);
    default: return launch_level<0>(n, A, 1, blocks, threads, lds, st);   // run-time d
    }
}

int floor_pow2(int64_t v)
{
    int p = 1;
    while ((int64_t)p * 2 <= v) p *= 2;
    return p;
}

// widest vector store (floats) that base + k * stride keeps aligned for every k
int store_width(const void *base, int64_t stride)
{
    if (!base) return 4;
    const uintptr_t p = reinterpret_cast<uintptr_t>(base);
    if (p % 16 == 0 && stride % 4 == 0) return 4;
    if (p % 8 == 0 && stride % 2 == 0) return 2;
    return 1;
}

}  // namespace

bool level_scan_available(int d, int depth) { return d >= 1 && d <= kLsMaxD && depth >= 1 && depth <= kLsMaxLevel; }

int64_t level_scan_scratch_floats(int64_t B, int64_t L, const RowShape &rs, int stream_flag)
{
    (void)stream_flag;   // both modes keep the levels below the top one in dense tensors
    if (rs.depth == 1) return 0;
    return B * (L - 1) * (rs.D - rs.pow[rs.depth]);
}

bool level_scan_fits(int64_t L, const RowShape &rs, int stream_flag)
{
    // a lane addresses the rows of its workgroup's paths with 32-bit offsets built by 24-bit multiplies; when one
    // path exceeds 2^22 floats a workgroup takes a single path (see launch_level_scan)
    const int64_t widest = stream_flag ? rs.D : (rs.depth > 1 ? rs.pow[rs.depth - 1] : 1);
    return L - 1 < (1 << 24) && widest < (1 << 24) && (L - 1) * widest < ((int64_t)1 << 30);
}

int level_scan_chunks(int64_t B, int64_t L, const RowShape &rs, int level, int forced, int cus)
{
    const int64_t K = L - 1;
    int64_t C;
    if (forced > 0) {
        C = forced;
    } else {
        // enough lanes for four wavefronts on every SIMD, chunks of at least eight steps
        const int64_t want = (int64_t)cus * 4 * 4 * kWave;
        const int64_t items = B * rs.pow[level - 1];
        C = floor_pow2((want + items - 1) / items);
        if (C > K / 8) C = floor_pow2(K / 8 > 0 ? K / 8 : 1);
    }
    if (C > K) C = K;
    if (C > kLsMaxChunks) C = kLsMaxChunks;
    if (C < 1) C = 1;
    return (int)C;
}

hipError_t launch_level_scan(const float *path, float *out, float *scratch, int64_t B, int64_t L, const RowShape &rs,
                             int stream_flag, int forced_chunks, int cus, hipStream_t st)
{
    if (!level_scan_available(rs.d, rs.depth) || !level_scan_fits(L, rs, stream_flag)) return hipErrorInvalidValue;
    const int d = rs.d, N = rs.depth;
    const int64_t K = L - 1;
    // where level m of every prefix lives: the dense scratch tensor of the level; the top level of the stream mode
    // goes straight into the output rows
    auto level_base = [&](int m) { return (stream_flag && m == N) ? out + rs.off[m] : scratch + B * K * rs.off[m]; };
    auto level_stride = [&](int m) { return (stream_flag && m == N) ? rs.D : rs.pow[m]; };
    for (int n = 1; n <= N; ++n) {
        float *hi = (stream_flag || n < N) ? level_base(n) : nullptr;
        float *fin = stream_flag ? nullptr : out + rs.off[n];
        const int64_t hi_stride = level_stride(n), fin_stride = rs.D;
        if (n == 1) {
            const int64_t total = B * K * d;
            const int64_t blocks = (total + kLsThreads - 1) / kLsThreads;
            if (blocks > INT32_MAX) return hipErrorInvalidValue;
            hipLaunchKernelGGL(sig_level_one_kernel, dim3((unsigned)blocks), dim3(kLsThreads), 0, st, path, hi, hi_stride,
                               fin, fin_stride, B, L, d);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            continue;
        }
        LevelScanArgs A{};
        A.path = path;
        A.B = B;
        A.L = L;
        for (int m = 1; m < n; ++m) {
            A.lo[m] = level_base(m);
            A.lo_stride[m] = (int32_t)level_stride(m);
        }
        A.hi = hi;
        A.hi_stride = hi_stride;
        A.fin = fin;
        A.fin_stride = fin_stride;
        if (stream_flag && n == N) {
            A.cat = out;
            for (int m = 1; m < n; ++m) A.cat_off[m] = (int32_t)rs.off[m];
        }
        const int vh = store_width(hi, hi_stride), vf = store_width(fin, fin_stride);
        const int vec = vh < vf ? vh : vf;
        // work items of a path: one per parent word, or (more than 10 channels) one per block of four children
        const int64_t P = rs.pow[n - 1] * (d <= 10 ? 1 : (d + kWideBlock - 1) / kWideBlock);
        if (P > INT32_MAX) return hipErrorInvalidValue;
        const int per_item = d <= 10 ? d : kWideBlock;
        int C = level_scan_chunks(B, L, rs, n, forced_chunks, cus);
        constexpr int kPair = 2 * kLsBatch;
        int64_t PW, G;
        for (;;) {
            PW = kLsThreads / C;
            if (PW > P) PW = P;
            G = kLsThreads / (PW * C);
            if (G > B) G = B;
            // 32-bit offsets inside the rows of a workgroup's paths
            const int64_t widest = stream_flag ? rs.D : rs.pow[n < N ? n : n - 1];
            while (G > 1 && G * K * widest >= ((int64_t)1 << 30)) --G;
            // the increment tile holds at least one pair of batches for every (path, chunk) of the workgroup
            const int64_t by_tile = kLsTileFloats / ((int64_t)C * d * kPair);
            if (by_tile >= 1) {
                if (G > by_tile) G = by_tile;
                break;
            }
            C /= 2;   // many channels: fewer chunks (C = 1 always fits: d <= 256)
        }
        const int T = (int)((K + C - 1) / C);
        int64_t TT = kLsTileFloats / (G * C * d) / kPair * kPair;   // whole batch pairs
        if (TT > T) TT = T;
        if (TT < 1) return hipErrorInvalidValue;
        const int64_t TP = (TT + kPair - 1) / kPair * kPair;
        const int64_t wblocks = (P + PW - 1) / PW;
        const int64_t blocks = wblocks * ((B + G - 1) / G);
        if (blocks > INT32_MAX) return hipErrorInvalidValue;
        A.d = d;
        A.items = (int32_t)P;
        A.pw = (int32_t)PW;
        A.wblocks = (int32_t)wblocks;
        A.chunks = C;
        A.groups = (int32_t)G;
        A.chunk_steps = T;
        A.tile_steps = (int32_t)TT;
        int shift = 0;
        while (shift < 6 && (1 << shift) < TP * d) ++shift;
        A.sub_shift = shift;
        const int used = (int)(G * C * PW);
        const int threads = (used + kWave - 1) / kWave * kWave;
        const size_t lds = (size_t)(G * C * TP * d + (C > 1 ? threads * per_item : 0)) * sizeof(float);
        hipError_t e = launch_level_d(d, n, A, vec, (int)blocks, threads, lds, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sig

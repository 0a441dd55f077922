// Level-scan family: the level-by-level formulation of the paper's Section 2.2 (Eqs. 6-10), one launch per level.
//
// Section 2.2 replaces the fold over time by one cumulative sum per level: level n of every prefix signature is
// the running sum over the steps of a per-step term that needs only the LOWER levels of the prefix before the
// step.  In the reading that agrees with Eq. 3 (S on the left, exclusive prefix, tensor powers over factorials):
//     S_n(j) = sum_{i <= j} T_n(i),    T_n(i) = sum_{m=0}^{n-1} S_m(i-1) (x) dX_i^{(x)(n-m)} / (n-m)!.
// For one word w.a (parent w of length n-1, last letter a) the inner sum is a Horner chain along the prefixes
// of w, exactly the chain of the fused step:
//     g_0 = 1,  g_m = S_m(i-1)[w_{1:m}] + g_{m-1} * dX_i[w_m] / (n-m+1)   (m = 1 .. n-1),   T_n(i)[w.a] = g_{n-1} * dX_i[a],
// so a term costs n-1 loads of lower-level coefficients, n-1+d FMAs and touches no other word.  The lower levels
// of every prefix must therefore be in memory (the intermediates of shape (B, L-1, d^m) the paper names as its
// memory cost): in stream mode they are the output rows themselves, in final mode a scratch tensor.
//
// Mapping.  Launch n computes level n from levels 1 .. n-1.  A lane owns one parent word w (its d children are
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
// d^{n-2} + ... distinct floats, twice when C > 1) and writes d^n; over all levels that is D written once plus
// about D / (d - 1) read (stream mode), or 2 * (D - d^N) * (1 + 1 / (d - 1)) moved through scratch (final mode).
#include "sig_internal.h"

namespace sig {

namespace {

constexpr int kLsThreads = 256;
constexpr int kLsTileFloats = 4096;  // LDS floats of the increment tile of one workgroup
constexpr int kLsBatch = 4;          // steps whose lower-level loads are in flight together
constexpr int kLsMaxD = 10;
constexpr int kLsMaxLevel = 8;

struct LevelScanArgs {
    const float *path;   // [B][L][d]
    const float *lo;     // levels 1 .. n-1 of prefix (b, j) at lo + (b * K + j) * lo_stride + off[m]
    float *hi;           // level n of prefix (b, j) goes to hi + (b * K + j) * hi_stride + off_n; null: not stored
    float *fin;          // level n of the whole path goes to fin + b * fin_stride + off_n; null: not stored
    int64_t lo_stride, hi_stride, fin_stride;
    int64_t B, L;
    int32_t off[kLsMaxLevel + 1];  // off[m] = d + ... + d^{m-1}, m = 1 .. n
    int32_t parents;     // P = d^{n-1}
    int32_t pw;          // parents per workgroup
    int32_t wblocks;     // ceil(P / pw)
    int32_t chunks;      // C
    int32_t groups;      // G paths per workgroup; G * C * pw <= blockDim.x
    int32_t chunk_steps; // T = ceil(K / C)
    int32_t tile_steps;  // TT <= T; G * C * TT * d <= kLsTileFloats
};

template <int d, int n>
__global__ __launch_bounds__(kLsThreads) void sig_level_scan_kernel(LevelScanArgs A)
{
    constexpr int M = n - 1;  // lower levels on the chain
    extern __shared__ float ls_smem[];
    float *tile = ls_smem;                  // [G][C][TT][d]
    float *tot = ls_smem + kLsTileFloats;   // [G][C][pw][d], used when C > 1

    const int tid = threadIdx.x;
    const int PW = A.pw, C = A.chunks, G = A.groups, T = A.chunk_steps, TT = A.tile_steps;
    const int64_t K = A.L - 1;
    const int wl = tid % PW;
    const int c = (tid / PW) % C;
    const int g = tid / (PW * C);
    const int64_t b0 = (int64_t)(blockIdx.x / A.wblocks) * G;
    const int64_t b = b0 + g;
    const int w = (int)(blockIdx.x % A.wblocks) * PW + wl;
    const bool lane_ok = g < G && b < A.B && w < A.parents;

    // prefixes of the parent word: idx[m] = w_{1:m} as a number in base d, let[m] = w_m
    int ofs[M > 0 ? M : 1], let[M > 0 ? M : 1];
    float rc[M > 0 ? M : 1];
    {
        int rest = lane_ok ? w : 0;
#pragma unroll
        for (int m = M; m >= 1; --m) {
            ofs[m - 1] = A.off[m] + rest;
            let[m - 1] = rest % d;
            rest /= d;
            rc[m - 1] = 1.0f / (float)(n - m + 1);
        }
    }
    const int64_t j_begin = (int64_t)c * T;
    const int64_t j_end = (j_begin + T < K) ? j_begin + T : K;   // may be <= j_begin for trailing chunks
    const float *lo_path = A.lo + (lane_ok ? b : 0) * K * A.lo_stride;
    float *hi_path = A.hi ? A.hi + (lane_ok ? b : 0) * K * A.hi_stride + A.off[n] + (int64_t)w * d : nullptr;
    const float *my_tile = tile + (size_t)((g < G ? g : 0) * C + c) * TT * d;
    const int tiles = (T + TT - 1) / TT;

    float acc[d];
#pragma unroll
    for (int a = 0; a < d; ++a) acc[a] = 0.0f;

    // differenced increments of tile i of every (path, chunk) of the workgroup; zero past the end of a chunk
    auto load_tile = [&](int i) {
        const int total = G * C * TT * d;
        for (int e = tid; e < total; e += blockDim.x) {
            const int a = e % d;
            const int t = (e / d) % TT;
            const int gc = e / (d * TT);
            const int cc = gc % C;
            const int64_t bb = b0 + gc / C;
            const int64_t j = (int64_t)cc * T + (int64_t)i * TT + t;
            const int64_t jend = ((int64_t)(cc + 1) * T < K) ? (int64_t)(cc + 1) * T : K;
            float v = 0.0f;
            if (bb < A.B && j < jend && (int64_t)i * TT + t < T) {
                const float *x = A.path + (bb * A.L + j) * d + a;
                v = x[d] - x[0];
            }
            tile[e] = v;
        }
    };

    // lower-level coefficients of the prefix before step j (zero before the first step)
    auto fetch = [&](int64_t j, bool on, float (&s)[M > 0 ? M : 1]) {
        const bool rd = on && j > 0;
        const float *row = lo_path + (rd ? j - 1 : 0) * A.lo_stride;
#pragma unroll
        for (int m = 0; m < M; ++m) s[m] = rd ? row[ofs[m]] : 0.0f;
    };

    auto sweep = [&](bool emit, bool reload) {
        for (int i = 0; i < tiles; ++i) {
            if (reload) {
                __syncthreads();   // the previous tile has been consumed
                load_tile(i);
                __syncthreads();
            }
            const int64_t jt = j_begin + (int64_t)i * TT;
            float cur[kLsBatch][M > 0 ? M : 1], nxt[kLsBatch][M > 0 ? M : 1];
#pragma unroll
            for (int u = 0; u < kLsBatch; ++u) fetch(jt + u, lane_ok && jt + u < j_end && u < TT, cur[u]);
            for (int t0 = 0; t0 < TT; t0 += kLsBatch) {
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u) {
                    const int t = t0 + kLsBatch + u;
                    fetch(jt + t, lane_ok && t < TT && jt + t < j_end, nxt[u]);
                }
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u) {
                    const int t = t0 + u;
                    const int64_t j = jt + t;
                    const bool on = lane_ok && t < TT && j < j_end;
                    if (on) {
                        const float *dx = my_tile + t * d;
                        float h = 1.0f;
#pragma unroll
                        for (int m = 0; m < M; ++m) h = fmaf(h, dx[let[m]] * rc[m], cur[u][m]);
#pragma unroll
                        for (int a = 0; a < d; ++a) acc[a] = fmaf(h, dx[a], acc[a]);
                        if (emit && hi_path) {
                            float *dst = hi_path + j * A.hi_stride;
#pragma unroll
                            for (int a = 0; a < d; ++a) dst[a] = acc[a];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kLsBatch; ++u)
#pragma unroll
                    for (int m = 0; m < M; ++m) cur[u][m] = nxt[u][m];
            }
        }
    };

    const bool one_tile = tiles == 1;
    if (one_tile) {
        load_tile(0);
        __syncthreads();
    }
    if (C > 1) {
        sweep(false, !one_tile);
        float *mine = tot + (size_t)tid * d;
        if (tid < G * C * PW) {
#pragma unroll
            for (int a = 0; a < d; ++a) mine[a] = acc[a];
        }
        __syncthreads();
        // exclusive prefix over the chunks of this (path, parent), earliest chunk first; the lane of the last
        // chunk also needs nothing more than its own carry-in.  Without per-step stores the sum of all chunks is
        // the result and chunk 0 writes it.
        if (!A.hi) {
            if (lane_ok && c == 0 && A.fin) {
#pragma unroll
                for (int a = 0; a < d; ++a) acc[a] = 0.0f;
                for (int cc = 0; cc < C; ++cc) {
                    const float *src = tot + (size_t)((g * C + cc) * PW + wl) * d;
#pragma unroll
                    for (int a = 0; a < d; ++a) acc[a] += src[a];
                }
                float *dst = A.fin + b * A.fin_stride + A.off[n] + (int64_t)w * d;
#pragma unroll
                for (int a = 0; a < d; ++a) dst[a] = acc[a];
            }
            return;
        }
#pragma unroll
        for (int a = 0; a < d; ++a) acc[a] = 0.0f;
        if (lane_ok) {
            for (int cc = 0; cc < c; ++cc) {
                const float *src = tot + (size_t)((g * C + cc) * PW + wl) * d;
#pragma unroll
                for (int a = 0; a < d; ++a) acc[a] += src[a];
            }
        }
    }
    sweep(true, !one_tile);
    // the chunk that holds the last step also holds the level of the whole path
    if (lane_ok && A.fin && j_begin < K && j_end == K) {
        float *dst = A.fin + b * A.fin_stride + A.off[n] + (int64_t)w * d;
#pragma unroll
        for (int a = 0; a < d; ++a) dst[a] = acc[a];
    }
}

template <int d, int n>
hipError_t launch_one(const LevelScanArgs &A, int blocks, int threads, size_t lds, hipStream_t st)
{
    hipLaunchKernelGGL((sig_level_scan_kernel<d, n>), dim3(blocks), dim3(threads), lds, st, A);
    return hipGetLastError();
}

template <int d>
hipError_t launch_level(int n, const LevelScanArgs &A, int blocks, int threads, size_t lds, hipStream_t st)
{
    switch (n) {
    case 1: return launch_one<d, 1>(A, blocks, threads, lds, st);
    case 2: return launch_one<d, 2>(A, blocks, threads, lds, st);
    case 3: return launch_one<d, 3>(A, blocks, threads, lds, st);
    case 4: return launch_one<d, 4>(A, blocks, threads, lds, st);
    case 5: return launch_one<d, 5>(A, blocks, threads, lds, st);
    case 6: return launch_one<d, 6>(A, blocks, threads, lds, st);
    case 7: return launch_one<d, 7>(A, blocks, threads, lds, st);
    case 8: return launch_one<d, 8>(A, blocks, threads, lds, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_level_d(int d, int n, const LevelScanArgs &A, int blocks, int threads, size_t lds, hipStream_t st)
{
    switch (d) {
    case 1: return launch_level<1>(n, A, blocks, threads, lds, st);
    case 2: return launch_level<2>(n, A, blocks, threads, lds, st);
    case 3: return launch_level<3>(n, A, blocks, threads, lds, st);
    case 4: return launch_level<4>(n, A, blocks, threads, lds, st);
    case 5: return launch_level<5>(n, A, blocks, threads, lds, st);
    case 6: return launch_level<6>(n, A, blocks, threads, lds, st);
    case 7: return launch_level<7>(n, A, blocks, threads, lds, st);
    case 8: return launch_level<8>(n, A, blocks, threads, lds, st);
    case 9: return launch_level<9>(n, A, blocks, threads, lds, st);
    case 10: return launch_level<10>(n, A, blocks, threads, lds, st);
    default: return hipErrorInvalidValue;
    }
}

int floor_pow2(int64_t v)
{
    int p = 1;
    while ((int64_t)p * 2 <= v) p *= 2;
    return p;
}

}  // namespace

bool level_scan_available(int d, int depth) { return d >= 1 && d <= kLsMaxD && depth >= 1 && depth <= kLsMaxLevel; }

int64_t level_scan_scratch_floats(int64_t B, int64_t L, const RowShape &rs, int stream_flag)
{
    if (stream_flag || rs.depth == 1) return 0;
    return B * (L - 1) * (rs.D - rs.pow[rs.depth]);
}

int level_scan_chunks(int64_t B, int64_t L, const RowShape &rs, int level, int forced, int cus)
{
    const int64_t K = L - 1;
    int64_t C;
    if (forced > 0) {
        C = forced;
    } else {
        // enough lanes for four wavefronts on every SIMD, chunks of at least four steps
        const int64_t want = (int64_t)cus * 4 * 4 * kWave;
        const int64_t items = B * rs.pow[level - 1];
        C = floor_pow2((want + items - 1) / items);
        if (C > K / 4) C = K / 4;
        if (C > 32) C = 32;
    }
    if (C > K) C = K;
    if (C > kLsThreads) C = kLsThreads;
    if (C < 1) C = 1;
    return (int)C;
}

hipError_t launch_level_scan(const float *path, float *out, float *scratch, int64_t B, int64_t L, const RowShape &rs,
                             int stream_flag, int forced_chunks, int cus, hipStream_t st)
{
    if (!level_scan_available(rs.d, rs.depth)) return hipErrorInvalidValue;
    const int d = rs.d, N = rs.depth;
    const int64_t K = L - 1;
    const int64_t lower = rs.D - rs.pow[N];  // row length of the scratch tensor (levels 1 .. N-1)
    for (int n = 1; n <= N; ++n) {
        LevelScanArgs A{};
        A.path = path;
        A.B = B;
        A.L = L;
        if (stream_flag) {
            A.lo = out;  A.lo_stride = rs.D;
            A.hi = out;  A.hi_stride = rs.D;
            A.fin = nullptr;  A.fin_stride = 0;
        } else {
            A.lo = scratch;  A.lo_stride = lower;
            A.hi = n < N ? scratch : nullptr;  A.hi_stride = lower;
            A.fin = out;  A.fin_stride = rs.D;
        }
        for (int m = 1; m <= n; ++m) A.off[m] = (int32_t)rs.off[m];
        const int64_t P = rs.pow[n - 1];
        const int C = level_scan_chunks(B, L, rs, n, forced_chunks, cus);
        int64_t PW = kLsThreads / C;
        if (PW > P) PW = P;
        int64_t G = kLsThreads / (PW * C);
        if (G > B) G = B;
        const int T = (int)((K + C - 1) / C);
        int64_t TT = kLsTileFloats / (G * C * d);
        if (TT > T) TT = T;
        if (TT < 1) return hipErrorInvalidValue;  // cannot happen: G * C <= 256 and d <= 10
        const int64_t wblocks = (P + PW - 1) / PW;
        const int64_t blocks = wblocks * ((B + G - 1) / G);
        if (blocks > INT32_MAX) return hipErrorInvalidValue;
        A.parents = (int32_t)P;
        A.pw = (int32_t)PW;
        A.wblocks = (int32_t)wblocks;
        A.chunks = C;
        A.groups = (int32_t)G;
        A.chunk_steps = T;
        A.tile_steps = (int32_t)TT;
        const int used = (int)(G * C * PW);
        const int threads = (used + kWave - 1) / kWave * kWave;
        const size_t lds = (size_t)(kLsTileFloats + (C > 1 ? threads * d : 0)) * sizeof(float);
        hipError_t e = launch_level_d(d, n, A, (int)blocks, threads, lds, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sig

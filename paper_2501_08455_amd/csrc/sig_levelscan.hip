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
#include "sig_levelscan.h"

namespace sig {

using namespace levelscan;

namespace {

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
        hipError_t e = A.cat ? launch_rows_level(d, n, A, vec, (int)blocks, threads, lds, st)
                             : launch_level_d<false>(d, n, A, vec, (int)blocks, threads, lds, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sig

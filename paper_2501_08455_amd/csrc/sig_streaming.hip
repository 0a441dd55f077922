// HBM-streaming kernels: any (d, depth), state in device memory.
//
//   sig_hbm_streaming_kernel  the fused multiply-by-exponential of Eq. 3 applied increment by
//                             increment to state that lives in the output rows themselves
//   sig_combine_rows_kernel   batched truncated product of Eq. 4
//
// Writing out (S (x) exp(v))[w] for a word w = (i_1 .. i_n) with Eqs. 2 and 4 gives
//   S'[w] = S[w] + sum_{m=0}^{n-1} S[w_{1:m}] * v[i_{m+1}] ... v[i_n] / (n - m)!      (S[empty] = 1)
// i.e. the new coefficient of w needs only the old coefficients of the prefixes of w.  In
// Horner form:  g_0 = 1,  g_m = S[w_{1:m}] + g_{m-1} * v[i_m] / (n - m + 1)  (m = 1 .. n-1),
//               S'[w] = S[w] + g_{n-1} * v[i_n].
// Two consequences used here: (i) the words below a fixed prefix u form a sub-tree that evolves
// on its own, given the few scalars S[u_{1:m}], so sub-trees go to different workgroups with no
// communication; (ii) updating levels from depth down to 1 may be done in place.
#include "sig_internal.h"

namespace sig {

namespace {

struct StreamingParams {
    const float *path;
    float *out;
    int64_t L;
    int64_t D;
    int d;
    int depth;
    int p;          // prefix depth of the sub-tree a workgroup owns
    int stream;     // 0: in place in out[b]; 1: row k is written from row k-1
    int tile_steps; // increments staged in LDS at a time
    int gcap;       // floats of each of the two Horner-chain buffers in LDS (>= d^{depth-1-p})
    uint32_t ntiles;             // d^p
    uint32_t pw[kMaxDepth + 1];  // d^n
    int64_t off[kMaxDepth + 2];  // start of level n in a row
};

// Dynamic LDS: [tile_steps][d] increments, then two chain buffers of gcap floats.
extern __shared__ float sig_smem[];

// One workgroup per (path, sub-tree below a prefix u of length p).  Per increment and level n (from depth
// down to p+1) the Horner chain g_m (m = p .. n-1, see the file header) is swept level by level over the whole
// sub-tree: g_m[c] = S_m[c] + g_{m-1}[c / d] * v[c mod d] / (n - m + 1), one thread per word c, reading S_m with
// consecutive threads on consecutive floats and keeping g in LDS; then S_n[c] += g_{n-1}[c / d] * v[c mod d]
// streams through the level once (read-modify-write in final mode, row k-1 -> row k in stream mode).  The
// levels below the top one are d times smaller each, so the traffic is that of the top level: 8 bytes per
// coefficient and increment.
__global__ __launch_bounds__(256) void sig_hbm_streaming_kernel(StreamingParams P)
{
    __shared__ float pre[kMaxDepth + 1];    // pre[m] = S[u_{1:m}], m = 1..p (old values during a step)
    __shared__ int ulet[kMaxDepth + 1];     // ulet[m] = letter u_m
    __shared__ uint32_t pw[kMaxDepth + 1];  // d^n (copied out of the kernel arguments: they are indexed at run time)
    __shared__ int64_t off[kMaxDepth + 2];

    const int d = P.d, depth = P.depth, p = P.p;
    const uint32_t tile = blockIdx.x % P.ntiles;   // u as a number in base d
    const int64_t b = blockIdx.x / P.ntiles;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t K = P.L - 1;
    const float *X = P.path + b * P.L * d;
    float *sh_delta = sig_smem;
    float *g0 = sig_smem + P.tile_steps * d;
    float *g1 = g0 + P.gcap;

    for (int i = tid; i <= depth; i += nthr) pw[i] = P.pw[i];
    for (int i = tid; i <= depth + 1; i += nthr) off[i] = P.off[i];
    if (tid == 0) {
        uint32_t rest = tile;
        for (int m = p; m >= 1; --m) { ulet[m] = (int)(rest % (uint32_t)d); rest /= (uint32_t)d; }
        for (int m = 0; m <= p; ++m) pre[m] = 0.0f;
    }
    __syncthreads();

    for (int64_t k = 0; k < K; ++k) {
        const int kt = (int)(k % P.tile_steps);
        if (kt == 0) {
            // coalesced loader: consecutive threads read consecutive floats of the path
            int64_t steps = K - k < P.tile_steps ? K - k : P.tile_steps;
            int64_t n = steps * d;
            __syncthreads();
            for (int64_t i = tid; i < n; i += nthr) sh_delta[i] = X[k * d + i + d] - X[k * d + i];
            __syncthreads();
        }
        const float *dl = sh_delta + kt * d;
        const bool first = (k == 0);  // the state before the first increment is the identity: all levels >= 1 are 0
        const float *src = P.stream ? P.out + (b * K + (first ? 0 : k - 1)) * P.D : P.out + b * P.D;
        float *dst = P.stream ? P.out + (b * K + k) * P.D : P.out + b * P.D;

        for (int n = depth; n > p; --n) {
            // g_p at the word u itself, from the prefix scalars (every thread computes it: p is small)
            float gu = 1.0f;
            for (int m = 1; m <= p; ++m) gu = fmaf(gu, dl[ulet[m]] * (1.0f / (float)(n - m + 1)), pre[m]);
            // sweep the chain down the sub-tree: gprev holds g_{m-1} (size d^{m-1-p}), gcur receives g_m
            float *gprev = g0, *gcur = g1;
            if (tid == 0) gprev[0] = gu;
            __syncthreads();
            for (int m = p + 1; m <= n - 1; ++m) {
                const uint32_t cnt = pw[m - p];
                const float scale = 1.0f / (float)(n - m + 1);
                const float *sm = src + off[m] + (int64_t)tile * cnt;
                for (uint32_t c = tid; c < cnt; c += nthr) {
                    const uint32_t w = c / (uint32_t)d;
                    const float Sm = first ? 0.0f : sm[c];
                    gcur[c] = fmaf(gprev[w], dl[c - w * d] * scale, Sm);
                }
                __syncthreads();
                float *t = gprev; gprev = gcur; gcur = t;
            }
            // update level n: consecutive threads on consecutive coefficients
            {
                const uint32_t cnt = pw[n - p];
                const int64_t base = off[n] + (int64_t)tile * cnt;
                for (uint32_t c = tid; c < cnt; c += nthr) {
                    const uint32_t w = c / (uint32_t)d;
                    const float old = first ? 0.0f : src[base + c];
                    dst[base + c] = fmaf(gprev[w], dl[c - w * d], old);
                }
            }
            // in place: level n-1 may only be overwritten after every reader of it at level n is done; the
            // chain buffers are reused by the next level
            __syncthreads();
        }
        if (tid == 0) {
            // the words u_{1:n}, n = p .. 1, shared by every sub-tree with this prefix; kept per workgroup
            for (int n = p; n >= 1; --n) {
                float g = 1.0f;
                for (int m = 1; m <= n - 1; ++m) g = fmaf(g, dl[ulet[m]] * (1.0f / (float)(n - m + 1)), pre[m]);
                pre[n] = fmaf(g, dl[ulet[n]], pre[n]);
                // exactly one sub-tree (remaining letters all 0) writes the shared word to the row
                uint32_t span = pw[p - n];
                if (tile % span == 0) dst[off[n] + tile / span] = pre[n];
            }
        }
        __syncthreads();
    }
}

struct CombineParams {
    const float *a;
    const float *b;
    float *out;
    int64_t a_stride, b_stride, out_stride;
    int64_t D;
    int d;
    int depth;
    uint32_t pw[kMaxDepth + 1];
    float inv_pw[kMaxDepth + 1];   // 1 / d^n
    int64_t off[kMaxDepth + 2];
};

// one thread per output word:  c_n[w] = a_n[w] + b_n[w] + sum_{i=1}^{n-1} a_i[w / d^{n-i}] * b_{n-i}[w mod d^{n-i}]
__global__ __launch_bounds__(256) void sig_combine_rows_kernel(CombineParams P, int64_t rows)
{
    // rows and words flattened: no idle threads at the end of short rows
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * P.D) return;
    const int64_t row = idx / P.D;
    const int64_t pos = idx - row * P.D;
    const float *a = P.a + row * P.a_stride;
    const float *b = P.b + row * P.b_stride;
    int n = 1;
    while (pos >= P.off[n + 1]) ++n;
    const uint32_t w = (uint32_t)(pos - P.off[n]);
    float c = a[pos] + b[pos];
    // w = hi * split + lo.  Below 2^24 the quotient comes from a float multiply (exact integers) with a one-step
    // correction instead of an integer division, which costs about forty instructions on this hardware.
    const bool small = P.pw[n] <= (1u << 24);
    const float wf = (float)w;
    for (int i = 1; i < n; ++i) {
        const uint32_t split = P.pw[n - i];
        uint32_t hi, lo;
        if (small) {
            hi = (uint32_t)(wf * P.inv_pw[n - i]);
            int32_t r = (int32_t)(w - hi * split);
            if (r < 0) { --hi; r += (int32_t)split; }
            else if (r >= (int32_t)split) { ++hi; r -= (int32_t)split; }
            lo = (uint32_t)r;
        } else {
            hi = w / split;
            lo = w - hi * split;
        }
        c = fmaf(a[P.off[i] + hi], b[P.off[n - i] + lo], c);
    }
    P.out[row * P.out_stride + pos] = c;
}

// Rows whose levels below the top one fit LDS twice over.  Every word of the product needs, besides its own
// a[w] + b[w], only coefficients of lower levels (a_i[hi] b_{n-i}[lo], i = 1 .. n-1), so a workgroup stages levels
// 1 .. depth-1 of a[row] and b[row] (consecutive threads on consecutive floats) and the gathers hit LDS instead of
// the caches; the top level, most of the row, streams through once.  A row's top level is cut into `slices` pieces
// that go to different workgroups (slice 0 also takes the lower levels); a workgroup walks (row, slice) items, and
// within a level one thread takes one word, so the split points are the same for the whole workgroup.
__global__ __launch_bounds__(256) void sig_combine_rows_lds_kernel(CombineParams P, int64_t rows, int slices)
{
    const int N = P.depth;
    const int64_t low = P.off[N];      // floats of levels 1 .. N-1
    float *sa = sig_smem;
    float *sb = sig_smem + low;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const uint32_t top = P.pw[N];
    const uint32_t per_slice = (top + slices - 1) / slices;
    for (int64_t item = blockIdx.x; item < rows * slices; item += gridDim.x) {
        const int64_t row = item / slices;
        const int slice = (int)(item - row * slices);
        const float *a = P.a + row * P.a_stride;
        const float *b = P.b + row * P.b_stride;
        float *out = P.out + row * P.out_stride;
        __syncthreads();   // the previous item has been consumed
        for (int64_t i = tid; i < low; i += nthr) {
            sa[i] = a[i];
            sb[i] = b[i];
        }
        __syncthreads();
        for (int n = (slice == 0 ? 1 : N); n <= N; ++n) {
            const int64_t base = P.off[n];
            uint32_t w_begin = 0, w_end = P.pw[n];
            if (n == N) {
                w_begin = (uint32_t)slice * per_slice;
                w_end = w_begin + per_slice < top ? w_begin + per_slice : top;
            }
            for (uint32_t w = w_begin + tid; w < w_end; w += nthr) {
                float c = (n == N) ? a[base + w] + b[base + w] : sa[base + w] + sb[base + w];
                const float wf = (float)w;   // levels of at most 2^24 words (checked by the host)
                for (int i = 1; i < n; ++i) {
                    const uint32_t split = P.pw[n - i];
                    uint32_t hi = (uint32_t)(wf * P.inv_pw[n - i]);
                    int32_t r = (int32_t)(w - hi * split);
                    if (r < 0) { --hi; r += (int32_t)split; }
                    else if (r >= (int32_t)split) { ++hi; r -= (int32_t)split; }
                    c = fmaf(sa[P.off[i] + hi], sb[P.off[n - i] + r], c);
                }
                out[base + w] = c;
            }
        }
    }
}

// Many short rows (a batch of products of signatures of a few hundred to a few thousand floats): `per_wg` rows to a
// workgroup, so that every thread has several words to do between the two barriers and the loads of several rows are
// in flight together.  The lower levels of the workgroup's rows are staged in LDS as above; the words of its rows are
// taken flattened (thread t: words t, t + 256, ... of the per_wg * D), consecutive threads on consecutive floats.
__global__ __launch_bounds__(256) void sig_combine_short_rows_kernel(CombineParams P, int64_t rows, int per_wg)
{
    const int N = P.depth;
    const int low = (int)P.off[N];     // floats of levels 1 .. N-1
    float *sa = sig_smem;              // [per_wg][low]
    float *sb = sig_smem + (size_t)per_wg * low;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t row0 = (int64_t)blockIdx.x * per_wg;
    const int nr = rows - row0 < per_wg ? (int)(rows - row0) : per_wg;
    // (index / length by a float multiply with a one-step correction: exact below 2^24, which the host checks)
    const float inv_low = 1.0f / (float)(low > 0 ? low : 1);
    for (int i = tid; i < nr * low; i += nthr) {
        int r = (int)((float)i * inv_low);
        int x = i - r * low;
        if (x < 0) { --r; x += low; }
        else if (x >= low) { ++r; x -= low; }
        sa[i] = P.a[(row0 + r) * P.a_stride + x];
        sb[i] = P.b[(row0 + r) * P.b_stride + x];
    }
    __syncthreads();
    // level by level, so that the level and its split points are the same for the whole workgroup (a lane that looks
    // them up by its own level indexes the kernel arguments per lane, which costs more than the product)
    for (int n = 1; n <= N; ++n) {
        const int cnt = (int)P.pw[n], base = (int)P.off[n];
        const float inv_cnt = P.inv_pw[n];
        for (int idx = tid; idx < nr * cnt; idx += nthr) {
            int r = (int)((float)idx * inv_cnt);
            int wi = idx - r * cnt;
            if (wi < 0) { --r; wi += cnt; }
            else if (wi >= cnt) { ++r; wi -= cnt; }
            const uint32_t w = (uint32_t)wi;
            const float *la = sa + (size_t)r * low, *lb = sb + (size_t)r * low;
            float c = (n == N) ? P.a[(row0 + r) * P.a_stride + base + wi] + P.b[(row0 + r) * P.b_stride + base + wi]
                               : la[base + wi] + lb[base + wi];
            const float wf = (float)w;
            for (int k = 1; k < n; ++k) {
                const uint32_t split = P.pw[n - k];
                uint32_t hi = (uint32_t)(wf * P.inv_pw[n - k]);
                int32_t q = (int32_t)(w - hi * split);
                if (q < 0) { --hi; q += (int32_t)split; }
                else if (q >= (int32_t)split) { ++hi; q -= (int32_t)split; }
                c = fmaf(la[P.off[k] + hi], lb[P.off[n - k] + q], c);
            }
            P.out[(row0 + r) * P.out_stride + base + wi] = c;
        }
    }
}

}  // namespace

bool make_row_shape(int d, int depth, RowShape *rs)
{
    if (d < 1 || depth < 1 || depth > kMaxDepth) return false;
    rs->d = d;
    rs->depth = depth;
    int64_t p = 1, total = 0;
    rs->pow[0] = 1;
    for (int n = 1; n <= depth; ++n) {
        if (p > (int64_t)INT32_MAX / d) return false;  // d^n must fit in int32
        p *= d;
        rs->pow[n] = p;
        rs->off[n] = total;
        total += p;
    }
    rs->off[depth + 1] = total;
    rs->pow[depth + 1] = 0;
    rs->D = total;
    return true;
}

hipError_t launch_hbm_streaming(const float *path, float *out, int64_t B, int64_t L, const RowShape &rs,
                                int p, int stream_flag, int threads, hipStream_t st)
{
    StreamingParams P;
    P.path = path;
    P.out = out;
    P.L = L;
    P.D = rs.D;
    P.d = rs.d;
    P.depth = rs.depth;
    P.p = p;
    P.stream = stream_flag;
    int tile = 8192 / rs.d;
    if (tile > 64) tile = 64;
    if (tile < 1) tile = 1;
    P.tile_steps = tile;
    P.ntiles = (uint32_t)rs.pow[p];
    for (int n = 0; n <= rs.depth; ++n) P.pw[n] = (uint32_t)rs.pow[n];
    for (int n = 1; n <= rs.depth + 1; ++n) P.off[n] = rs.off[n];
    P.off[0] = 0;
    int64_t grid = B * rs.pow[p];
    if (grid <= 0 || grid > INT32_MAX) return hipErrorInvalidValue;
    // the chain buffers hold up to d^{depth-1-p} floats each
    const int64_t gcap = rs.depth - 1 - p >= 0 ? rs.pow[rs.depth - 1 - p] : 1;
    P.gcap = (int)gcap;
    const int64_t lds_floats = (int64_t)tile * rs.d + 2 * gcap;
    if (lds_floats * (int64_t)sizeof(float) > kMaxLdsBytes) return hipErrorInvalidValue;
    size_t lds = (size_t)lds_floats * sizeof(float);
    hipLaunchKernelGGL(sig_hbm_streaming_kernel, dim3((unsigned)grid), dim3(threads), lds, st, P);
    return hipGetLastError();
}

hipError_t launch_combine_rows(const float *a, int64_t a_stride, const float *b, int64_t b_stride,
                               float *out, int64_t out_stride, int64_t B, const RowShape &rs,
                               hipStream_t st)
{
    CombineParams P;
    P.a = a; P.b = b; P.out = out;
    P.a_stride = a_stride; P.b_stride = b_stride; P.out_stride = out_stride;
    P.D = rs.D; P.d = rs.d; P.depth = rs.depth;
    for (int n = 0; n <= rs.depth; ++n) {
        P.pw[n] = (uint32_t)rs.pow[n];
        P.inv_pw[n] = 1.0f / (float)rs.pow[n];
    }
    for (int n = 1; n <= rs.depth + 1; ++n) P.off[n] = rs.off[n];
    P.off[0] = 0;
    const int64_t low = rs.off[rs.depth];   // floats of the levels below the top one
    // A batch of short rows: several rows to a workgroup, about 3,072 words, within 48 KB of staged lower levels
    // (down to rows of six floats: 2^20 products of (2,3) rows 86 -> 67 us against one thread per word).
    if (rs.depth >= 2 && rs.D >= 6 && rs.D <= 4096 && B >= 2048) {
        int64_t per_wg = (3072 + rs.D - 1) / rs.D;
        while (per_wg > 1 && 2 * per_wg * low * (int64_t)sizeof(float) > 48 * 1024) --per_wg;
        if (per_wg > B / 1024) per_wg = B / 1024;   // at least four workgroups for every compute unit
        const int64_t grid = (B + per_wg - 1) / per_wg;
        if (2 * per_wg * low * (int64_t)sizeof(float) <= 48 * 1024 && grid <= INT32_MAX) {
            const size_t lds = (size_t)(2 * per_wg * low) * sizeof(float);
            hipLaunchKernelGGL(sig_combine_short_rows_kernel, dim3((unsigned)grid), dim3(256), lds, st, P, B, (int)per_wg);
            return hipGetLastError();
        }
    }
    if (rs.D >= 64 && rs.pow[rs.depth] <= ((int64_t)1 << 24) && 2 * low * (int64_t)sizeof(float) <= 48 * 1024) {
        // lower levels staged in LDS; pieces of at least 8192 top-level words, enough workgroups to fill the chip
        int64_t slices = rs.pow[rs.depth] / 8192;
        if (slices < 1) slices = 1;
        if (slices > 4096) slices = 4096;
        // few rows (the joins of a handful of long paths): shorter pieces, down to 512 words, for about two
        // workgroups per compute unit
        if (B * slices < 512) {
            int64_t want = (512 + B - 1) / B, most = rs.pow[rs.depth] / 512;
            if (want > most) want = most;
            if (want > slices) slices = want;
        }
        const int64_t items = B * slices;
        const int64_t grid = items < 8 * 256 ? items : 8 * 256;
        const size_t lds = (size_t)(2 * low) * sizeof(float);
        hipLaunchKernelGGL(sig_combine_rows_lds_kernel, dim3((unsigned)grid), dim3(256), lds, st, P, B, (int)slices);
        return hipGetLastError();
    }
    // very short rows, and rows too long for LDS: one thread per word of the whole batch, in slabs of rows whose
    // word count fits the grid
    const int64_t max_words = (int64_t)INT32_MAX / 2 * 256;
    int64_t slab = max_words / rs.D;
    if (slab < 1) return hipErrorInvalidValue;   // cannot happen: D < 2^32
    for (int64_t b0 = 0; b0 < B; b0 += slab) {
        const int64_t nb = B - b0 < slab ? B - b0 : slab;
        CombineParams Q = P;
        Q.a += b0 * a_stride; Q.b += b0 * b_stride; Q.out += b0 * out_stride;
        const int64_t blocks = (nb * rs.D + 255) / 256;
        hipLaunchKernelGGL(sig_combine_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, Q, nb);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sig

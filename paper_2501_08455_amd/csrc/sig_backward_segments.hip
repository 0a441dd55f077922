// Gradient of the signature with respect to the path, cut in time across workgroups: few long paths (final mode;
// stream mode further down, at sig_backward_segment_affine_kernel).
//
// The reverse sweep (see sig_backward.hip) walks the K increments of a path one after the other, and a workgroup
// per path (and slice of its lanes) leaves most of the chip idle when there are few paths.  Chen's relation (paper
// Eq. 3: the signature of a concatenation is the product of the signatures) lets the sweep start anywhere: segment
// s of W, the increments [s T, (s + 1) T), needs the signature S_end(s) of the path up to its end and the gradient
// A_end(s) of the loss with respect to that signature.  With E_s the signature of segment s alone,
//     S_end(s) = E_0 (x) ... (x) E_s,
//     A_end(s)[u] = sum_x d(loss)/d(out)[(u, x)] Y_{s+1}[x],      Y_s = E_s (x) ... (x) E_{W-1}
// (the transpose of the product of Eq. 4 with respect to its left factor; x runs over all words including the empty
// one, whose coefficient is 1).  The launches:
//   1. every (path, segment) folds its increments from the identity: E_s                          (T steps)
//   2. ceil(log2 W) rounds of a scan give all prefix products S_end(s) and all suffix products Y_s at once
//   3. every segment pulls the upstream gradient back through Y_{s+1}: A_end(s)
//   4. every piece runs the reverse sweep over its own increments                                 (T steps)
//   5. the sums of d(loss)/d(increment) are added up over the slices and differenced into d(loss)/dX.
// Launch 4 is the sliced sweep on (path, segment, slice of lanes) for shapes with more than 128 lanes per path, and
// the register sweep with several (path, segment) pieces per workgroup for the others (both in sig_backward.h).
#include "sig_backward.h"

namespace sig {
namespace onchip {

// 1. E[(b, s)] = signature of segment s of path b alone
template <int d, int N, int P>
//    shifted != 0 (stream mode): piece (b, s >= 1) writes to row (b, s - 1) and row (b, W - 1) is the identity, so that
//    row s holds the signature of the segment that follows segment s
__global__ __launch_bounds__(kSliceLanes) void sig_backward_segment_fold_kernel(const float *path, float *E, int64_t L,
                                                                                int W, int T, int shifted)
{
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr int slices = (Q + kSliceLanes - 1) / kSliceLanes;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int slice = (int)(blockIdx.x % slices);
    const int64_t piece = blockIdx.x / slices;
    const int64_t b = piece / W;
    const int seg = (int)(piece - b * W);
    const int64_t k0 = (int64_t)seg * T;
    int64_t K = L - 1 - k0;
    if (K > T) K = T;
    if (K < 0) K = 0;
    const unsigned u_raw = (unsigned)(slice * kSliceLanes + tid);
    const bool active = u_raw < (unsigned)Q;
    const unsigned u = active ? u_raw : 0u;

    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    }

    float *tile = sig_backward_smem;   // [K][d] increments
    {
        const float *x = path + (b * L + k0) * d;
        for (int i = tid; i < (int)K * d; i += nthr) tile[i] = x[i + d] - x[i];
    }
    __syncthreads();
    Lane<d, N, P> ln;
    identity_state<d, N, P>(ln);
    for (int k = 0; k < (int)K; ++k) {
        Inc<d, P> inc;
        load_inc<d, P>(inc, tile + k * d, letter);
        fused_step<d, N, P>(ln, inc);
    }
    if (shifted && seg == 0) identity_state<d, N, P>(ln);
    const int64_t dst = !shifted ? piece : seg > 0 ? piece - 1 : b * W + (W - 1);
    if (active) store_state<d, N, P>(E + dst * D, u, ln);
}

// out[u] = sum over the words x (the empty one included) of A[(u, x)] E[x] on rows of D floats: the transpose of
// c = a (x) E (Eq. 4) with respect to a.  Word v of level j collects A_n[v d^{n-j} + x] E_{n-j}[x] for every deeper
// level n: a wavefront per word where that is 128 terms or more (lanes stride over the terms, fixed-order butterfly
// sum), a thread per word otherwise.  Called by `threads` threads numbered tid = 0 .. threads - 1 in whole
// wavefronts (they may belong to several workgroups); out may not overlap A.
template <int d, int N>
__device__ __forceinline__ void row_adjoint_product(const float *A, const float *E, float *out, int tid, int threads,
                                                    const float *plus = nullptr)   // plus: a row added to the result
{
    using Sh = Shape<d, N, 0>;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int waves = threads / kWave;
    static_for<1, N + 1>([&](auto jc) __attribute__((always_inline)) {
        constexpr int j = decltype(jc)::value;
        constexpr int cnt = cpow(d, j);
        constexpr int terms = geom(d, N - j + 1) - 1;   // d + ... + d^{N-j}
        if constexpr (terms >= 128) {
            for (int v = wave; v < cnt; v += waves) {
                float acc = 0.0f;
                static_for<j + 1, N + 1>([&](auto nc) __attribute__((always_inline)) {
                    constexpr int n = decltype(nc)::value;
                    constexpr int run = cpow(d, n - j);
                    const float *a = A + Sh::row_off(n) + (int64_t)v * run;
                    const float *e = E + Sh::row_off(n - j);
                    // (a fixed trip count, so that the loads of several rounds are in flight together)
                    constexpr int rounds = (run + kWave - 1) / kWave;
#pragma unroll 8
                    for (int i = 0; i < rounds; ++i) {
                        const int x = lane + i * kWave;
                        if (x < run) acc = fmaf(a[x], e[x], acc);
                    }
                });
#pragma unroll
                for (int off = kWave / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
                if (lane == 0) out[Sh::row_off(j) + v] = A[Sh::row_off(j) + v] + acc + (plus ? plus[Sh::row_off(j) + v] : 0.0f);
            }
        } else {
            for (int v = tid; v < cnt; v += threads) {
                float acc = A[Sh::row_off(j) + v];
                static_for<j + 1, N + 1>([&](auto nc) __attribute__((always_inline)) {
                    constexpr int n = decltype(nc)::value;
                    constexpr int run = cpow(d, n - j);
                    const float *a = A + Sh::row_off(n) + (int64_t)v * run;
                    const float *e = E + Sh::row_off(n - j);
#pragma unroll
                    for (int x = 0; x < run; ++x) acc = fmaf(a[x], e[x], acc);
                });
                out[Sh::row_off(j) + v] = acc + (plus ? plus[Sh::row_off(j) + v] : 0.0f);
            }
        }
    });
}

// 2. One round of both scans over the W rows of a path (ping-pong buffers):
//    blockIdx.y = 0: Sout[s] = Sin[s - off] (x) Sin[s] for s >= off, else Sin[s]      (prefix products)
//    blockIdx.y = 1: Yout[s] = Yin[s] (x) Yin[s + off] for s + off < W, else Yin[s]   (suffix products)
//    row_workgroups<d, N>() workgroups (blockIdx.z) share a row; the rows stay in device memory.
template <int d, int N>
constexpr int row_workgroups()
{
    const int want = RowProduct<d, N>::ITEMS / 256;   // about one parent word per thread: the products are bound by
                                                      // the latency of their loads, not by arithmetic
    return want < 1 ? 1 : (want > 32 ? 32 : want);
}

template <int d, int N>
__global__ __launch_bounds__(256) void sig_backward_segment_scan_kernel(const float *Sin, float *Sout, const float *Yin,
                                                                        float *Yout, int W, int off)
{
    using RP = RowProduct<d, N>;
    constexpr int D = Shape<d, N, 0>::D;
    constexpr int threads = 256 * row_workgroups<d, N>();
    const int tid = (int)(blockIdx.z * 256 + threadIdx.x);
    const int64_t piece = blockIdx.x;
    const int s = (int)(piece % W);
    const bool prefix = blockIdx.y == 0;
    const float *in = prefix ? Sin : Yin;
    float *out = (prefix ? Sout : Yout) + piece * D;
    const float *self = in + piece * D;
    const bool joined = prefix ? s >= off : s + off < W;
    if (!joined) {
        for (int x = tid; x < D; x += threads) out[x] = self[x];
        return;
    }
    const float *left = prefix ? in + (piece - off) * D : self;
    const float *right = prefix ? self : in + (piece + off) * D;
    for (int x = tid; x < RP::ITEMS; x += threads) RP::item(left, right, out, x);
}

// 3. A_end(s) = d(loss)/d(out) pulled back through Y_{s+1}, s = 0 .. W-2 (row W-1 is not written: the last segment
//    starts from the upstream gradient itself)
template <int d, int N>
__global__ __launch_bounds__(256) void sig_backward_segment_adjoint_kernel(const float *grad_out, const float *Y, float *Aend,
                                                                           int W)
{
    constexpr int D = Shape<d, N, 0>::D;
    const int64_t piece = blockIdx.x;
    const int64_t b = piece / W;
    const int s = (int)(piece - b * W);
    if (s >= W - 1) return;
    row_adjoint_product<d, N>(grad_out + b * D, Y + (piece + 1) * D, Aend + piece * D, (int)(blockIdx.z * 256 + threadIdx.x),
                              256 * row_workgroups<d, N>());
}

// Stream mode.  Every output row has its own upstream gradient, so what reaches the end of segment s from the later
// segments is  R_s = c_{s+1} + (the transpose of . (x) E_{s+1}) R_{s+1},  R_{W-1} = 0,  with c_t what the rows of
// segment t themselves leave at its start (a first sweep of every segment from a zero adjoint).  One round of the
// scan that solves this recursion for all s at once: row s stands for the map R_s = C_s + transpose(. (x) P_s) R_{s+off}
// over a window of `off` segments, and two windows are joined by
//     C_s <- C_s + transpose(. (x) P_s) C_{s+off},      P_s <- P_s (x) P_{s+off}          (s + off < W, else kept).
// blockIdx.y = 0: the C rows, 1: the P rows; after ceil(log2 W) rounds C_s = R_s.
template <int d, int N>
__global__ __launch_bounds__(256) void sig_backward_segment_affine_kernel(const float *Cin, float *Cout, const float *Pin,
                                                                          float *Pout, int W, int off)
{
    using RP = RowProduct<d, N>;
    constexpr int D = Shape<d, N, 0>::D;
    constexpr int threads = 256 * row_workgroups<d, N>();
    const int tid = (int)(blockIdx.z * 256 + threadIdx.x);
    const int64_t piece = blockIdx.x;
    const int s = (int)(piece % W);
    const bool joined = s + off < W;
    if (blockIdx.y == 0) {
        if (joined) row_adjoint_product<d, N>(Cin + (piece + off) * D, Pin + piece * D, Cout + piece * D, tid, threads, Cin + piece * D);
        else for (int x = tid; x < D; x += threads) Cout[piece * D + x] = Cin[piece * D + x];
    } else {
        if (joined) for (int x = tid; x < RP::ITEMS; x += threads) RP::item(Pin + piece * D, Pin + (piece + off) * D, Pout + piece * D, x);
        else for (int x = tid; x < D; x += threads) Pout[piece * D + x] = Pin[piece * D + x];
    }
}

// Stream-mode cut of the sliced shapes: the first sweep leaves, per (piece, slice), the slice's sums of the partial
// adjoints of the words of levels 1 .. P-1 (the first `words` floats of a row); this adds the slices in order into the
// row that the sweep's lanes wrote their own words to (piece (b, s) hands its row to (b, s - 1); the last row of a
// path is zero).
__global__ __launch_bounds__(256) void sig_backward_segment_prefix_kernel(const float *side, float *rows, int64_t pieces,
                                                                          int W, int slices, int words, int64_t D)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= pieces * words) return;
    const int64_t piece = idx / words;
    const int w = (int)(idx - piece * words);
    const int64_t b = piece / W;
    const int seg = (int)(piece - b * W);
    float sum = 0.0f;
    for (int sl = 0; sl < slices; ++sl) sum += side[(piece * slices + sl) * words + w];
    rows[(seg > 0 ? piece - 1 : b * W + (W - 1)) * D + w] = seg > 0 ? sum : 0.0f;
}

// shapes whose lanes fit a workgroup at least twice take the register sweep with several pieces per workgroup
template <int d, int N, int P>
constexpr bool segments_packed() { return Shape<d, N, P>::Q * 2 <= 256; }

// does a segment of T increments fit the LDS of its sweep?
template <int d, int N, int P>
bool segment_fits(int64_t T)
{
    if constexpr (segments_packed<d, N, P>()) return backward_lds_bytes<d, N, P>(T + 1, 1) <= kMaxLdsBytes;
    else return backward_sliced_steps<d>(T + 1) >= 1;
}

template <int d, int N, int P>
hipError_t backward_segmented_launch(const BackwardArgs &A0, float *scratch, int W, int cus, hipStream_t st)
{
    using Sh = Shape<d, N, P>;
    constexpr bool packed = segments_packed<d, N, P>();
    constexpr int slices = (Sh::Q + kSliceLanes - 1) / kSliceLanes;
    const int64_t K = A0.L - 1;
    if (W < 2 || W > K || !scratch || cus < 1) return hipErrorInvalidValue;
    const int64_t T = (K + W - 1) / W;
    W = (int)((K + T - 1) / T);   // no trailing segment without increments
    const int64_t pieces = A0.B * W;
    if (W < 2 || !segment_fits<d, N, P>(T) || pieces * slices > INT32_MAX || A0.B > INT32_MAX) return hipErrorInvalidValue;
    const int64_t rows = pieces * Sh::D;
    float *E = scratch, *S0 = E + rows, *S1 = S0 + rows, *Y0 = S1 + rows, *Y1 = Y0 + rows, *part = Y1 + rows;
    static_assert(slices * shared_prefix_words<d, P>() <= Sh::D, "the per-slice prefix sums of a piece fit one row");
    if (A0.stream_flag) {
        // stream mode: fold (rows shifted by one segment), first sweep, the scan above, second sweep, finish
        float *P0 = E, *P1 = S0, *C0 = S1, *C1 = Y0, *side = Y1;
        const int fold_threads = Sh::Q >= kSliceLanes ? kSliceLanes : (Sh::Q + kWave - 1) / kWave * kWave;
        hipLaunchKernelGGL((sig_backward_segment_fold_kernel<d, N, P>), dim3((unsigned)(pieces * slices)), dim3(fold_threads),
                           (size_t)(T * d) * sizeof(float), st, A0.path, P0, A0.L, W, (int)T, 1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        BackwardArgs A = A0;
        A.segs = W;
        A.seg_steps = (int32_t)T;
        A.seg_part = part;
        A.seg_adj_out = C0;
        // launch geometry of the two sweeps
        int G = 1, ts = 1;
        size_t lds;
        dim3 grid;
        if constexpr (packed) {
            G = 256 / Sh::Q;
            const int64_t per_cu = (pieces + cus - 1) / cus;
            if ((int64_t)G > per_cu) G = (int)per_cu;
            while (G > 1 && backward_lds_bytes<d, N, P>(T + 1, G) > kMaxLdsBytes) --G;
            if (per_cu > G) {   // the same number of pieces on every compute unit (see backward_launch)
                const int64_t rounds = (per_cu + G - 1) / G;
                G = (int)((per_cu + rounds - 1) / rounds);
            }
            A.groups = G;
            lds = (size_t)backward_lds_bytes<d, N, P>(T + 1, G);
            grid = dim3((unsigned)((pieces + G - 1) / G));
            hipLaunchKernelGGL((sig_backward_kernel<d, N, P, true, true, false>), grid, dim3(256), lds, st, A);
        } else {
            ts = backward_sliced_steps<d>(T + 1);
            lds = (size_t)backward_sliced_bytes_with<d>(T + 1, ts);
            grid = dim3((unsigned)(pieces * slices));
            hipLaunchKernelGGL((sig_backward_sliced_kernel<d, N, P, true, false>), grid, dim3(kSliceLanes), lds, st, A, side, ts);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            constexpr int words = shared_prefix_words<d, P>();
            if constexpr (words > 0) {
                const int64_t blocks = (pieces * words + 255) / 256;
                hipLaunchKernelGGL(sig_backward_segment_prefix_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const float *)side,
                                   C0, pieces, W, slices, words, (int64_t)Sh::D);
            }
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        {
            const float *Cin = C0, *Pin = P0;
            float *Cout = C1, *Pout = P1;
            for (int off = 1; off < W; off *= 2) {
                hipLaunchKernelGGL((sig_backward_segment_affine_kernel<d, N>), dim3((unsigned)pieces, 2, row_workgroups<d, N>()),
                                   dim3(256), 0, st, Cin, Cout, Pin, Pout, W, off);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
                Cin = Cout;
                Pin = Pout;
                Cout = Cout == C1 ? C0 : C1;
                Pout = Pout == P1 ? P0 : P1;
            }
            A.seg_grad = Cin;
            if constexpr (packed)
                hipLaunchKernelGGL((sig_backward_kernel<d, N, P, true, true, true>), grid, dim3(256), lds, st, A);
            else
                hipLaunchKernelGGL((sig_backward_sliced_kernel<d, N, P, true, true>), grid, dim3(kSliceLanes), lds, st, A, part, ts);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            return launch_backward_finish(part, A.grad_path, A.B, A.L, d, slices, st);
        }
    }

    const int fold_threads = Sh::Q >= kSliceLanes ? kSliceLanes : (Sh::Q + kWave - 1) / kWave * kWave;
    hipLaunchKernelGGL((sig_backward_segment_fold_kernel<d, N, P>), dim3((unsigned)(pieces * slices)), dim3(fold_threads),
                       (size_t)(T * d) * sizeof(float), st, A0.path, E, A0.L, W, (int)T, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const float *Sin = E, *Yin = E;
    float *Sout = S0, *Yout = Y0;
    for (int off = 1; off < W; off *= 2) {
        hipLaunchKernelGGL((sig_backward_segment_scan_kernel<d, N>), dim3((unsigned)pieces, 2, row_workgroups<d, N>()), dim3(256),
                           0, st, Sin, Sout, Yin, Yout, W, off);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        Sin = Sout;
        Yin = Yout;
        Sout = Sout == S0 ? S1 : S0;
        Yout = Yout == Y0 ? Y1 : Y0;
    }
    // the scan's last input buffer of the suffix products is free now: it takes the pulled-back gradients
    float *Aend = Yout;
    hipLaunchKernelGGL((sig_backward_segment_adjoint_kernel<d, N>), dim3((unsigned)pieces, 1, row_workgroups<d, N>()), dim3(256),
                       0, st, A0.grad_out, Yin, Aend, W);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    BackwardArgs A = A0;
    A.segs = W;
    A.seg_steps = (int32_t)T;
    A.seg_sig = Sin;
    A.seg_grad = Aend;
    A.seg_part = part;
    if constexpr (packed) {
        // pieces per workgroup: as many as the threads hold, spread over the compute units first, fewer if LDS is short
        int G = 256 / Sh::Q;
        const int64_t per_cu = (pieces + cus - 1) / cus;
        if ((int64_t)G > per_cu) G = (int)per_cu;
        while (G > 1 && backward_lds_bytes<d, N, P>(T + 1, G) > kMaxLdsBytes) --G;
        if (per_cu > G) {   // the same number of pieces on every compute unit (see backward_launch)
            const int64_t rounds = (per_cu + G - 1) / G;
            G = (int)((per_cu + rounds - 1) / rounds);
        }
        A.groups = G;
        const size_t lds = (size_t)backward_lds_bytes<d, N, P>(T + 1, G);
        hipLaunchKernelGGL((sig_backward_kernel<d, N, P, false, true>), dim3((unsigned)((pieces + G - 1) / G)), dim3(256), lds,
                           st, A);
    } else {
        const int ts = backward_sliced_steps<d>(T + 1);
        const size_t lds = (size_t)backward_sliced_bytes_with<d>(T + 1, ts);
        hipLaunchKernelGGL((sig_backward_sliced_kernel<d, N, P, false>), dim3((unsigned)(pieces * slices)), dim3(kSliceLanes),
                           lds, st, A, part, ts);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_backward_finish(part, A.grad_path, A.B, A.L, d, slices, st);
}

}  // namespace onchip

namespace {

template <int d, int N, int P>
int uncut_chunks(int64_t L, int stream_flag)
{
    if constexpr (onchip::Shape<d, N, P>::Q <= 256) return onchip::backward_chunks<d, N, P>(L, stream_flag, 256);
    else return 1;
}

struct SegmentedEntry {
    int d, depth;
    int lanes;        // Q = d^P
    int64_t row;      // D
    hipError_t (*launch)(const onchip::BackwardArgs &, float *, int, int, hipStream_t);
    bool (*fits)(int64_t);             // does a segment of T increments fit the LDS of its sweep?
    int (*uncut_chunks)(int64_t L, int stream_flag);   // chunks the uncut sweep holds side by side in a workgroup
};
#define SIG_SEGMENTED_ENTRY(d, N, P) \
    {d, N, onchip::Shape<d, N, P>::Q, onchip::Shape<d, N, P>::D, &onchip::backward_segmented_launch<d, N, P>, &onchip::segment_fits<d, N, P>, \
     &uncut_chunks<d, N, P>},
const SegmentedEntry kSegmented[] = {
    SIG_BACKWARD_SHAPES(SIG_SEGMENTED_ENTRY, SIG_SEGMENTED_ENTRY)
    {0, 0, 0, 0, nullptr, nullptr, nullptr},
};

const SegmentedEntry *find_segmented(int d, int depth)
{
    for (const SegmentedEntry *e = kSegmented; e->launch; ++e)
        if (e->d == d && e->depth == depth) return e;
    return nullptr;
}

constexpr int kMaxSegments = 32;
constexpr int64_t kMaxSegmentFloats = 1 << 21;   // floats of the B * W rows of one scan buffer
constexpr int64_t kMaxSegmentRow = 1 << 17;   // one workgroup forms a product of two rows: rows up to this many floats

}  // namespace

// Time segments for the final-mode sweep of B paths of L points (<= 1: do not cut).  Cutting pays when the uncut
// launch leaves most of the chip idle and the path is long: the sequential part drops from K steps (2 K / C for a
// shape whose plain sweep holds C chunks of a path side by side in its workgroup) to about K / W, for
// ceil(log2 W) + 3 more launches of 3-6 us each.  Rules, from a measured grid (15 shapes, B = 1 .. 1,024,
// L = 100 .. 2,000):
//   * from 128 increments on, while the uncut launch has fewer than two workgroups per compute unit (between one
//     and two, a few segments still pay: d = 8, depth 4, 128 paths of 500 points, 292 -> 187 us with four);
//   * shapes whose plain sweep holds eight or more chunks: only from 512 increments on; with six or more chunks:
//     only up to 32 paths (cutting wins or ties at every measured point up to there; beyond, the plain sweep's
//     workgroups fill enough of the chip).  Long paths leave the plain sweep fewer chunks (their increments take
//     the LDS), so they are cut at larger batches as well (d = 5, depth 4, 128 paths of 2,000 points: three chunks,
//     328 -> 173 us);
//   * W = K / 24, at most 32, at most two workgroups per compute unit (two wavefronts per SIMD for the shapes that
//     pack several pieces into a workgroup), one set of rows within 8 MB (beyond, the scan's traffic costs more
//     than the shorter sweeps save); a launch that has a workgroup per compute unit already: at most 4 segments,
//     four workgroups per compute unit, 16 MB;
//   * a path whose increments do not fit the LDS of the uncut sweep (uncut_fits == false) is cut at any batch size,
//     as little as makes a segment fit.
int backward_segments(int d, int depth, int64_t B, int64_t L, int cus, bool uncut_fits, int stream_flag)
{
    const SegmentedEntry *e = find_segmented(d, depth);
    if (!e || e->row > kMaxSegmentRow || B <= 0) return 1;
    const int64_t K = L - 1;
    const bool packed = e->lanes * 2 <= onchip::kSliceLanes;   // several pieces share a workgroup
    const int64_t slices = (e->lanes + onchip::kSliceLanes - 1) / onchip::kSliceLanes;
    const int64_t chip_lanes = (int64_t)cus * 4 * kWave * 2;   // two wavefronts on every SIMD
    bool busy = B * slices >= 2 * (int64_t)cus;   // the uncut launch already has two workgroups for every compute unit
    // (stream mode cuts cost two sweeps and a second read of the upstream gradient: the sliced shapes are cut only
    // below a workgroup per compute unit, half of that for paths under 512 increments)
    if (stream_flag && !packed) busy = B * slices >= (K < 512 ? cus / 2 : cus);
    int64_t min_steps = 128;
    if (packed && uncut_fits) {
        const int chunks = e->uncut_chunks(L, stream_flag);
        if (chunks >= 8) min_steps = 512;
        if (B > 32 && chunks >= 6) busy = true;
        // stream mode, rows of a few dozen floats (d = 2 at depth 3, d = 5 at depth 2): the plain sweep with its
        // chunks is as fast at every measured length
        if (stream_flag && chunks >= 8 && e->row <= 32) busy = true;
    }
    if (uncut_fits && (K < min_steps || busy)) return 1;
    // a stream-mode batch that fills the chip: walking the path in tiles (one sweep) beats cutting it (two)
    if (stream_flag && busy) return 1;
    int64_t W = 2;
    if (!busy) {
        W = K / 24;
        if (W > kMaxSegments) W = kMaxSegments;
        // a launch that already has a workgroup per compute unit takes at most four segments
        const bool half_full = !stream_flag && B * slices >= cus;
        if (half_full && W > 4) W = 4;
        const int64_t room = packed ? chip_lanes / (B * e->lanes) : ((half_full ? 4 : 2) * (int64_t)cus) / (B * slices);
        if (W > room) W = room;
        // the scan reads and writes all B * W rows in every round: keep one set of rows within 8 MB (16 MB for the
        // few segments of a half-full launch)
        const int64_t by_rows = (half_full ? 2 : 1) * kMaxSegmentFloats / (B * e->row);
        if (W > by_rows) W = by_rows;
        if (W < 2) {
            if (uncut_fits) return 1;
            W = 2;
        }
    }
    while (W <= kMaxSegments && W <= K && !e->fits((K + W - 1) / W)) ++W;
    if (W > kMaxSegments || W > K || (K + W - 1) / W < 2) return 1;
    const int64_t T = (K + W - 1) / W;   // increments per segment; no segment is left without increments
    W = (K + T - 1) / T;
    // huge batches of long paths: the five sets of segment rows would take more than 2 GiB of scratch; the caller's
    // tiled sweep needs none of them
    if (5 * B * W * e->row > ((int64_t)1 << 29)) return 1;
    return W < 2 ? 1 : (int)W;
}

int64_t backward_segmented_scratch_floats(int d, int depth, int64_t B, int64_t L, int segs)
{
    const SegmentedEntry *e = find_segmented(d, depth);
    if (!e || segs < 2) return 0;
    const int64_t slices = (e->lanes + onchip::kSliceLanes - 1) / onchip::kSliceLanes;
    return 5 * B * segs * e->row + B * slices * (L - 1) * d;
}

hipError_t launch_backward_segmented(const float *path, const float *sig, const float *grad_out, float *grad_path,
                                     float *scratch, int64_t B, int64_t L, int d, int depth, int stream_flag, int segs,
                                     int cus, hipStream_t st)
{
    const SegmentedEntry *e = find_segmented(d, depth);
    if (!e) return hipErrorInvalidValue;
    onchip::BackwardArgs A{};
    A.path = path;
    A.sig = sig;
    A.grad_out = grad_out;
    A.grad_path = grad_path;
    A.B = B;
    A.L = L;
    A.stream_flag = stream_flag;
    return e->launch(A, scratch, segs, cus, st);
}

}  // namespace sig

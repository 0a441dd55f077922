// Gradient of the signature with respect to the path (reverse sweep), on-chip family.
//
// The signature layer is trained between other layers (paper Section 4.2, Eq. 11), so d(loss)/d(path) is
// needed from d(loss)/d(output).  The paper differentiates Eqs. 2-5 automatically; here the reverse sweep is
// written by hand on the same lane layout as the forward kernels:
//
//   * A lane owns the sub-tree of words below its prefix u, |u| = P, of BOTH the signature S and its adjoint
//     A = d(loss)/dS, plus private copies of the prefix scalars S[u_{1:m}] and private PARTIAL adjoints of
//     them (everything is linear in A, so the partials of the lanes that share a prefix word never have to be
//     added up: only their sum would be the adjoint of that word, and nothing needs it).
//   * No prefix signature is stored: signatures of paths are invertible, S_{k-1} = S_k (x) exp(-dX_k), so the
//     sweep k = K-1 .. 0 first takes the forward fused step with the negated increment and then runs the
//     transpose of the forward step S_{k-1} -> S_k.
//   * Forward step in Horner form (see sig_onchip.h): for every target level n, g_{n,0} = 1,
//       g_{n,m}[w a] = S_m[w a] + g_{n,m-1}[w] v[a] / (n-m+1)   (m < n),   S'_n[w a] = S_n[w a] + g_{n,n-1}[w] v[a].
//     Transposed, with gb the adjoint of g:  gb_{n,n-1}[w] = sum_a A'_n[w a] v[a],
//       A_m[w a] += gb_{n,m}[w a],  gb_{n,m-1}[w] = sum_a gb_{n,m}[w a] v[a] / (n-m+1),
//     and d(loss)/dv[a] collects A'_n[w a] g_{n,n-1}[w] and gb_{n,m}[w a] g_{n,m-1}[w] / (n-m+1).
//     Chains are taken in the order n = 1 .. N so that A can be updated in place (chain n reads level n as it
//     came in and adds to the levels below it).
//   * d(loss)/dv of one step is a sum over the Q = d^P lanes of a path.  Lanes park their partial sums of
//     TS = min(max(1, Q / d), 8) consecutive steps in LDS; then lane c of the path adds up column c = (step, channel)
//     in a fixed order (deterministic) and writes the sum over the increment it belongs to, which is no
//     longer needed.  When the sweep is done the tile holds d(loss)/d(dX_k) and the workgroup writes
//     d(loss)/dX_j = d/d(dX_{j-1}) - d/d(dX_j) with consecutive threads on consecutive floats.
//   * Stream mode: row k of the output is S_k, so its upstream gradient is added to A when the sweep reaches
//     k (prefix words by the one lane of each prefix whose remaining letters are 0).
#include "sig_backward.h"

namespace sig {
namespace onchip {

// Transpose of reg_product with respect to its left factor.  For c = a (x) b (Eq. 4), c[w] = sum over the
// splits w = (v, x) of a[v] b[x], so d(loss)/da[v] = sum_x d(loss)/dc[(v, x)] b[x].  `ad` holds d(loss)/dc on
// entry and d(loss)/da on return, in the lane layout of the sweep (sub-tree below u, private partials for the
// prefix words); b is a row of D floats in LDS.  All words (v, x) a lane needs lie in its own sub-tree or on its
// own prefix, so nothing crosses lanes.
template <int d, int N, int P>
__device__ __forceinline__ void reg_adjoint_product(Lane<d, N, P> &ad, const float *b, unsigned u)
{
    using Sh = Shape<d, N, P>;
    // prefix words u_{1:i}, i = 1 .. P, shortest first (they read the longer ones and the sub-tree as they came in)
    static_for<1, P + 1>([&](auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        float acc = prefix_value<i>(ad);
        // longer prefix words u_{1:n}: x = u_{i+1:n}
        static_for<i + 1, P + 1>([&](auto nc) __attribute__((always_inline)) {
            constexpr int n = decltype(nc)::value;
            const unsigned suffix = (u / (unsigned)cpow(d, P - n)) % (unsigned)cpow(d, n - i);
            acc = fmaf(prefix_value<n>(ad), b[Sh::row_off(n - i) + suffix], acc);
        });
        // words (u, v), |v| = r >= 1: x = (u_{i+1:P}, v), a run of d^r floats of level P + r - i
        static_for<1, Sh::R + 1>([&](auto rc) __attribute__((always_inline)) {
            constexpr int r = decltype(rc)::value;
            constexpr int cnt = cpow(d, r);
            const float *bs = b + Sh::row_off(P + r - i) + (u % (unsigned)cpow(d, P - i)) * cnt;
#pragma unroll
            for (int v = 0; v < cnt; ++v) acc = fmaf(ad.s[Sh::sub_off(r) + v], bs[v], acc);
        });
        prefix_ref<i>(ad) = acc;
    });
    // the empty prefix (P == 0): the lane's root is the empty word, whose gradient is not needed
    // sub-tree words (u, v), |v| = r = 1 .. R-1, shallowest first: x = the rest of a deeper word
    static_for<1, Sh::R>([&](auto rc) __attribute__((always_inline)) {
        constexpr int r = decltype(rc)::value;
        constexpr int cnt = cpow(d, r);
        static_for<r + 1, Sh::R + 1>([&](auto qc) __attribute__((always_inline)) {
            constexpr int r2 = decltype(qc)::value;
            constexpr int tail = cpow(d, r2 - r);
            const float *bs = b + Sh::row_off(r2 - r);
#pragma unroll
            for (int v = 0; v < cnt; ++v) {
                float acc = ad.s[Sh::sub_off(r) + v];
#pragma unroll
                for (int x = 0; x < tail; ++x) acc = fmaf(ad.s[Sh::sub_off(r2) + v * tail + x], bs[x], acc);
                ad.s[Sh::sub_off(r) + v] = acc;
            }
        });
    });
}

// a lane's registers in LDS, register i of lane u at i * Q + u (consecutive lanes on consecutive banks)
template <int d, int N, int P>
__device__ __forceinline__ void store_private(float *buf, unsigned u, const Lane<d, N, P> &x)
{
    using Sh = Shape<d, N, P>;
#pragma unroll
    for (int i = 0; i < Sh::SZ; ++i) buf[i * Sh::Q + u] = x.s[i];
#pragma unroll
    for (int i = 0; i < Sh::NPRE; ++i) buf[(Sh::SZ + i) * Sh::Q + u] = x.pre[i];
}

template <int d, int N, int P>
__device__ __forceinline__ void load_private(const float *buf, unsigned u, Lane<d, N, P> &x)
{
    using Sh = Shape<d, N, P>;
#pragma unroll
    for (int i = 0; i < Sh::SZ; ++i) x.s[i] = buf[i * Sh::Q + u];
#pragma unroll
    for (int i = 0; i < Sh::NPRE; ++i) x.pre[i] = buf[(Sh::SZ + i) * Sh::Q + u];
}

// The sweep cut in time: one workgroup per path, C chunks of T increments side by side.
//   1. every chunk folds its increments from the identity: its own signature E_c                (T steps)
//   2. a scan from the left gives every prefix S_end(c) = E_0 (x) ... (x) E_c; the workgroup shares each product
//   3. the adjoint A_end(c) at the end of every chunk:
//      final mode  - a scan from the right gives X_c = E_{c+1} (x) ... (x) E_{C-1}, and every chunk pulls the
//                    upstream gradient back through X_c on its own                               (C products)
//      stream mode - a first sweep of every chunk from a zero adjoint gives what its own rows leave at its
//                    start; the lanes of chunk 0 then walk the chunks from the last to the first   (T steps, C products)
//   4. every chunk runs the reverse sweep over its own increments from (S_end(c), A_end(c))       (T steps)
// so the critical path is about 2 T (stream: 3 T) steps and 2 C short products instead of C T steps.
// PIPE (stream mode): the fetch of the upstream rows as a software pipeline, see sig_backward_kernel.
template <int d, int N, int P, bool STREAM, bool PIPE = false>
__global__ __launch_bounds__(256) void sig_backward_chunked_kernel(BackwardArgs A)
{
    static_assert(!PIPE || STREAM, "the pipelined fetch belongs to stream mode");
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr int TS = reduce_steps<d, P>();
    constexpr int ROW = chunk_row_floats<d, N, P>();
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int K = (int)(A.L - 1);
    const int C = A.groups;  // chunks per path
    const int T = (K + C - 1) / C;
    const int c_raw = tid / Q;
    const unsigned u = (unsigned)(tid - c_raw * Q);
    const bool active = c_raw < C;
    const int c = active ? c_raw : 0;
    const int64_t b = blockIdx.x;
    int steps = K - c * T;
    if (steps > T) steps = T;
    if (steps < 0 || !active) steps = 0;

    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    }

    float *tile = sig_backward_smem;                 // [K][d] increments, later their gradients
    float *rowsE = tile + (K * d + 3) / 4 * 4;       // [C][ROW] chunk signatures, later the parked partial sums
    float *rowsS = rowsE + C * ROW;                  // [C][ROW] prefixes S_end(c), then (final mode) the X_c
    float *rowsA = rowsS + C * ROW;                  // stream mode: [C][private_floats] adjoints, lane layout
    for (int i = tid; i < K * d; i += nthr) {
        const float *x = A.path + b * A.L * d + i;
        tile[i] = x[d] - x[0];
    }
    __syncthreads();

    // 1. chunk signatures
    Lane<d, N, P> ln, ad;
    identity_state<d, N, P>(ln);
    for (int t = 0; t < steps; ++t) {
        Inc<d, P> inc;
        load_inc<d, P>(inc, tile + (c * T + t) * d, letter);
        fused_step<d, N, P>(ln, inc);
    }
    if (active) store_state<d, N, P>(rowsE + c * ROW, u, ln);
    __syncthreads();
    // 2. prefixes S_end(c) = E_0 (x) ... (x) E_c, left to right; the whole workgroup shares each product
    //    (one work item per parent word, see RowProduct)
    using RP = RowProduct<d, N>;
    for (int x = tid; x < D; x += nthr) rowsS[x] = rowsE[x];
    __syncthreads();
    for (int c2 = 1; c2 < C; ++c2) {
        for (int x = tid; x < RP::ITEMS; x += nthr)
            RP::item(rowsS + (c2 - 1) * ROW, rowsE + c2 * ROW, rowsS + c2 * ROW, x);
        __syncthreads();
    }
    if (active) load_state<d, N, P>(rowsS + c * ROW, u, ln);
    __syncthreads();
    // The sweep of this lane's chunk from (ln, ad) = (S_end(c), A_end(c)), t = T-1 .. 0 for every chunk alike
    // (chunks with fewer increments idle in the surplus iterations).  EMIT: the partial sums of d(loss)/d(dX) are
    // parked in rowsE, added up and written over the increments.  Stream mode adds row k's upstream gradient
    // before step k; the rows are fetched PD steps ahead (see the unchunked kernel).
    float *mypark = rowsE + c * ROW;
    using Pk = Park<d, P>;
    constexpr int PD = !STREAM ? 1 : Sh::SZ <= 24 ? 4 : Sh::SZ <= 48 ? 2 : 1;
    const PrefixOwner<d, N, P> owner(u);
    auto sweep = [&](auto emit_tag) __attribute__((always_inline)) {
        constexpr bool EMIT = decltype(emit_tag)::value;
        Lane<d, N, P> up[PD];
        // Stream mode: the upstream rows of the chunk, one fetch per step in the order of the sweep, PD steps
        // ahead and without conditions (see the PIPE sweep of sig_backward_kernel): row min(c T + max(t, 0), K - 1)
        // for t = T - 1, T - 2, ...; rows of steps that the chunk does not have are fetched and not used.
        const int top = c * T + T - 1 < K - 1 ? c * T + T - 1 : K - 1;
        [[maybe_unused]] const float *next_row = A.grad_out + (b * K + top) * D;
        [[maybe_unused]] int tn = T - 1;
        [[maybe_unused]] auto fetch = [&](Lane<d, N, P> &dst) __attribute__((always_inline)) {
            load_adjoint<d, N, P, false, false>(next_row, u, dst);
            next_row -= (tn > 0 && c * T + tn <= K - 1) ? D : 0;
            --tn;
        };
        if constexpr (STREAM) {
            static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                identity_state<d, N, P>(up[j]);
                if constexpr (PIPE) {
                    fetch(up[j]);
                } else {
                    const int t = T - 1 - j;
                    if (t >= 0 && t < steps)
                        load_adjoint<d, N, P, false, false>(A.grad_out + (b * K + (c * T + t)) * D, u, up[j]);
                }
            });
        }
        // one step of the sweep; `refill` runs between the arithmetic and the parked sums (the plain fetch of the
        // row that replaces `row`)
        auto one = [&](int t, const Lane<d, N, P> &row, auto refill) __attribute__((always_inline)) {
            const int ts = (T - 1 - t) % TS;
            float dbar[d];
#pragma unroll
            for (int a = 0; a < d; ++a) dbar[a] = 0.0f;
            if (t < steps) {
                const int k = c * T + t;
                if constexpr (STREAM) add_row<d, N, P>(ad, row, owner);
                Inc<d, P> inc, neg;
                load_inc<d, P>(inc, tile + k * d, letter);
#pragma unroll
                for (int a = 0; a < d; ++a) neg.v[a] = -inc.v[a];
                neg.du[0] = 0.0f;
#pragma unroll
                for (int m = 0; m < P; ++m) neg.du[m] = -inc.du[m];
                if (k > 0) fused_step<d, N, P>(ln, neg);
                else identity_state<d, N, P>(ln);
                backward_step<d, N, P>(ln, ad, inc, letter, dbar);
            }
            refill();
            if constexpr (EMIT) {
                if (active) {
#pragma unroll
                    for (int a = 0; a < d; ++a) mypark[Pk::at(ts, (int)u, a)] = dbar[a];
                }
                if (ts == TS - 1 || t == 0) {
                    __syncthreads();
                    if (active) {
                        for (int col = (int)u; col < (ts + 1) * d; col += Q) {
                            const int tp = col / d, a = col - tp * d;
                            const int tt = t + (ts - tp);  // step of this chunk the column belongs to
                            if (tt < steps) {
                                float sum = 0.0f;
                                for (int q = 0; q < Q; ++q) sum += mypark[Pk::at(tp, q, a)];
                                tile[(c * T + tt) * d + a] = sum;
                            }
                        }
                    }
                    __syncthreads();
                }
            }
        };
        if constexpr (PIPE) {
            int t0 = T - 1;
            for (; t0 >= PD - 1; t0 -= PD) {
                static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
                    constexpr int j = decltype(jc)::value;
                    one(t0 - j, up[j], [] {});
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(up[j]);
                    __builtin_amdgcn_sched_barrier(0x81);
                });
            }
            static_for<0, PD - 1>([&](auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                if (t0 - j >= 0) one(t0 - j, up[j], [] {});
            });
        } else {
            for (int t0 = T - 1; t0 >= 0; t0 -= PD) {
                static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
                    constexpr int j = decltype(jc)::value;
                    const int t = t0 - j;
                    if (t >= 0) {
                        one(t, up[j], [&]() __attribute__((always_inline)) {
                            if constexpr (STREAM) {
                                const int tnext = t - PD;
                                if (tnext >= 0 && tnext < steps)
                                    load_adjoint<d, N, P, false, false>(A.grad_out + (b * K + (c * T + tnext)) * D, u, up[j]);
                            }
                        });
                    }
                });
            }
        }
    };

    identity_state<d, N, P>(ad);
    if (P == 0) ad.s[0] = 0.0f;
    if constexpr (!STREAM) {
        // 3. the adjoint at the end of chunk c is the upstream gradient pulled back through everything after
        //    the chunk: A_end(c) = transpose of (. (x) X_c) applied to d(loss)/d(out), X_c = E_{c+1} (x) ... (x)
        //    E_{C-1}.  The X_c are a scan from the right (X_{C-1} is the identity: a row of zeros); then every
        //    chunk pulls the gradient back on its own.
        for (int x = tid; x < D; x += nthr) rowsS[(C - 1) * ROW + x] = 0.0f;
        __syncthreads();
        for (int c2 = C - 1; c2 >= 1; --c2) {
            for (int x = tid; x < RP::ITEMS; x += nthr)
                RP::item(rowsE + c2 * ROW, rowsS + c2 * ROW, rowsS + (c2 - 1) * ROW, x);
            __syncthreads();
        }
        if (active) {
            load_adjoint<d, N, P, false>(A.grad_out + b * D, u, ad);
            if (c < C - 1) reg_adjoint_product<d, N, P>(ad, rowsS + c * ROW, u);
        }
        __syncthreads();
        // 4. the sweep of every chunk; rowsE now parks the partial sums
        sweep(std::true_type{});
    } else {
        // Stream mode: every row has its own upstream gradient, so what reaches the end of chunk c from the later
        // chunks is r_{c+1} + transpose of (. (x) E_{c+1}) applied to A_end(c+1), where r_c is what chunk c's own
        // rows leave at its start.
        // 3a. a first sweep from a zero adjoint, without output, gives r_c
        sweep(std::false_type{});
        if (active) store_private<d, N, P>(rowsA + c * private_floats<d, N, P>(), u, ad);
        __syncthreads();
        // 3b. the lanes of chunk 0 walk the chunks from the last to the first: A_end(c-1) = r_c + pull-back of
        //     A_end(c) through E_c; A_end(c) takes r_c's place in LDS
        if (active && c == 0) {
            Lane<d, N, P> run, r;
            identity_state<d, N, P>(run);
            if (P == 0) run.s[0] = 0.0f;
            for (int c2 = C - 1; c2 >= 1; --c2) {
                float *slot = rowsA + c2 * private_floats<d, N, P>();
                load_private<d, N, P>(slot, u, r);
                store_private<d, N, P>(slot, u, run);
                reg_adjoint_product<d, N, P>(run, rowsE + c2 * ROW, u);
#pragma unroll
                for (int i = 0; i < Sh::SZ; ++i) run.s[i] += r.s[i];
#pragma unroll
                for (int i = 0; i < Sh::NPRE; ++i) run.pre[i] += r.pre[i];
            }
            store_private<d, N, P>(rowsA, u, run);
        }
        __syncthreads();
        // 4. the second sweep, from the true adjoint, with output (rowsE parks the partial sums from here on)
        if (active) {
            load_state<d, N, P>(rowsS + c * ROW, u, ln);
            load_private<d, N, P>(rowsA + c * private_floats<d, N, P>(), u, ad);
        }
        __syncthreads();
        sweep(std::true_type{});
    }

    const int out_row = (int)A.L * d;
    for (int i = tid; i < out_row; i += nthr) {
        const float before = i >= d ? tile[i - d] : 0.0f;
        const float after = i < K * d ? tile[i] : 0.0f;
        A.grad_path[b * out_row + i] = before - after;
    }
}

}  // namespace onchip

// d(loss)/dX_j = sum over the slices, in order, of (d/d(dX_{j-1}) - d/d(dX_j))
__global__ __launch_bounds__(256) void sig_backward_slices_finish_kernel(const float *part, float *grad_path, int64_t B,
                                                                         int64_t L, int d, int slices)
{
    const int64_t out_row = L * d, row_floats = (L - 1) * d;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= B * out_row) return;
    const int64_t b = e / out_row, r = e - b * out_row;
    float sum = 0.0f;
    for (int s = 0; s < slices; ++s) {
        const float *t = part + (b * slices + s) * row_floats;
        const float before = r >= d ? t[r - d] : 0.0f;
        const float after = r < row_floats ? t[r] : 0.0f;
        sum += before - after;
    }
    grad_path[e] = sum;
}

hipError_t launch_backward_finish(const float *part, float *grad_path, int64_t B, int64_t L, int d, int slices,
                                  hipStream_t st)
{
    const int64_t blocks = (B * L * d + 255) / 256;
    if (blocks <= 0 || blocks > INT32_MAX) return hipErrorInvalidValue;
    hipLaunchKernelGGL(sig_backward_slices_finish_kernel, dim3((unsigned)blocks), dim3(256), 0, st, part, grad_path, B, L,
                       d, slices);
    return hipGetLastError();
}

namespace onchip {

// LDS of the launch (what backward_fits compares with the limit): with the fewest parked steps if need be
template <int d, int N, int P>
int64_t backward_sliced_lds_bytes(int64_t L, int)
{
    const int ts = backward_sliced_steps<d>(L);
    return backward_sliced_bytes_with<d>(L, ts > 0 ? ts : 1);
}

template <int d, int N, int P>
int64_t backward_sliced_scratch_floats(int64_t B, int64_t L)
{
    constexpr int slices = (Shape<d, N, P>::Q + kSliceLanes - 1) / kSliceLanes;
    return B * slices * (L - 1) * d;
}

template <int d, int N, int P>
hipError_t backward_sliced_launch(const BackwardArgs &A0, float *scratch, int, int, hipStream_t st)
{
    constexpr int slices = (Shape<d, N, P>::Q + kSliceLanes - 1) / kSliceLanes;
    BackwardArgs A = A0;
    int64_t points = A.L;   // points of what is staged in LDS at a time
    if (backward_sliced_steps<d>(A.L) < 1) {
        // the path's increments do not fit LDS at once: the workgroup walks tiles of kTiledSteps increments
        A.tiled = 1;
        A.seg_steps = kTiledSteps;
        A.segs = (int32_t)((A.L - 1 + kTiledSteps - 1) / kTiledSteps);
        points = kTiledSteps + 1;
    }
    const int ts = backward_sliced_steps<d>(points);
    const int64_t lds = backward_sliced_bytes_with<d>(points, ts > 0 ? ts : 1);
    const int64_t grid = A.B * slices;
    if (!scratch || ts < 1 || lds > kMaxLdsBytes || grid <= 0 || grid > INT32_MAX || (A.L - 1) / kTiledSteps > INT32_MAX / 2)
        return hipErrorInvalidValue;
    if (A.stream_flag)
        hipLaunchKernelGGL((sig_backward_sliced_kernel<d, N, P, true>), dim3((unsigned)grid), dim3(kSliceLanes), (size_t)lds, st, A, scratch, ts);
    else
        hipLaunchKernelGGL((sig_backward_sliced_kernel<d, N, P, false>), dim3((unsigned)grid), dim3(kSliceLanes), (size_t)lds, st, A, scratch, ts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_backward_finish(scratch, A.grad_path, A.B, A.L, d, slices, st);
}

// the register sweep needs device scratch only for paths it has to walk in tiles: the sums over the increments
// The increments of a path fit LDS, but so few paths' worth of them that at most half of the lanes of 256 threads
// would hold a path (long paths: (5,4) with 2,000 points takes 40 KB, one path and 25 lanes per workgroup).  On a batch
// that fills the chip the plain sweep then runs 1.4-5.7 times slower than either alternative: the sweep cut in time
// inside the workgroup (one path per workgroup, its chunks side by side), which wins for kernels with fewer than 16
// lanes per path (measured 1.15-1.6x over the tiled walk), and the walk in tiles of kTiledSteps increments, which
// wins for the others ((5,4) with 2,000 points at 16,384 paths: plain 24.3 ms, cut in time 10.9 ms, tiles 6.0 ms).
constexpr int kStarvedChunkedMaxLanes = 16;
template <int d, int N, int P>
bool backward_starved(int64_t L)
{
    constexpr int Q = Shape<d, N, P>::Q;
    if (backward_lds_bytes<d, N, P>(L, 1) > kMaxLdsBytes) return false;
    int G = 256 / Q;
    while (G > 1 && backward_lds_bytes<d, N, P>(L, G) > kMaxLdsBytes) --G;
    return G * Q * 2 <= 256;
}

// Kernels with fewer than 16 lanes per path whose LDS holds fewer paths than a workgroup has lanes for (the
// increments of a path take L d floats for a handful of lanes): on a batch that needs the plain sweep's resident
// workgroups more than one and a half times over (final mode), the paths are walked in short tiles instead, sized so that a full
// workgroup's tiles take 32 KB and two or more workgroups stay on a CU.  Measured: (5,3), 100 points, 65,536 paths
// 461 -> 303 us; stream mode, 256 points, 16,384 paths 1,001 -> 685; (6,3), (7,3), (3,4), (2,6) at 100 points
// 1.25-1.35x; on a chip that the plain sweep fills about once it loses 20-40 %.  Returns the tile length, 0 if the
// shape is not of this kind.
template <int d, int N, int P>
int backward_short_tile(int64_t L, int threads)
{
    constexpr int Q = Shape<d, N, P>::Q;
    if (Q >= kStarvedChunkedMaxLanes || threads < Q || backward_lds_bytes<d, N, P>(L, 1) > kMaxLdsBytes) return 0;
    const int full = threads / Q;
    int fit = full;
    while (fit > 1 && backward_lds_bytes<d, N, P>(L, fit) > kMaxLdsBytes) --fit;
    if (fit >= full) return 0;
    int T = kTiledSteps;
    while (T > 16 && backward_lds_bytes<d, N, P>(T + 1, full) > 32 * 1024) T -= 8;
    return T < L - 1 ? T : 0;
}

template <int d, int N, int P>
int64_t backward_tiled_scratch_floats(int64_t B, int64_t L)
{
    constexpr bool tiles_when_starved = Shape<d, N, P>::Q >= kStarvedChunkedMaxLanes;
    const bool starved = tiles_when_starved && backward_starved<d, N, P>(L);
    if (backward_short_tile<d, N, P>(L, 256) > 0) return B * (L - 1) * d;
    return backward_lds_bytes<d, N, P>(L, 1) <= kMaxLdsBytes && !starved ? 0 : B * (L - 1) * d;
}

// wavefronts per SIMD that the registers of a kernel allow (512 registers per lane of a SIMD, allocated in eights,
// at most eight wavefronts); asked of the runtime once per kernel
template <typename Kernel>
int waves_by_registers(Kernel kernel)
{
    hipFuncAttributes fa{};
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(kernel)) != hipSuccess || fa.numRegs <= 0) {
        (void)hipGetLastError();   // not an error of the launch that follows
        return 8;
    }
    const int w = 512 / ((fa.numRegs + 7) / 8 * 8);
    return w > 8 ? 8 : (w < 1 ? 1 : w);
}

// Workgroups of the register sweep that stay resident on a CU: what its LDS holds (the increments of the
// workgroup's paths plus the parked sums), then what the registers allow.
template <int d, int N, int P>
int64_t resident_sweep_workgroups(int64_t L, int stream_flag, int threads, int groups, int park_steps)
{
    static const int regs_final = waves_by_registers(&sig_backward_kernel<d, N, P, false>);
    static const int regs_stream = waves_by_registers(&sig_backward_kernel<d, N, P, true>);
    const int64_t by_regs = (stream_flag ? regs_stream : regs_final) * 4 / ((threads + kWave - 1) / kWave);
    const int64_t by_lds = kCuLdsBytes / backward_lds_bytes<d, N, P>(L, groups, park_steps);
    return by_lds < by_regs ? by_lds : by_regs;
}

template <int d, int N, int P>
hipError_t backward_launch(const BackwardArgs &A0, float *scratch, int threads, int cus, hipStream_t st)
{
    constexpr int Q = Shape<d, N, P>::Q;
    if (threads < Q || threads > 256 || threads % kWave) return hipErrorInvalidValue;
    BackwardArgs A = A0;
    // Lanes below which the sweep is cut in time inside the workgroup (one path per workgroup).  The cut sweeps every
    // increment twice (three times in stream mode) and multiplies rows between the chunks, so it pays only while the
    // plain sweep would leave the chip nearly empty: final mode below one wavefront per SIMD, half of one for paths of
    // up to 128 increments of kernels with fewer than 64 lanes per path (14 shapes x 32 ... 500 points x 128 ... 8,192 paths against a limit of two: (5,4), 100 points,
    // 4,096 paths 208 -> 80 us, (3,5), 32 points, 8,192 paths 120 -> 31; long paths between half a wavefront and one
    // lose 10-45 % with the lower limit); stream mode below a wavefront per CU.
    const int64_t full_lanes = (int64_t)cus * 4 * kWave * 2;
    const int64_t few_lanes = A.stream_flag ? (int64_t)cus * kWave
                              : (A.L - 1 <= 128 && Q < kWave) ? (int64_t)cus * 4 * kWave / 2 : (int64_t)cus * 4 * kWave;
    // A shape that fills at most half of a workgroup's lanes (see backward_starved) ...
    bool half_empty = backward_starved<d, N, P>(A.L);
    if (half_empty && Q < kStarvedChunkedMaxLanes && N >= 3) {
        // ... unless, for the kernels with few lanes per path, the plain sweep still keeps enough lanes on a CU.  The
        // cut in time sweeps every increment three times (stream mode; twice in final mode) and multiplies whole rows
        // between the chunks, which costs more the deeper the signature: measured on 14 shapes x 64 ... 2,000 points x
        // 2,048 ... 32,768 paths, the plain sweep is 1.1-7x faster above these lane counts (stream mode, 256 points,
        // 8,192 paths: (2,6) 2,504 -> 501 us, (3,4) 843 -> 261, (5,3) 636 -> 426) and up to 5x slower below them; at
        // depth 2 the cut always wins.
        int G = threads / Q;
        while (G > 1 && backward_lds_bytes<d, N, P>(A.L, G) > kMaxLdsBytes) --G;
        const int64_t lanes = resident_sweep_workgroups<d, N, P>(A.L, A.stream_flag, threads, G, 0) * G * Q;
        const int64_t enough = !A.stream_flag ? 224 : N >= 4 ? 56 : 112;
        if (lanes >= enough) half_empty = false;
    }
    // ... keeps the cut further: final mode up to two wavefronts per SIMD; stream mode, where the row products between
    // the chunks are cheap (depth up to 3, or rows of up to 400 floats), up to two wavefronts per CU, four for kernels
    // with 64 lanes per path or more ((4,4), 500 points, 1,024 paths 381 -> 269 us; (8,3), 256 points, 512 paths 176
    // -> 111; (10,3), 512 paths 239 -> 141; (5,4), (6,4), (4,5) lose 15-35 % there).  From there on it is walked in
    // tiles, or cut anyway if it has fewer than 16 lanes per path.
    constexpr bool cheap_products = N <= 3 || Shape<d, N, P>::D <= 400;
    const int64_t half_empty_lanes = !A.stream_flag ? full_lanes
                                     : cheap_products ? few_lanes * (Q >= kWave ? 4 : 2) : few_lanes;
    const bool starved = half_empty && A.B * Q >= half_empty_lanes;
    const bool starved_tiles = starved && Q >= kStarvedChunkedMaxLanes && scratch;
    const bool starved_chunks = starved && Q < kStarvedChunkedMaxLanes;
    // few-lane kernels that LDS keeps from filling their workgroups, on a batch that needs the plain sweep's resident
    // workgroups more than one and a half times over: short tiles (see backward_short_tile)
    int short_tile = 0;
    if (scratch && !half_empty && A.B * Q >= few_lanes) {
        short_tile = backward_short_tile<d, N, P>(A.L, threads);
        if (short_tile) {
            int fit = threads / Q;
            while (fit > 1 && backward_lds_bytes<d, N, P>(A.L, fit) > kMaxLdsBytes) --fit;
            const int64_t resident = resident_sweep_workgroups<d, N, P>(A.L, A.stream_flag, threads, fit, 0) * fit * Q * cus;
            // (stream mode: from two and a half times over, unless the lane state is large; at twice over (2,3),
            // (2,4), (3,4) and (6,3) with 256 points lose 15-25 % to the plain sweep, (2,6) gains 2x)
            const int64_t times2 = !A.stream_flag || Shape<d, N, P>::SZ >= 48 ? 3 : 5;
            if (A.B * Q * 2 < resident * times2) short_tile = 0;
        }
    }
    if (backward_lds_bytes<d, N, P>(A.L, 1) > kMaxLdsBytes || starved_tiles || short_tile) {
        // the path's increments do not fit LDS at once (or too few paths' do): tiles of increments, walked by one workgroup
        if (!scratch || (A.L - 1) / kTiledSteps > INT32_MAX / 2) return hipErrorInvalidValue;
        const int tile = short_tile ? short_tile : kTiledSteps;
        A.tiled = 1;
        A.seg_steps = tile;
        A.segs = (int32_t)((A.L - 1 + tile - 1) / tile);
        A.seg_part = scratch;
        int G = threads / Q;
        const int64_t per_cu = (A.B + cus - 1) / (cus > 0 ? cus : 1);
        if ((int64_t)G > per_cu) G = per_cu > 1 ? (int)per_cu : 1;
        while (G > 1 && backward_lds_bytes<d, N, P>(tile + 1, G) > kMaxLdsBytes) --G;
        if (per_cu > G) {   // the same number of paths on every CU, see below
            const int64_t rounds = (per_cu + G - 1) / G;
            G = (int)((per_cu + rounds - 1) / rounds);
        }
        const size_t lds = (size_t)backward_lds_bytes<d, N, P>(tile + 1, G);
        const int64_t grid = (A.B + G - 1) / G;
        if (lds > (size_t)kMaxLdsBytes || grid <= 0 || grid > INT32_MAX) return hipErrorInvalidValue;
        A.groups = G;
        if (A.stream_flag)
            hipLaunchKernelGGL((sig_backward_tiled_kernel<d, N, P, true>), dim3((unsigned)grid), dim3(threads), lds, st, A);
        else
            hipLaunchKernelGGL((sig_backward_tiled_kernel<d, N, P, false>), dim3((unsigned)grid), dim3(threads), lds, st, A);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_backward_finish(scratch, A.grad_path, A.B, A.L, d, 1, st);
    }
    // Few paths (fewer lanes than two wavefronts per SIMD): cut the sweep in time, one workgroup per path with
    // as many chunks as its threads and LDS hold, at least eight increments each.
    // (stream mode reads the upstream gradient twice when cut, so only far below one wavefront per SIMD)
    if ((A.B * Q < few_lanes || (half_empty && A.B * Q < half_empty_lanes) || starved_chunks) && A.B <= INT32_MAX) {
        const int C = backward_chunks<d, N, P>(A.L, A.stream_flag, threads);
        if (C > 1) {
            A.groups = C;
            const size_t lds = (size_t)backward_chunked_lds_bytes<d, N, P>(A.L, C, A.stream_flag);
            // (stream mode fetches the upstream rows as a pipeline where four rows fit the registers and the launch
            // leaves the SIMDs a wavefront each or less: (4,4), 256 points, 128 paths 45 -> 37 us; with two rows,
            // or on fuller chips, the plain fetch is up to a quarter faster)
            constexpr bool kFourRows = Shape<d, N, P>::SZ <= 24;
            const int64_t busy_wavefronts = A.B * (((int64_t)C * Q + kWave - 1) / kWave);
            if (A.stream_flag && kFourRows && busy_wavefronts <= (int64_t)cus * 4)
                hipLaunchKernelGGL((sig_backward_chunked_kernel<d, N, P, true, kFourRows>), dim3((unsigned)A.B), dim3(threads), lds, st, A);
            else if (A.stream_flag)
                hipLaunchKernelGGL((sig_backward_chunked_kernel<d, N, P, true>), dim3((unsigned)A.B), dim3(threads), lds, st, A);
            else
                hipLaunchKernelGGL((sig_backward_chunked_kernel<d, N, P, false>), dim3((unsigned)A.B), dim3(threads), lds, st, A);
            return hipGetLastError();
        }
    }
    // paths per workgroup: as many as the threads hold, fewer if their LDS does not fit, spread over the CUs first
    int G = threads / Q;
    const int64_t per_cu = (A.B + cus - 1) / (cus > 0 ? cus : 1);
    if ((int64_t)G > per_cu) G = per_cu > 1 ? (int)per_cu : 1;
    while (G > 1 && backward_lds_bytes<d, N, P>(A.L, G) > kMaxLdsBytes) --G;
    // ... and the same number of paths on every CU: with 16 paths per CU and room for 12 per workgroup, workgroups of 8
    // put two on every CU where workgroups of 12 put two on a third of the CUs and one on the rest
    if (per_cu > G) {
        const int64_t rounds = (per_cu + G - 1) / G;
        G = (int)((per_cu + rounds - 1) / rounds);
    }
    // Parked steps: the most that is useful, unless fewer keep more workgroups resident on a batch that fills
    // the chip.  Measured at kShortPark against the most: (5,4) at 65,536 paths 749 -> 698 us, (6,4) 352 -> 333,
    // (8,3) 895 -> 657, (5,4) of 300 points 1199 -> 950; where the residency is the same (stream mode, whose
    // registers allow two or three wavefronts per SIMD) the shorter park only adds barriers (1-3 % slower).
    // (Smaller workgroups for shapes whose 64 KiB hold fewer paths than 256 threads, and fewer paths per workgroup,
    // were measured too: between 11 % faster and 10 % slower with no rule that told the two apart.)
    int short_park = 0;
    if constexpr (reduce_steps<d, P>() > kShortPark) {
        if (backward_lds_bytes<d, N, P>(A.L, G) <= kMaxLdsBytes) {
            const int64_t longest = resident_sweep_workgroups<d, N, P>(A.L, A.stream_flag, threads, G, 0);
            if (per_cu > G * longest &&
                resident_sweep_workgroups<d, N, P>(A.L, A.stream_flag, threads, G, kShortPark) > longest)
                short_park = 1;
        }
    }
    const int park_steps = short_park ? kShortPark : 0;
    if (backward_lds_bytes<d, N, P>(A.L, G, park_steps) > kMaxLdsBytes) return hipErrorInvalidValue;
    A.groups = G;
    const int64_t grid = (A.B + G - 1) / G;
    if (grid <= 0 || grid > INT32_MAX) return hipErrorInvalidValue;
    const size_t lds = (size_t)backward_lds_bytes<d, N, P>(A.L, G, park_steps);
    if constexpr (reduce_steps<d, P>() > kShortPark) {
        if (short_park) {
            if (A.stream_flag)
                hipLaunchKernelGGL((sig_backward_kernel<d, N, P, true, false, true, kShortPark>), dim3((unsigned)grid), dim3(threads), lds, st, A);
            else
                hipLaunchKernelGGL((sig_backward_kernel<d, N, P, false, false, true, kShortPark>), dim3((unsigned)grid), dim3(threads), lds, st, A);
            return hipGetLastError();
        }
    }
    // Stream mode on a launch that leaves the SIMDs a wavefront each or less: the upstream rows as a software pipeline
    // (measured against the plain fetch: (4,4), 256 points, 1,024 paths 156 -> 114 us; (3,5), 100 points, 4,096
    // paths 162 -> 134; with more wavefronts than SIMDs it loses 3-10 %: its rows in flight evict each other's
    // lines from the vector cache, whose requests to L2 rise by a fifth).
    const int64_t busy_wavefronts = grid * (((int64_t)G * Q + kWave - 1) / kWave);
    if (A.stream_flag && busy_wavefronts <= (int64_t)cus * 4)
        hipLaunchKernelGGL((sig_backward_kernel<d, N, P, true, false, true, 0, true>), dim3((unsigned)grid), dim3(threads), lds, st, A);
    else if (A.stream_flag)
        hipLaunchKernelGGL((sig_backward_kernel<d, N, P, true>), dim3((unsigned)grid), dim3(threads), lds, st, A);
    else
        hipLaunchKernelGGL((sig_backward_kernel<d, N, P, false>), dim3((unsigned)grid), dim3(threads), lds, st, A);
    return hipGetLastError();
}

}  // namespace onchip

namespace {
struct BackwardEntry {
    int d, depth;
    hipError_t (*launch)(const onchip::BackwardArgs &, float *, int, int, hipStream_t);
    int64_t (*lds_bytes)(int64_t, int);
    int64_t (*scratch_floats)(int64_t, int64_t);
};
#define SIG_BACKWARD_ENTRY(d, N, P) \
    {d, N, &onchip::backward_launch<d, N, P>, &onchip::backward_lds_bytes<d, N, P>, &onchip::backward_tiled_scratch_floats<d, N, P>},
#define SIG_BACKWARD_SLICED(d, N, P)                                                                  \
    {d, N, &onchip::backward_sliced_launch<d, N, P>, &onchip::backward_sliced_lds_bytes<d, N, P>, \
     &onchip::backward_sliced_scratch_floats<d, N, P>},
const BackwardEntry kBackward[] = {
    SIG_BACKWARD_SHAPES(SIG_BACKWARD_ENTRY, SIG_BACKWARD_SLICED)
    {0, 0, nullptr, nullptr, nullptr},
};
const BackwardEntry *find_backward(int d, int depth)
{
    for (const BackwardEntry *e = kBackward; e->launch; ++e)
        if (e->d == d && e->depth == depth) return e;
    return nullptr;
}
}  // namespace

bool backward_available(int d, int depth) { return find_backward(d, depth) != nullptr; }

bool backward_fits(int d, int depth, int64_t L)
{
    const BackwardEntry *e = find_backward(d, depth);
    return e && e->lds_bytes(L, 1) <= kMaxLdsBytes;
}

bool backward_tiles_fit(int d, int depth)
{
    const BackwardEntry *e = find_backward(d, depth);
    return e && e->lds_bytes(onchip::kTiledSteps + 1, 1) <= kMaxLdsBytes;
}

int64_t backward_scratch_floats(int d, int depth, int64_t B, int64_t L)
{
    const BackwardEntry *e = find_backward(d, depth);
    return e ? e->scratch_floats(B, L) : 0;
}

hipError_t launch_backward(const float *path, const float *sig, const float *grad_out, float *grad_path, float *scratch,
                           int64_t B, int64_t L, int d, int depth, int stream_flag, int cus, hipStream_t st)
{
    const BackwardEntry *e = find_backward(d, depth);
    if (!e) return hipErrorInvalidValue;
    onchip::BackwardArgs A{};
    A.path = path;
    A.sig = sig;
    A.grad_out = grad_out;
    A.grad_path = grad_path;
    A.B = B;
    A.L = L;
    A.stream_flag = stream_flag;
    return e->launch(A, scratch, 256, cus, st);
}

}  // namespace sig

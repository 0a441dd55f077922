// Device code shared by the reverse-sweep translation units: the transposed fused step on a lane's sub-tree, the
// loaders of adjoint rows, the layout of the parked per-step sums, and the sliced sweep kernel (one workgroup per
// path, slice of its lanes and, when the sweep is cut in time, segment of its increments).  The method is
// described at the top of sig_backward.hip.
#ifndef SIG_BACKWARD_H_
#define SIG_BACKWARD_H_

#include "sig_internal.h"
#include "sig_onchip.h"

namespace sig {
namespace onchip {

// value / reference of the lane's copy of the prefix word u_{1:m}, m = 1 .. P (u itself is s[0])
template <int m, int d, int N, int P>
__device__ __forceinline__ float prefix_value(const Lane<d, N, P> &x)
{
    if constexpr (m < P) return x.pre[m - 1];
    else return x.s[0];
}
template <int m, int d, int N, int P>
__device__ __forceinline__ float &prefix_ref(Lane<d, N, P> &x)
{
    if constexpr (m < P) return x.pre[m - 1];
    else return x.s[0];
}

// Transposed chain n inside a lane's sub-tree.  The node has index idx in sub-level r and forward chain
// value g; returns the adjoint of g.  s = S_{k-1} (read only), ad = adjoint (updated in place),
// dbar[a] accumulates d(loss)/dv[a].
template <int d, int N, int P, int n, int r>
struct Ascend {
    using Sh = Shape<d, N, P>;
    static __device__ __forceinline__ float run(const float (&s)[Sh::SZ], float (&ad)[Sh::SZ],
                                                const float (&dls)[Sh::R][d], float (&dbar)[d], float g, int idx)
    {
        constexpr int tgt = n - P;  // sub-level of the chain's target
        constexpr int m = r + 1;    // sub-level of this node's children
        float gb = 0.0f;
        if constexpr (m == tgt) {
#pragma unroll
            for (int a = 0; a < d; ++a) {
                const float up = ad[Sh::sub_off(tgt) + idx * d + a];
                gb = fmaf(up, dls[0][a], gb);
                dbar[a] = fmaf(up, g, dbar[a]);
            }
        } else {
            constexpr int c = tgt - r;  // the forward step divides v by this on the way to the children
            const float gs = g * (1.0f / (float)c);
#pragma unroll
            for (int a = 0; a < d; ++a) {
                const int child = idx * d + a;
                const float gc = fmaf(g, dls[c - 1][a], s[Sh::sub_off(m) + child]);
                const float cb = Ascend<d, N, P, n, m>::run(s, ad, dls, dbar, gc, child);
                ad[Sh::sub_off(m) + child] += cb;
                gb = fmaf(cb, dls[c - 1][a], gb);
                dbar[a] = fmaf(cb, gs, dbar[a]);
            }
        }
        return gb;
    }
};

// Transpose of the fused step: ln = S_{k-1}, ad = A_k on entry and A_{k-1} on return; dbar (zeroed here)
// receives this lane's part of d(loss)/dv.
template <int d, int N, int P>
__device__ __forceinline__ void backward_step(const Lane<d, N, P> &ln, Lane<d, N, P> &ad, const Inc<d, P> &inc,
                                              const int *letter, float (&dbar)[d])
{
    using Sh = Shape<d, N, P>;
    float dls[Sh::R][d];
#pragma unroll
    for (int a = 0; a < d; ++a) dls[0][a] = inc.v[a];
#pragma unroll
    for (int c = 1; c < Sh::R; ++c)
#pragma unroll
        for (int a = 0; a < d; ++a) dls[c][a] = inc.v[a] * (1.0f / (float)(c + 1));
#pragma unroll
    for (int a = 0; a < d; ++a) dbar[a] = 0.0f;
    float dbu[P > 0 ? P : 1];  // adjoint of inc.du[m-1] = v[u_m]
#pragma unroll
    for (int m = 0; m < (P > 0 ? P : 1); ++m) dbu[m] = 0.0f;

    static_for<1, N + 1>([&](auto nc) __attribute__((always_inline)) {
        constexpr int n = decltype(nc)::value;
        constexpr int mtop = (n - 1 < P) ? n - 1 : P;
        // forward values of the chain along the lane's own prefix
        float gp[P + 1];
        gp[0] = 1.0f;
        static_for<1, mtop + 1>([&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value;
            gp[m] = fmaf(gp[m - 1], inc.du[m - 1] * (1.0f / (float)(n - m + 1)), prefix_value<m>(ln));
        });
        float gb;  // adjoint of gp[mtop]
        if constexpr (n <= P) {
            const float up = prefix_value<n>(ad);
            gb = up * inc.du[n - 1];
            dbu[n - 1] = fmaf(up, gp[n - 1], dbu[n - 1]);
        } else {
            gb = Ascend<d, N, P, n, 0>::run(ln.s, ad.s, dls, dbar, gp[P], 0);
        }
        static_for<0, mtop>([&](auto qc) __attribute__((always_inline)) {
            constexpr int m = mtop - decltype(qc)::value;  // mtop .. 1
            prefix_ref<m>(ad) += gb;
            constexpr float c = 1.0f / (float)(n - m + 1);
            dbu[m - 1] = fmaf(gb * c, gp[m - 1], dbu[m - 1]);
            gb = gb * (inc.du[m - 1] * c);
        });
    });
    // v[u_m] is component letter[m-1] of v
    static_for<0, P>([&](auto mc) __attribute__((always_inline)) {
        constexpr int m = decltype(mc)::value;
#pragma unroll
        for (int a = 0; a < d; ++a) dbar[a] += (letter[m] == a) ? dbu[m] : 0.0f;
    });
}

// ad (+)= row, laid out like an output row; the prefix words are taken by the lane whose remaining letters are 0
// OWNED = false leaves the choice of the lane that takes a prefix word to the caller: every lane gets the value
template <int d, int N, int P, bool ADD, bool OWNED = true>
__device__ __forceinline__ void load_adjoint(const float *row, unsigned u, Lane<d, N, P> &ad)
{
    using Sh = Shape<d, N, P>;
    static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) __attribute__((always_inline)) {
        constexpr int r = decltype(rc)::value;
        constexpr int cnt = cpow(d, r);
        const float *src = row + Sh::row_off(P + r) + u * cnt;
#pragma unroll
        for (int i = 0; i < cnt; ++i) {
            if constexpr (ADD) ad.s[Sh::sub_off(r) + i] += src[i];
            else ad.s[Sh::sub_off(r) + i] = src[i];
        }
    });
    if constexpr (P == 0 && !ADD) ad.s[0] = 0.0f;
    // (!OWNED: every lane loads.  A load under a condition would keep the compiler from counting the loads in
    // flight, and a sweep that fetches rows ahead would wait for all of them at every step)
    static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
        constexpr int m = decltype(mc)::value;
        constexpr unsigned span = cpow(d, P - m);
        float g = 0.0f;
        if (!OWNED || u % span == 0) g = row[Sh::row_off(m) + u / span];
        if constexpr (ADD) ad.pre[m - 1] += g;
        else ad.pre[m - 1] = g;
    });
}

// The lanes that take the prefix words of a row (word u_{1:m}: the lane whose remaining letters are 0), for rows
// fetched with OWNED = false, and the sum ad += row of such a row.  The choice is made where the row is used and not
// where it is fetched: a fetch that masks its own loads waits for them at once, and a sweep that fetches rows ahead
// of their use would have nothing in flight.
template <int d, int N, int P>
struct PrefixOwner {
    bool w[Shape<d, N, P>::NPRE];
    __device__ __forceinline__ explicit PrefixOwner(unsigned u)
    {
#pragma unroll
        for (int i = 0; i < Shape<d, N, P>::NPRE; ++i) w[i] = i + 1 < P && u % cpow(d, P - 1 - i) == 0;
    }
};
template <int d, int N, int P>
__device__ __forceinline__ void add_row(Lane<d, N, P> &ad, const Lane<d, N, P> &row, const PrefixOwner<d, N, P> &own,
                                        bool use = true)
{
    using Sh = Shape<d, N, P>;
#pragma unroll
    for (int i = 0; i < Sh::SZ; ++i) ad.s[i] += use ? row.s[i] : 0.0f;
#pragma unroll
    for (int i = 0; i < Sh::NPRE; ++i) ad.pre[i] += (use && own.w[i]) ? row.pre[i] : 0.0f;
}

struct BackwardArgs {
    const float *path;      // [B][L][d]
    const float *sig;       // the forward result: [B][D] or [B][K][D]
    const float *grad_out;  // same shape as sig
    float *grad_path;       // [B][L][d]
    int64_t B, L;
    int32_t groups;         // paths per workgroup
    int32_t stream_flag;
    // Sliced sweep cut in time (final mode; segs <= 1: the whole path in one piece).  Segment s covers the
    // increments [s * seg_steps, (s + 1) * seg_steps) and starts from the signature of the path up to its end and
    // the gradient with respect to that signature: rows [B][segs][D], the last of which is not read (it is the
    // forward result and its upstream gradient).
    int32_t segs;
    int32_t seg_steps;
    const float *seg_sig;
    const float *seg_grad;
    float *seg_part;        // register sweep cut in time: d(loss)/d(increment), [B][L-1][d]
    float *seg_adj_out;     // first sweep of the stream-mode cut: what a piece's own rows leave at its start, see
                            // sig_backward_segments.hip; row of piece (b, s >= 1) at (b * segs + s - 1), zeros at the
                            // last row of every path
    // Long paths whose increments do not fit LDS at once (either mode): tiled != 0 makes a workgroup walk the segs
    // pieces of its paths one after the other, last first, with its state in registers; no seg_sig / seg_grad rows.
    int32_t tiled;
};

// steps whose partial sums are parked before they are added up: enough for every lane of a path to have a
// column (Q / d), but no more than eight (the parked sums take TS * Park::kStepFloats floats of LDS per path)
template <int d, int P>
constexpr int reduce_steps()
{
    const int want = cpow(d, P) / d;
    return want < 1 ? 1 : (want > 8 ? 8 : want);
}

// Layout of the parked sums of a path.  As [step][lane][channel] a lane's d sums are d floats from its neighbour's,
// so the lanes of a wavefront write to 32 / gcd(d, 32) of the 32 LDS banks: all of them for odd d, half for d = 2, 6,
// 10, but only eight for d = 4 and four for d = 8.  Those shapes keep the sums as [step][channel][lane] with rows of
// an odd number of floats: the lanes' writes (consecutive lanes, one row) and the column sums' reads (consecutive
// rows, one lane) then both spread over the banks (measured: d = 8, depth 3, 1.6x; d = 4, depth 4, 1.3x on
// saturated batches; for the other channel counts the change is within a few percent either way).
template <int d, int P>
struct Park {
    static constexpr int Q = cpow(d, P);
    static constexpr bool kByChannel = d % 4 == 0;
    static constexpr int kRow = Q | 1;
    static constexpr int kStepFloats = kByChannel ? d * kRow : d * Q;
    // sum of lane u for channel a in parked step t
    static __device__ __forceinline__ int at(int t, int u, int a) { return kByChannel ? (t * d + a) * kRow + u : (t * Q + u) * d + a; }
};

extern __shared__ float sig_backward_smem[];

// increments per tile when a path is too long for the LDS of the uncut sweep and one workgroup walks it in tiles
constexpr int kTiledSteps = 256;

// Register sweep: the d^P lanes of a path fit a workgroup, which takes `groups` paths side by side.
// SEG (final mode): the sweep is cut in time and the workgroup takes `groups` (path, segment) pieces instead, piece
// = b * segs + s; every piece is swept as seg_steps increments (the last segment of a path is filled up with zero
// increments behind its end, which leave the signature and the adjoint as they are), starts from the rows
// seg_sig / seg_grad (see BackwardArgs) and leaves its sums over the increments in seg_part.
// SEG in stream mode: a piece starts from the output row at its end (row k of a stream output is the signature of
// the path up to increment k) and from the gradient seg_grad that the later pieces leave there, and adds the
// upstream gradients of its own rows as it goes.  EMIT = false is the first of the two sweeps that provide seg_grad:
// from a zero adjoint, without sums over the increments; it writes what the piece's own rows leave at its start to
// seg_adj_out (the lanes' partial adjoints of a prefix word are added up there).
// TSV: steps whose partial sums are parked before they are added up; 0 = reduce_steps, the most that is useful.
// Fewer steps take less LDS, which buys resident workgroups on saturated batches (kShortPark, see backward_launch).
constexpr int kShortPark = 3;
// PIPE (stream mode, uncut): the upstream rows are fetched as a software pipeline that keeps PD rows in flight
// at every step; for launches that leave the SIMDs a wavefront each or less, where nothing else hides a row's latency.
template <int d, int N, int P, bool STREAM, bool SEG = false, bool EMIT = true, int TSV = 0, bool PIPE = false>
__global__ __launch_bounds__(256) void sig_backward_kernel(BackwardArgs A)
{
    static_assert(!PIPE || (STREAM && !SEG), "the pipelined fetch belongs to the uncut stream sweep");
    static_assert(EMIT || (STREAM && SEG), "the sweep without output belongs to the stream-mode cut");
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr int TS = TSV > 0 ? TSV : reduce_steps<d, P>();
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t Kall = A.L - 1;                     // increments of a path
    const int64_t K = SEG ? A.seg_steps : Kall;       // increments of a workgroup's rows
    const int W = SEG ? A.segs : 1;
    const int64_t rows = A.B * W;                     // paths, or pieces
    const int G = A.groups;
    const int gi_raw = tid / Q;
    const unsigned u = (unsigned)(tid - gi_raw * Q);
    const int64_t b0 = (int64_t)blockIdx.x * G;       // first path (piece) of the workgroup
    const bool active = gi_raw < G && b0 + gi_raw < rows;
    const int gi = gi_raw < G ? gi_raw : 0;
    const int64_t piece = active ? b0 + gi : 0;
    const int64_t b = piece / W;
    const int seg = (int)(piece - b * W);
    const int64_t k0 = SEG ? (int64_t)seg * K : 0;    // first increment of the piece

    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    }

    // LDS: increments [G][K*d] (overwritten step by step with their gradients), parked partial sums [G][TS] x Park
    const int row_floats = (int)K * d;
    float *tile = sig_backward_smem;
    float *park = tile + (G * row_floats + 3) / 4 * 4;
    for (int i = tid; i < G * row_floats; i += nthr) {
        const int g2 = i / row_floats;
        const int r = i - g2 * row_floats;
        float v = 0.0f;
        if (b0 + g2 < rows) {
            if constexpr (SEG) {
                const int64_t b2 = (b0 + g2) / W;
                const int64_t first = (b0 + g2 - b2 * W) * K;
                if (first * d + r < Kall * d) {
                    const float *x = A.path + (b2 * A.L + first) * d + r;
                    v = x[d] - x[0];
                }
            } else {
                const float *x = A.path + (b0 + g2) * A.L * d + r;
                v = x[d] - x[0];
            }
        }
        tile[i] = v;
    }

    Lane<d, N, P> ln, ad;
    identity_state<d, N, P>(ln);
    identity_state<d, N, P>(ad);
    if (P == 0) ad.s[0] = 0.0f;
    if (active) {
        const bool inner = SEG && seg < W - 1;   // a segment that ends inside the path
        if constexpr (STREAM && SEG) {
            const int64_t last = k0 + K < Kall ? k0 + K - 1 : Kall - 1;   // last increment of the piece
            load_state<d, N, P>(A.sig + (b * Kall + last) * D, u, ln);
            if constexpr (EMIT) load_adjoint<d, N, P, false>(A.seg_grad + piece * D, u, ad);
        } else {
            const float *srow = STREAM ? A.sig + (b * K + (K - 1)) * D : inner ? A.seg_sig + piece * D : A.sig + b * D;
            load_state<d, N, P>(srow, u, ln);
            if constexpr (!STREAM) load_adjoint<d, N, P, false>(inner ? A.seg_grad + piece * D : A.grad_out + b * D, u, ad);
        }
    }
    __syncthreads();

    using Pk = Park<d, P>;
    float *mypark = park + (size_t)gi * TS * Pk::kStepFloats;
    float *myrow = tile + gi * row_floats;
    const PrefixOwner<d, N, P> owner(u);
    // One step of the sweep; `upk` is the upstream gradient of row k (stream mode).
    auto step = [&](int64_t k, const Lane<d, N, P> *upk) __attribute__((always_inline)) {
        const int ts = (int)((K - 1 - k) % TS);
        if constexpr (STREAM) {
            // (rows behind the end of the path, in the filled-up last piece of a cut sweep, count as zero)
            if constexpr (PIPE) {
                add_row<d, N, P>(ad, *upk, owner);
            } else {
#pragma unroll
                for (int i = 0; i < Sh::SZ; ++i) ad.s[i] += upk->s[i];
#pragma unroll
                for (int i = 0; i < Sh::NPRE; ++i) ad.pre[i] += upk->pre[i];
            }
        }
        Inc<d, P> inc, neg;
        load_inc<d, P>(inc, myrow + k * d, letter);
#pragma unroll
        for (int a = 0; a < d; ++a) neg.v[a] = -inc.v[a];
        neg.du[0] = 0.0f;
#pragma unroll
        for (int m = 0; m < P; ++m) neg.du[m] = -inc.du[m];
        if (k0 + k > 0) fused_step<d, N, P>(ln, neg);  // S_{k-1} = S_k (x) exp(-dX_k)
        else identity_state<d, N, P>(ln);               // before the first increment: the identity, exactly
        float dbar[d];
        backward_step<d, N, P>(ln, ad, inc, letter, dbar);
        if constexpr (EMIT) {
            if (active) {
#pragma unroll
                for (int a = 0; a < d; ++a) mypark[Pk::at(ts, (int)u, a)] = dbar[a];
            }
            if (ts == TS - 1 || k == 0) {
                __syncthreads();
                // column c = (parked step t, channel a): the sum over the path's lanes is d(loss)/d(dX)[a] of step
                // k + (ts - t); it replaces that increment, which no lane reads again
                if (active) {
                    for (int c = (int)u; c < (ts + 1) * d; c += Q) {
                        const int t = c / d, a = c - t * d;
                        float sum = 0.0f;
                        for (int q = 0; q < Q; ++q) sum += mypark[Pk::at(t, q, a)];
                        myrow[(k + (ts - t)) * d + a] = sum;
                    }
                }
                __syncthreads();
            }
        }
    };
    // A wavefront none of whose lanes has a path (the workgroup's paths need not fill its threads) only keeps the
    // other wavefronts' barriers company: one pair for every TS steps.
    const int first_group = __builtin_amdgcn_readfirstlane(tid) / Q;
    const bool idle_wavefront = !(first_group < G && b0 + first_group < rows);
    if (idle_wavefront) {
        if constexpr (EMIT) {
            for (int64_t e = 0; e < (K + TS - 1) / TS; ++e) {
                __syncthreads();
                __syncthreads();
            }
        }
    } else if constexpr (STREAM && PIPE) {
        // The upstream gradient rows are fetched PD steps ahead into registers, as in the plain stream sweep
        // below, but every lane fetches at every step, from a row that exists: the compiler waits for a fetched row
        // by counting the loads issued after it, and a load under a condition makes that count zero, i.e. a wait
        // for everything in flight (the plain sweep waits like that once in PD steps).  Idle lanes read the first
        // path's rows; the fetches behind the first row read it again.  One fetch per call, in the order of the sweep.
        constexpr int PD = Sh::SZ <= 24 ? 4 : Sh::SZ <= 48 ? 2 : 1;
        Lane<d, N, P> up[PD];
        const float *next_row = A.grad_out + (b * Kall + (Kall - 1)) * D;
        int64_t kn = K - 1;
        auto fetch = [&](Lane<d, N, P> &dst) __attribute__((always_inline)) {
            load_adjoint<d, N, P, false, false>(next_row, u, dst);
            next_row -= kn > 0 ? D : 0;
            --kn;
        };
        static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            identity_state<d, N, P>(up[j]);   // (the fields that a row does not fill)
            fetch(up[j]);
        });
        int64_t kk = K - 1;
        for (; kk >= PD - 1; kk -= PD) {
            static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                step(kk - j, &up[j]);
                // (the loads stay behind the step that uses the row they replace: moved up, they would need
                // registers of their own and a copy at the top of the loop, which waits for every row in flight;
                // arithmetic and LDS reads of the next step may pass them)
                __builtin_amdgcn_sched_barrier(0);
                fetch(up[j]);
                __builtin_amdgcn_sched_barrier(0x81);
            });
        }
        // the K % PD steps that are left
        static_for<0, PD - 1>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            if (kk - j >= 0) step(kk - j, &up[j]);
        });
    } else if constexpr (STREAM) {
        // The upstream gradient rows are fetched PD steps ahead into registers: a row's HBM latency (well over
        // a microsecond) is several steps long, and at one or two wavefronts per SIMD nothing else hides it.
        // (as many rows as the registers hold beside the two lane states)
        constexpr int PD = Sh::SZ <= 24 ? 4 : Sh::SZ <= 48 ? 2 : 1;
        Lane<d, N, P> up[PD];
        static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            identity_state<d, N, P>(up[j]);
            if (P == 0) up[j].s[0] = 0.0f;
            if constexpr (SEG) {
                // (rows behind the end of the path, in the filled-up last piece, stay zero)
                if (active && K - 1 - j >= 0 && k0 + K - 1 - j < Kall)
                    load_adjoint<d, N, P, false>(A.grad_out + (b * Kall + (k0 + K - 1 - j)) * D, u, up[j]);
            } else {
                if (active && K - 1 - j >= 0) load_adjoint<d, N, P, false>(A.grad_out + (b * K + (K - 1 - j)) * D, u, up[j]);
            }
        });
        for (int64_t kk = K - 1; kk >= 0; kk -= PD) {
            static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                const int64_t k = kk - j;
                if (k >= 0) {
                    step(k, &up[j]);
                    if constexpr (SEG) {
                        if (active && k - PD >= 0 && k0 + k - PD < Kall)
                            load_adjoint<d, N, P, false>(A.grad_out + (b * Kall + (k0 + k - PD)) * D, u, up[j]);
                    } else {
                        if (active && k - PD >= 0) load_adjoint<d, N, P, false>(A.grad_out + (b * K + (k - PD)) * D, u, up[j]);
                    }
                }
            });
        }
    } else {
        for (int64_t k = K - 1; k >= 0; --k) step(k, nullptr);
    }

    if constexpr (!EMIT) {
        // what the piece's own rows leave at its start, as a row: a lane owns the words of its sub-tree; the partial
        // adjoints of a shorter prefix word are added up over the lanes that share it (fixed order)
        float *scr = mypark;   // [P-1][Q]
        static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value;
            if (active) scr[(m - 1) * Q + u] = ad.pre[m - 1];
        });
        __syncthreads();
        if (active) {
            // piece (b, s) hands its row to the piece before it; the last row of a path is zero (nothing follows)
            float *row = A.seg_adj_out + (seg > 0 ? piece - 1 : b * W + (W - 1)) * D;
            const bool keep = seg > 0;
            static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) __attribute__((always_inline)) {
                constexpr int r = decltype(rc)::value;
                constexpr int cnt = cpow(d, r);
#pragma unroll
                for (int i = 0; i < cnt; ++i) row[Sh::row_off(P + r) + u * cnt + i] = keep ? ad.s[Sh::sub_off(r) + i] : 0.0f;
            });
            static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
                constexpr int m = decltype(mc)::value;
                constexpr unsigned span = cpow(d, P - m);
                if (u % span == 0) {
                    float sum = 0.0f;
#pragma unroll
                    for (unsigned j = 0; j < span; ++j) sum += scr[(m - 1) * Q + u + j];
                    row[Sh::row_off(m) + u / span] = keep ? sum : 0.0f;
                }
            });
        }
        return;
    }
    if constexpr (SEG) {
        // the sums over the piece's own increments; another launch forms d(loss)/dX across the pieces
        for (int i = tid; i < G * row_floats; i += nthr) {
            const int g2 = i / row_floats;
            const int r = i - g2 * row_floats;
            if (b0 + g2 < rows) {
                const int64_t b2 = (b0 + g2) / W;
                const int64_t first = (b0 + g2 - b2 * W) * K;
                if (first * d + r < Kall * d) A.seg_part[(b2 * Kall + first) * d + r] = tile[i];
            }
        }
        return;
    }
    // d(loss)/dX_j = d/d(dX_{j-1}) - d/d(dX_j)
    const int out_row = (int)A.L * d;
    for (int i = tid; i < G * out_row; i += nthr) {
        const int g2 = i / out_row;
        const int r = i - g2 * out_row;
        if (b0 + g2 < A.B) {
            const float *t = tile + g2 * row_floats;
            const float before = r >= d ? t[r - d] : 0.0f;
            const float after = r < row_floats ? t[r] : 0.0f;
            A.grad_path[(b0 + g2) * out_row + r] = before - after;
        }
    }
}

// Register sweep over paths whose increments do not fit LDS at once: the workgroup walks the A.segs tiles of
// A.seg_steps increments of its `groups` paths one after the other, last first, with the lane states in registers,
// and leaves the sums over the increments in seg_part ([B][L-1][d]); another launch forms d(loss)/dX.  Sequential in
// time like the plain sweep (no chunks), but any length fits.  Stream mode fetches a row's upstream gradient one
// step ahead.
template <int d, int N, int P, bool STREAM>
__global__ __launch_bounds__(256) void sig_backward_tiled_kernel(BackwardArgs A)
{
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr int TS = reduce_steps<d, P>();
    using Pk = Park<d, P>;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t Kall = A.L - 1;
    const int64_t T = A.seg_steps;
    const int G = A.groups;
    const int gi_raw = tid / Q;
    const unsigned u = (unsigned)(tid - gi_raw * Q);
    const int64_t b0 = (int64_t)blockIdx.x * G;
    const bool active = gi_raw < G && b0 + gi_raw < A.B;
    const int gi = gi_raw < G ? gi_raw : 0;
    const int64_t b = active ? b0 + gi : 0;
    const PrefixOwner<d, N, P> owner(u);

    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    }

    const int row_stride = (int)T * d;   // a path's part of the tile
    float *tile = sig_backward_smem;
    float *park = tile + (G * row_stride + 3) / 4 * 4;
    float *mypark = park + (size_t)gi * TS * Pk::kStepFloats;
    float *myrow = tile + gi * row_stride;

    // Stream mode: the upstream rows of a tile are fetched PD steps ahead into registers, as in the plain sweep; every
    // tile starts with its first PD rows, asked for before its increments are staged.
    constexpr int PD = !STREAM ? 1 : Sh::SZ <= 24 ? 4 : Sh::SZ <= 48 ? 2 : 1;
    Lane<d, N, P> ln, ad, up[PD];
    identity_state<d, N, P>(ln);
    identity_state<d, N, P>(ad);
    static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
        identity_state<d, N, P>(up[decltype(jc)::value]);
        if (P == 0) up[decltype(jc)::value].s[0] = 0.0f;
    });
    if (P == 0) ad.s[0] = 0.0f;
    if (active) {
        load_state<d, N, P>(STREAM ? A.sig + (b * Kall + (Kall - 1)) * D : A.sig + b * D, u, ln);
        if constexpr (!STREAM) load_adjoint<d, N, P, false>(A.grad_out + b * D, u, ad);
    }

    for (int tl = A.segs - 1; tl >= 0; --tl) {
        const int64_t k0 = (int64_t)tl * T;
        const int64_t K = Kall - k0 < T ? Kall - k0 : T;
        const int row_floats = (int)K * d;
        if constexpr (STREAM) {
            static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                if (active && K - 1 - j >= 0)
                    load_adjoint<d, N, P, false, false>(A.grad_out + (b * Kall + (k0 + K - 1 - j)) * D, u, up[j]);
            });
        }
        if (tl != A.segs - 1) __syncthreads();   // the previous tile's sums have been written out
        for (int i = tid; i < G * row_floats; i += nthr) {
            const int g2 = i / row_floats;
            const int r = i - g2 * row_floats;
            float v = 0.0f;
            if (b0 + g2 < A.B) {
                const float *x = A.path + ((b0 + g2) * A.L + k0) * d + r;
                v = x[d] - x[0];
            }
            tile[g2 * row_stride + r] = v;
        }
        __syncthreads();
        for (int64_t kk = K - 1; kk >= 0; kk -= PD)
        static_for<0, PD>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            const int64_t k = kk - j;
            if (k < 0) return;
            const int ts = (int)((K - 1 - k) % TS);
            if constexpr (STREAM) {
                add_row<d, N, P>(ad, up[j], owner);
                if (active && k - PD >= 0)
                    load_adjoint<d, N, P, false, false>(A.grad_out + (b * Kall + (k0 + k - PD)) * D, u, up[j]);
            }
            Inc<d, P> inc, neg;
            load_inc<d, P>(inc, myrow + k * d, letter);
#pragma unroll
            for (int a = 0; a < d; ++a) neg.v[a] = -inc.v[a];
            neg.du[0] = 0.0f;
#pragma unroll
            for (int m = 0; m < P; ++m) neg.du[m] = -inc.du[m];
            if (k0 + k > 0) fused_step<d, N, P>(ln, neg);
            else identity_state<d, N, P>(ln);
            float dbar[d];
            backward_step<d, N, P>(ln, ad, inc, letter, dbar);
            if (active) {
#pragma unroll
                for (int a = 0; a < d; ++a) mypark[Pk::at(ts, (int)u, a)] = dbar[a];
            }
            if (ts == TS - 1 || k == 0) {
                __syncthreads();
                if (active) {
                    for (int c = (int)u; c < (ts + 1) * d; c += Q) {
                        const int t = c / d, a = c - t * d;
                        float sum = 0.0f;
                        for (int q = 0; q < Q; ++q) sum += mypark[Pk::at(t, q, a)];
                        myrow[(k + (ts - t)) * d + a] = sum;
                    }
                }
                __syncthreads();
            }
        });
        for (int i = tid; i < G * row_floats; i += nthr) {
            const int g2 = i / row_floats;
            const int r = i - g2 * row_floats;
            if (b0 + g2 < A.B) A.seg_part[((b0 + g2) * Kall + k0) * d + r] = tile[g2 * row_stride + r];
        }
    }
}

// LDS bytes of the register sweep with `groups` paths (or pieces) of L points per workgroup and park_steps parked
// steps (0: reduce_steps)
template <int d, int N, int P>
int64_t backward_lds_bytes(int64_t L, int groups, int park_steps)
{
    const int64_t tile = ((int64_t)groups * (L - 1) * d + 3) / 4 * 4;
    const int64_t park = (int64_t)groups * (park_steps > 0 ? park_steps : reduce_steps<d, P>()) * Park<d, P>::kStepFloats;
    return (tile + park) * (int64_t)sizeof(float);
}
template <int d, int N, int P>
int64_t backward_lds_bytes(int64_t L, int groups)
{
    return backward_lds_bytes<d, N, P>(L, groups, 0);
}

// LDS of the sweep cut in time inside a workgroup (sig_backward_chunked_kernel): a lane's registers in LDS, one
// chunk's row in either of its two buffers, and the launch's bytes
template <int d, int N, int P>
constexpr int private_floats() { return (Shape<d, N, P>::SZ + Shape<d, N, P>::NPRE) * Shape<d, N, P>::Q; }

template <int d, int N, int P>
constexpr int chunk_row_floats()  // one chunk's row in either LDS buffer of the chunked sweep
{
    using Sh = Shape<d, N, P>;
    int a = Sh::D;
    const int park = reduce_steps<d, P>() * Park<d, P>::kStepFloats;
    if (park > a) a = park;
    return (a + 3) / 4 * 4;
}

template <int d, int N, int P>
int64_t backward_chunked_lds_bytes(int64_t L, int chunks, int stream_flag)
{
    const int64_t tile = ((L - 1) * d + 3) / 4 * 4;
    int64_t per_chunk = 2 * (int64_t)chunk_row_floats<d, N, P>();
    if (stream_flag) per_chunk += private_floats<d, N, P>();
    return (tile + chunks * per_chunk) * (int64_t)sizeof(float);
}

// chunks of at least eight increments that one workgroup of `threads` threads sweeps side by side (1: it does not cut)
template <int d, int N, int P>
int backward_chunks(int64_t L, int stream_flag, int threads)
{
    int C = threads / Shape<d, N, P>::Q;
    if (C > (L - 1) / 8) C = (int)((L - 1) / 8);
    // The two scans over the chunk signatures walk the C chunks one after the other (a product and a barrier each),
    // the sweeps walk K / C increments: about sqrt(K) chunks balance the two (measured on shapes with 2 to 10
    // lanes per path, 300 to 2,000 points: 1.0-2.6x over as many chunks as the threads hold, never slower).
    int cap = 8;
    while ((int64_t)(cap + 1) * (cap + 1) <= L - 1) ++cap;
    if (C > cap) C = cap;
    while (C > 1 && backward_chunked_lds_bytes<d, N, P>(L, C, stream_flag) > kMaxLdsBytes) --C;
    return C < 1 ? 1 : C;
}

// ---------------------------------------------------------------------------------------------------------
// Sliced sweep: shapes whose d^P lanes per path exceed one workgroup.  A workgroup takes one path and one slice
// of up to 256 of its lanes; nothing crosses lanes in the sweep itself, only d(loss)/dv of a step is a sum over
// all lanes of the path.  Each slice adds up its own lanes (parked partial sums, two-stage column sums in a
// fixed order) over the increment the sum belongs to, writes its K * d partial sums to `part`, and a second
// launch adds the slices in order and forms d(loss)/dX.
constexpr int kSliceLanes = 256;
constexpr int kSliceSplit = 8;   // a parked column is summed in this many stretches of lanes first

template <int d>
constexpr int slice_reduce_steps()
{
    const int fit = 8192 / (kSliceLanes * d);   // parked sums take TS * 256 * d floats of LDS
    return fit < 1 ? 1 : (fit > 8 ? 8 : fit);
}

// Parked sums of one step: [channel][lane], lane q at q + q / 32.  Consecutive lanes write consecutive banks, and
// the extra float per stretch of 32 lanes puts the stretches, which are read side by side when a column is summed,
// in different LDS banks (32 floats apart they would all start in the same one).
constexpr int kParkRow = kSliceLanes + kSliceLanes / 32;
template <int d>
constexpr int slice_park_floats() { return d * kParkRow; }

// words of the levels below the prefix depth, 1 .. P-1: the lanes that share such a word hold partial adjoints of it
template <int d, int P>
constexpr int shared_prefix_words() { return P > 1 ? geom(d, P) - 1 : 0; }   // d + ... + d^{P-1}

template <int d, int N, int P, bool STREAM, bool EMIT = true>
__global__ __launch_bounds__(kSliceLanes) void sig_backward_sliced_kernel(BackwardArgs A, float *part, int TS)
{
    // TS: steps whose partial sums are parked before they are added up (at most slice_reduce_steps<d>(); fewer
    // when a long path leaves less LDS)
    // A.segs > 1 cuts the path into pieces of A.seg_steps increments: every piece a workgroup of its own (see
    // BackwardArgs; in stream mode a piece starts from the output row at its end and from seg_grad, like the register
    // sweep), or with A.tiled the workgroup walks the pieces of its path one after the other, last first, with its
    // state in registers, so that only one piece's increments are staged in LDS at a time.
    // EMIT = false (stream-mode pieces): the first of the two sweeps, from a zero adjoint and without sums over the
    // increments; the lane's own words of what the piece's rows leave at its start go to seg_adj_out, the slice's
    // sums of the partial adjoints of the shorter prefix words to `part` ([piece][slice][shared_prefix_words]).
    static_assert(EMIT || STREAM, "the sweep without output belongs to the stream-mode cut");
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr int slices = (Q + kSliceLanes - 1) / kSliceLanes;
    constexpr int kParkStep = slice_park_floats<d>();
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int slice = (int)(blockIdx.x % slices);
    const int64_t piece = blockIdx.x / slices;
    const int W = (!A.tiled && A.segs > 1) ? A.segs : 1;              // pieces that are workgroups of their own
    const int tiles = (A.tiled && A.segs > 1) ? A.segs : 1;           // pieces this workgroup walks
    const int64_t b = piece / W;
    const int seg = (int)(piece - b * W);
    const int64_t Kall = A.L - 1;                            // increments of the path
    const int64_t T = (W > 1 || tiles > 1) ? A.seg_steps : Kall;
    if (W > 1 && (int64_t)seg * T >= Kall) return;           // a trailing segment without increments
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

    // LDS: increments [T*d] (overwritten with this slice's sums), parked partial sums [TS][d][kParkRow], stretch sums
    float *tile = sig_backward_smem;
    float *park = tile + ((int)T * d + 3) / 4 * 4;
    float *red = park + TS * kParkStep;

    Lane<d, N, P> ln, ad;
    identity_state<d, N, P>(ln);
    identity_state<d, N, P>(ad);
    if (P == 0) ad.s[0] = 0.0f;
    // last increment of the workgroup's first piece (the whole path unless it is a piece of its own)
    const int64_t last = W > 1 && (int64_t)(seg + 1) * T < Kall ? (int64_t)(seg + 1) * T - 1 : Kall - 1;
    if (active) {
        const bool inner = seg < W - 1;   // a segment that ends inside the path
        const float *srow = STREAM ? A.sig + (b * Kall + last) * D : inner ? A.seg_sig + piece * D : A.sig + b * D;
        load_state<d, N, P>(srow, u, ln);
        if constexpr (!STREAM) load_adjoint<d, N, P, false>(inner ? A.seg_grad + piece * D : A.grad_out + b * D, u, ad);
        else if (W > 1 && EMIT) load_adjoint<d, N, P, false>(A.seg_grad + piece * D, u, ad);
    }
    Lane<d, N, P> up;   // upstream gradient of the row the sweep reaches next (stream mode), fetched one step ahead
    if constexpr (STREAM) {
        identity_state<d, N, P>(up);
        if (P == 0) up.s[0] = 0.0f;
        if (active) load_adjoint<d, N, P, false>(A.grad_out + (b * Kall + last) * D, u, up);
    }

    for (int tl = tiles - 1; tl >= 0; --tl) {
        const int64_t k0 = (int64_t)(W > 1 ? seg : tl) * T;   // first increment of this piece (one piece: 0)
        const int64_t K = Kall - k0 < T ? Kall - k0 : T;
        const int row_floats = (int)K * d;
        if (tl != tiles - 1) __syncthreads();   // the previous piece's sums have been written out
        {
            const float *x = A.path + (b * A.L + k0) * d;
            for (int i = tid; i < row_floats; i += nthr) tile[i] = x[i + d] - x[i];
        }
        __syncthreads();
        for (int64_t k = K - 1; k >= 0; --k) {
            const int ts = (int)((K - 1 - k) % TS);
            if constexpr (STREAM) {
#pragma unroll
                for (int i = 0; i < Sh::SZ; ++i) ad.s[i] += up.s[i];
#pragma unroll
                for (int i = 0; i < Sh::NPRE; ++i) ad.pre[i] += up.pre[i];
                if (active && k0 + k > 0) load_adjoint<d, N, P, false>(A.grad_out + (b * Kall + (k0 + k - 1)) * D, u, up);
            }
            Inc<d, P> inc, neg;
            load_inc<d, P>(inc, tile + k * d, letter);
#pragma unroll
            for (int a = 0; a < d; ++a) neg.v[a] = -inc.v[a];
            neg.du[0] = 0.0f;
#pragma unroll
            for (int m = 0; m < P; ++m) neg.du[m] = -inc.du[m];
            if (k0 + k > 0) fused_step<d, N, P>(ln, neg);  // S_{k-1} = S_k (x) exp(-dX_k)
            else identity_state<d, N, P>(ln);
            float dbar[d];
            backward_step<d, N, P>(ln, ad, inc, letter, dbar);
            if constexpr (!EMIT) continue;
#pragma unroll
            for (int a = 0; a < d; ++a) park[ts * kParkStep + a * kParkRow + tid + (tid >> 5)] = active ? dbar[a] : 0.0f;
            if (ts == TS - 1 || k == 0) {
                __syncthreads();
                // column c = (parked step t, channel a), first in kSliceSplit stretches of lanes, then the stretches
                const int cols = (ts + 1) * d;
                constexpr int stretch = kSliceLanes / kSliceSplit;
                static_assert(stretch == 32, "the parked layout pads one float per 32 lanes");
                for (int w = tid; w < cols * kSliceSplit; w += nthr) {
                    const int c = w / kSliceSplit, r = w - c * kSliceSplit;
                    const int t = c / d, a = c - t * d;
                    // (idle lanes parked zeros, so every stretch is summed in full: a fixed trip count lets the
                    // reads be issued together)
                    const float *src = park + t * kParkStep + a * kParkRow + r * (stretch + 1);
                    float sum = 0.0f;
#pragma unroll
                    for (int q = 0; q < stretch; ++q) sum += src[q];
                    red[w] = sum;
                }
                __syncthreads();
                for (int c = tid; c < cols; c += nthr) {
                    const int t = c / d, a = c - t * d;
                    float sum = 0.0f;
#pragma unroll
                    for (int r = 0; r < kSliceSplit; ++r) sum += red[c * kSliceSplit + r];
                    tile[(k + (ts - t)) * d + a] = sum;   // replaces the increment, which no lane reads again
                }
                __syncthreads();
            }
        }
        if constexpr (EMIT) {
            float *dst = part + ((b * slices + slice) * Kall + k0) * d;
            for (int i = tid; i < row_floats; i += nthr) dst[i] = tile[i];
        }
    }
    if constexpr (!EMIT) {
        // piece (b, s) hands its row to the piece before it; the last row of a path is zero (nothing follows it)
        const bool keep = seg > 0;
        float *row = A.seg_adj_out + (keep ? piece - 1 : b * W + (W - 1)) * D;
        if (active) {
            static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) __attribute__((always_inline)) {
                constexpr int r = decltype(rc)::value;
                constexpr int cnt = cpow(d, r);
#pragma unroll
                for (int i = 0; i < cnt; ++i) row[Sh::row_off(P + r) + u * cnt + i] = keep ? ad.s[Sh::sub_off(r) + i] : 0.0f;
            });
        }
        // the slice's sums of the partial adjoints of the words of levels 1 .. P-1 (zero where no lane of the slice
        // lies below a word); another launch adds the slices in order
        constexpr int NW = shared_prefix_words<d, P>();
        if constexpr (NW > 0) {
            __syncthreads();
            float *scr = park;   // [P-1][kSliceLanes]
            static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
                constexpr int m = decltype(mc)::value;
                scr[(m - 1) * kSliceLanes + tid] = active ? ad.pre[m - 1] : 0.0f;
            });
            __syncthreads();
            float *side = part + (piece * slices + slice) * NW;
            const int lane0 = slice * kSliceLanes;
            static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
                constexpr int m = decltype(mc)::value;
                constexpr int span = cpow(d, P - m);
                constexpr int words = cpow(d, m);
                for (int w = tid; w < words; w += nthr) {
                    int lo = w * span - lane0, hi = lo + span;
                    if (lo < 0) lo = 0;
                    if (hi > kSliceLanes) hi = kSliceLanes;
                    float sum = 0.0f;
                    for (int j = lo; j < hi; ++j) sum += scr[(m - 1) * kSliceLanes + j];
                    side[Sh::row_off(m) + w] = sum;
                }
            });
        }
    }
}

// LDS bytes of the sliced sweep over a path (or time segment) of L points with ts parked steps
template <int d>
int64_t backward_sliced_bytes_with(int64_t L, int ts)
{
    const int64_t tile = ((L - 1) * d + 3) / 4 * 4;
    return (tile + (int64_t)ts * slice_park_floats<d>() + (int64_t)ts * d * kSliceSplit) * (int64_t)sizeof(float);
}

// parked steps for a path of L points: as many as fit beside the path's increments, at least one (0: does not fit)
template <int d>
int backward_sliced_steps(int64_t L)
{
    int ts = slice_reduce_steps<d>();
    while (ts > 1 && backward_sliced_bytes_with<d>(L, ts) > kMaxLdsBytes) --ts;
    return backward_sliced_bytes_with<d>(L, ts) <= kMaxLdsBytes ? ts : 0;
}

}  // namespace onchip
}  // namespace sig

// Every compiled (d, depth, prefix depth) of the reverse sweep, one prefix depth per (d, depth): the one whose two
// lane states (S and its adjoint) fit the registers.  REG: the d^P lanes of a path fit a workgroup; SLICED: they
// span several (sliced sweep).
#define SIG_BACKWARD_SHAPES(REG, SLICED) \
    REG(2, 2, 1) REG(3, 2, 1) REG(4, 2, 1) REG(5, 2, 1) REG(6, 2, 1) REG(8, 2, 1) REG(10, 2, 1) REG(2, 3, 1) \
    REG(3, 3, 1) REG(4, 3, 1) REG(5, 3, 1) REG(6, 3, 1) REG(7, 3, 1) REG(8, 3, 2) REG(10, 3, 2) REG(2, 4, 1) \
    REG(3, 4, 1) REG(4, 4, 2) REG(5, 4, 2) REG(6, 4, 2) REG(7, 4, 2) REG(2, 5, 1) REG(3, 5, 2) REG(4, 5, 3) \
    REG(5, 5, 3) REG(2, 6, 1) REG(3, 6, 3) SLICED(8, 4, 3) SLICED(10, 4, 3) SLICED(6, 5, 3) SLICED(4, 6, 4) \
    SLICED(5, 6, 4) SLICED(10, 6, 4) REG(7, 2, 1) REG(9, 2, 1) REG(9, 3, 2) SLICED(9, 4, 3) SLICED(7, 5, 3) \
    SLICED(8, 5, 3) SLICED(9, 5, 3) SLICED(10, 5, 3)

#endif  // SIG_BACKWARD_H_

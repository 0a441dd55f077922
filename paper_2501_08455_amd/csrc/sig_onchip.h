// On-chip (register-resident) signature kernel, compiled per (d, depth N, prefix depth P).
//
// Lane ownership.  By the prefix-closure of the fused update (see sig_streaming.hip: the new
// coefficient of a word needs only old coefficients of its prefixes) the words below a fixed
// prefix u of length P evolve on their own.  A lane owns that sub-tree: 1 + d + ... + d^{N-P}
// floats in registers (contiguous index blocks of every level >= P of the output row), plus the
// P-1 scalars S[u_{1:m}] it shares with its neighbours and recomputes redundantly.  Q = d^P
// lanes cover one (path, time chunk); no lane ever needs another lane's registers.
//
// Time.  A path's K = L-1 increments are cut into `segments` (one workgroup each) times `chunks`
// (side by side inside a workgroup) pieces of `chunk_steps` increments.  Every piece is folded from
// the identity with the fused step of Eq. 3; pieces are joined with the product of Eq. 4, which
// is associative, in LDS (tree for the final signature, left-to-right scan for stream mode where
// every piece is then folded a second time from its carry-in while emitting each prefix).
//
// Loader.  Increments are staged through LDS: the workgroup reads the path with consecutive
// threads on consecutive floats, subtracts neighbouring points and stores rows of one increment
// each, double-buffered with the next tile's global loads in flight during the current tile's
// arithmetic.
#ifndef SIG_ONCHIP_H
#define SIG_ONCHIP_H

#include <type_traits>

#include "sig_internal.h"

namespace sig {
namespace onchip {

constexpr int cpow(int b, int e)
{
    int r = 1;
    for (int i = 0; i < e; ++i) r *= b;
    return r;
}

constexpr int kStage = kLoaderStage;

template <int d, int N, int P>
struct Shape {
    static_assert(P >= 0 && P < N, "prefix depth must leave at least one level to the lane");
    static constexpr int R = N - P;       // levels below the prefix word
    static constexpr int Q = cpow(d, P);  // lanes per (path, chunk)
    static constexpr int sub_off(int r)   // start of sub-level r (level P + r) in the lane's state
    {
        int s = 0, p = 1;
        for (int i = 0; i < r; ++i) { s += p; p *= d; }
        return s;
    }
    static constexpr int SZ = sub_off(R + 1);
    static constexpr int NPRE = P > 1 ? P - 1 : 1;
    static constexpr int row_off(int n)   // start of level n >= 1 in an output row
    {
        int s = 0, p = d;
        for (int i = 1; i < n; ++i) { s += p; p *= d; }
        return s;
    }
    static constexpr int D = row_off(N + 1);
    static constexpr int DP = (d + 3) / 4 * 4;  // LDS row of one increment, padded to float4
};

// registers of one lane: s = the sub-tree below its prefix word u (sub-level r at sub_off(r)),
// pre[m-1] = S[u_{1:m}] for m = 1 .. P-1
template <int d, int N, int P>
struct Lane {
    float s[Shape<d, N, P>::SZ];
    float pre[Shape<d, N, P>::NPRE];
};

// ------------------------------------------------------------------------------------------
// Fused step  S <- S (x) exp^N(v)  on one lane's sub-tree (Eq. 3 with Eqs. 2 and 4 expanded, Horner form).
//   dls[c-1][a] = v[a] / c ;  du[m-1] = v[u_m]
// Level n is updated from g_{n-1}, where g_0 = 1 and g_m[w a] = S_m[w a] + g_{m-1}[w] v[a] / (n - m + 1).
// Levels go from N down to 1 so that the old lower levels are still in place when needed.
template <int d, int N, int P, int n, int r>
struct Descend {
    using Sh = Shape<d, N, P>;
    // g belongs to the word (u, v) where v has index idx in sub-level r
    static __device__ __forceinline__ void run(float (&s)[Sh::SZ], const float (&dls)[N][d], float g, int idx)
    {
        constexpr int tgt = n - P;  // sub-level being updated
#pragma unroll
        for (int a = 0; a < d; ++a) {
            const int child = idx * d + a;
            if constexpr (r + 1 == tgt) {
                s[Sh::sub_off(tgt) + child] = fmaf(g, dls[0][a], s[Sh::sub_off(tgt) + child]);
            } else {
                float g2 = fmaf(g, dls[tgt - r - 1][a], s[Sh::sub_off(r + 1) + child]);
                Descend<d, N, P, n, r + 1>::run(s, dls, g2, child);
            }
        }
    }
};

template <int d, int N, int P, int n>
struct Level {
    using Sh = Shape<d, N, P>;
    static __device__ __forceinline__ void run(float (&s)[Sh::SZ], float (&pre)[Sh::NPRE],
                                               const float (&dls)[N][d], const float (&du)[P > 0 ? P : 1])
    {
        float g = 1.0f;
        constexpr int mtop = (n - 1 < P) ? n - 1 : P;
#pragma unroll
        for (int m = 1; m <= mtop; ++m) {
            const float Sm = (m < P) ? pre[m - 1] : s[0];
            g = fmaf(g, du[m - 1] * (1.0f / (float)(n - m + 1)), Sm);
        }
        if constexpr (n <= P) {
            if constexpr (n < P) pre[n - 1] = fmaf(g, du[n - 1], pre[n - 1]);
            else s[0] = fmaf(g, du[n - 1], s[0]);
        } else {
            Descend<d, N, P, n, 0>::run(s, dls, g, 0);
        }
        if constexpr (n > 1) Level<d, N, P, n - 1>::run(s, pre, dls, du);
    }
};

template <int d, int N, int P>
__device__ __forceinline__ void fused_step(Lane<d, N, P> &ln, const float *row, const int *letter)
{
    float dls[N][d];
    float du[P > 0 ? P : 1];
#pragma unroll
    for (int a = 0; a < d; ++a) dls[0][a] = row[a];
#pragma unroll
    for (int c = 2; c <= N; ++c)
#pragma unroll
        for (int a = 0; a < d; ++a) dls[c - 1][a] = dls[0][a] * (1.0f / (float)c);
    du[0] = 0.0f;
#pragma unroll
    for (int m = 0; m < P; ++m) du[m] = row[letter[m]];
    Level<d, N, P, N>::run(ln.s, ln.pre, dls, du);
}

// compile-time loop: f(std::integral_constant<int, I>) for I in [B, E)
template <int I, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// write / read a lane's state to / from a row laid out like an output row
template <int d, int N, int P>
__device__ __forceinline__ void store_state(float *row, unsigned u, const Lane<d, N, P> &ln)
{
    using Sh = Shape<d, N, P>;
    static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        constexpr int cnt = cpow(d, r);
        float *dst = row + Sh::row_off(P + r) + u * cnt;
#pragma unroll
        for (int i = 0; i < cnt; ++i) dst[i] = ln.s[Sh::sub_off(r) + i];
    });
    static_for<1, P>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        constexpr unsigned span = cpow(d, P - m);
        if (u % span == 0) row[Sh::row_off(m) + u / span] = ln.pre[m - 1];
    });
}

template <int d, int N, int P>
__device__ __forceinline__ void load_state(const float *row, unsigned u, Lane<d, N, P> &ln)
{
    using Sh = Shape<d, N, P>;
    static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        constexpr int cnt = cpow(d, r);
        const float *src = row + Sh::row_off(P + r) + u * cnt;
#pragma unroll
        for (int i = 0; i < cnt; ++i) ln.s[Sh::sub_off(r) + i] = src[i];
    });
    static_for<1, P>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        ln.pre[m - 1] = row[Sh::row_off(m) + u / (unsigned)cpow(d, P - m)];
    });
}

template <int d, int N, int P>
__device__ __forceinline__ void identity_state(Lane<d, N, P> &ln)
{
    using Sh = Shape<d, N, P>;
#pragma unroll
    for (int i = 0; i < Sh::SZ; ++i) ln.s[i] = 0.0f;
    if (P == 0) ln.s[0] = 1.0f;
#pragma unroll
    for (int i = 0; i < Sh::NPRE; ++i) ln.pre[i] = 0.0f;
}

// ------------------------------------------------------------------------------------------
// In-LDS product of Eq. 4 on rows of D floats, level by level from N down to 1 with a barrier
// after each level, so it may overwrite one of its operands:
//   c_n[w] = a_n[w] + b_n[w] + sum_{i=1}^{n-1} a_i[w / d^{n-i}] * b_{n-i}[w mod d^{n-i}]
// Products are addressed as (pair index) -> rows; TO_LEFT stores c over a, else over b.
template <int d, int N, int n, bool TO_LEFT, class PairRows>
__device__ __forceinline__ void lds_product_levels(float *sig, int npairs, PairRows rows, int tid, int nthr)
{
    using Sh = Shape<d, N, 0>;
    constexpr int sz = cpow(d, n);
    const int items = npairs * sz;
    for (int it = tid; it < items; it += nthr) {
        const int w = it % sz;
        const int pq = it / sz;
        int ia, ib;
        rows(pq, ia, ib);
        float *a = sig + ia * Sh::D;
        float *b = sig + ib * Sh::D;
        float c = a[Sh::row_off(n) + w] + b[Sh::row_off(n) + w];
        static_for<1, n>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int split = cpow(d, n - i);
            c = fmaf(a[Sh::row_off(i) + w / split], b[Sh::row_off(n - i) + w % split], c);
        });
        (TO_LEFT ? a : b)[Sh::row_off(n) + w] = c;
    }
    __syncthreads();
    if constexpr (n > 1) lds_product_levels<d, N, n - 1, TO_LEFT>(sig, npairs, rows, tid, nthr);
}

extern __shared__ float sig_onchip_smem[];

template <int d, int N, int P, int MAXT>
__global__ __launch_bounds__(MAXT) void sig_on_chip_kernel(OnChipArgs A)
{
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int DP = Sh::DP;
    constexpr int D = Sh::D;

    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int64_t K = A.L - 1;
    const int C = A.chunks, W = A.segments, T = A.chunk_steps, TT = A.tile_steps;
    const int64_t ngroups = A.B * W;  // (path, segment) pairs

    // ---- lane -> (group, chunk, prefix word)
    const bool big = Q > nthr;  // one chunk's lanes span several workgroups (then C == 1)
    int G, gi, c;
    unsigned u;
    int64_t group0;  // first group of this workgroup
    bool active;
    if (!big) {
        const int LG = C * Q;
        G = A.groups;
        gi = tid / LG;
        const int rem = tid - gi * LG;
        c = rem / Q;
        u = (unsigned)(rem - c * Q);
        group0 = (int64_t)blockIdx.x * G;
        active = gi < G && group0 + gi < ngroups;
        if (gi >= G) { gi = 0; c = 0; }
    } else {
        const int NB = (Q + nthr - 1) / nthr;
        G = 1;
        gi = 0;
        c = 0;
        group0 = blockIdx.x / NB;
        u = (unsigned)((blockIdx.x % NB) * nthr + tid);
        active = u < (unsigned)Q;
        if (!active) u = 0;
    }
    const int NGC = G * C;
    const int mygc = gi * C + c;
    int64_t mygroup = group0 + gi;
    if (mygroup >= ngroups) mygroup = ngroups - 1;
    const int64_t b = mygroup / W;
    const int seg = (int)(mygroup - b * W);
    const int64_t k_begin = ((int64_t)seg * C + c) * T;

    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    }

    // ---- LDS: two increment tiles, then the chunk signatures
    const int tile_floats = NGC * TT * DP;
    float *tile0 = sig_onchip_smem;
    float *sigrows = sig_onchip_smem + 2 * tile_floats;  // [NGC][D], used when C > 1

    // ---- loader.  Which floats of the path a thread stages does not depend on the tile, only the
    // time offset does, so the address and the number of valid steps are worked out once.
    float stage[kStage];
    const float *src[kStage];  // x[b][k0][a] of this thread's element e for the first tile
    int lim[kStage];           // element e is inside its chunk and inside the path while t0 < lim[e]
    const int tile_elems = NGC * TT * d;  // <= kStage * nthr (checked on the host)
#pragma unroll
    for (int e = 0; e < kStage; ++e) {
        const int idx = tid + e * nthr;
        src[e] = A.path;
        lim[e] = 0;
        if (idx < tile_elems) {
            const int gc = idx / (TT * d);
            const int r = idx - gc * (TT * d);
            const int t = r / d;
            const int g2 = gc / C;
            const int c2 = gc - g2 * C;
            const int64_t grp = group0 + g2;
            if (grp < ngroups) {
                const int64_t b2 = grp / W;
                const int64_t k0 = ((grp - b2 * W) * C + c2) * (int64_t)T + t;
                int64_t left = K - k0;
                if (left > T - t) left = T - t;
                lim[e] = left > 0 ? (int)left : 0;
                src[e] = A.path + (b2 * A.L + k0) * d + (r - t * d);
            }
        }
    }
    auto fetch_tile = [&](int t0) {  // global -> registers
#pragma unroll
        for (int e = 0; e < kStage; ++e) {
            float v = 0.0f;
            if (t0 < lim[e]) {
                const float *x = src[e] + (int64_t)t0 * d;
                v = x[d] - x[0];
            }
            stage[e] = v;
        }
    };
    auto commit_tile = [&](float *tile) {  // registers -> LDS rows of DP floats
#pragma unroll
        for (int e = 0; e < kStage; ++e) {
            const int idx = tid + e * nthr;
            if (idx < tile_elems) {
                const int row = idx / d;
                tile[row * DP + (idx - row * d)] = stage[e];
            }
        }
    };

    Lane<d, N, P> ln;

    // fold this lane's chunk, optionally emitting every prefix (stream mode)
    auto fold_chunk = [&](auto emit_tag) {
        constexpr bool emit = decltype(emit_tag)::value;
        const int ntile = (T + TT - 1) / TT;
        fetch_tile(0);
        commit_tile(tile0);
        __syncthreads();
        for (int i = 0; i < ntile; ++i) {
            float *cur = tile0 + (i & 1) * tile_floats;
            float *nxt = tile0 + ((i + 1) & 1) * tile_floats;
            const bool more = i + 1 < ntile;
            if (more) fetch_tile((i + 1) * TT);
            const int steps = (T - i * TT < TT) ? T - i * TT : TT;
            const float *row = cur + mygc * TT * DP;
            for (int t = 0; t < steps; ++t, row += DP) {
                fused_step<d, N, P>(ln, row, letter);
                if constexpr (emit) {
                    const int64_t k = k_begin + (int64_t)i * TT + t;
                    if (active && k < K) store_state<d, N, P>(A.out + (b * K + k) * D, u, ln);
                }
            }
            if (more) commit_tile(nxt);
            __syncthreads();
        }
    };

    identity_state<d, N, P>(ln);
    const bool stream = A.stream_flag != 0;
    // with one chunk per path, stream mode is a single emitting fold
    if (!(stream && C == 1)) fold_chunk(std::false_type{});

    if (C == 1 && !stream) {
        if (active) {
            float *dst = (W == 1) ? A.out + b * D : A.partial + mygroup * D;
            store_state<d, N, P>(dst, u, ln);
        }
        return;
    }

    // ---- several chunks per group: join them in LDS
    if (C > 1) {
        if (active) store_state<d, N, P>(sigrows + mygc * D, u, ln);
        __syncthreads();
    }

    if (!stream) {
        // pairwise tree: round with stride st joins chunk q*2st with chunk q*2st + st, result on the left
        for (int st = 1; st < C; st <<= 1) {
            const int per_group = (C - st + 2 * st - 1) / (2 * st);
            auto rows = [=](int pq, int &ia, int &ib) {
                const int g2 = pq / per_group;
                const int q = pq - g2 * per_group;
                ia = g2 * C + q * 2 * st;
                ib = ia + st;
            };
            lds_product_levels<d, N, N, true>(sigrows, G * per_group, rows, tid, nthr);
        }
        for (int idx = tid; idx < G * D; idx += nthr) {
            const int g2 = idx / D;
            const int pos = idx - g2 * D;
            const int64_t grp = group0 + g2;
            if (grp < ngroups) {
                float *dst = (W == 1) ? A.out + grp * D : A.partial + grp * D;
                dst[pos] = sigrows[(g2 * C) * D + pos];
            }
        }
        return;
    }

    // stream mode: inclusive scan left to right (chunk c2 <- chunk c2-1 (x) chunk c2), then every
    // chunk restarts from the signature of everything before it and emits each of its prefixes
    for (int c2 = 1; c2 < C; ++c2) {
        auto rows = [=](int pq, int &ia, int &ib) {
            ib = pq * C + c2;
            ia = ib - 1;
        };
        lds_product_levels<d, N, N, false>(sigrows, G, rows, tid, nthr);
    }
    if (c == 0) identity_state<d, N, P>(ln);
    else load_state<d, N, P>(sigrows + (mygc - 1) * D, u, ln);
    fold_chunk(std::true_type{});
}

// LDS bytes of a launch (same formula as in the kernel)
template <int d, int N, int P>
int64_t on_chip_lds_bytes(const OnChipArgs &A)
{
    using Sh = Shape<d, N, P>;
    const int64_t NGC = (int64_t)A.groups * A.chunks;
    int64_t floats = 2 * NGC * A.tile_steps * Sh::DP;
    if (A.chunks > 1) floats += NGC * Sh::D;
    return floats * (int64_t)sizeof(float);
}

template <int d, int N, int P>
hipError_t on_chip_launch(const OnChipArgs &A, hipStream_t st)
{
    using Sh = Shape<d, N, P>;
    const int64_t ngroups = A.B * A.segments;
    int64_t grid;
    if (Sh::Q > A.threads) {
        grid = ngroups * ((Sh::Q + A.threads - 1) / A.threads);
    } else {
        const int G = A.groups;
        if (G < 1 || (int64_t)G * A.chunks * Sh::Q > A.threads) return hipErrorInvalidValue;
        grid = (ngroups + G - 1) / G;
    }
    if (grid <= 0 || grid > INT32_MAX) return hipErrorInvalidValue;
    const int64_t lds = on_chip_lds_bytes<d, N, P>(A);
    if (lds > kMaxLdsBytes) return hipErrorInvalidValue;
    hipLaunchKernelGGL((sig_on_chip_kernel<d, N, P, 256>), dim3((unsigned)grid), dim3(A.threads), (size_t)lds, st, A);
    return hipGetLastError();
}

#define SIG_ON_CHIP_ENTRY(d, N, P)                                                        \
    {                                                                                     \
        d, N, P, ::sig::onchip::Shape<d, N, P>::Q, ::sig::onchip::Shape<d, N, P>::SZ,     \
            &::sig::onchip::on_chip_launch<d, N, P>, &::sig::onchip::on_chip_lds_bytes<d, N, P> \
    }

}  // namespace onchip
}  // namespace sig
#endif

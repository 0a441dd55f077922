// On-chip (register-resident) signature kernels, compiled per (d, depth N, prefix depth P).
//
// Lane ownership.  By the prefix-closure of the fused update (see sig_streaming.hip: the new
// coefficient of a word needs only old coefficients of its prefixes) the words below a fixed
// prefix u of length P evolve on their own.  A lane owns that sub-tree: 1 + d + ... + d^{N-P}
// floats in registers (contiguous index blocks of every level >= P of the output row), plus the
// P-1 scalars S[u_{1:m}] it shares with its neighbours and recomputes redundantly.  Q = d^P
// lanes cover one (path, time chunk); no lane ever needs another lane's registers.
//
// Occupancy.  One wavefront issues a vector instruction only every five to six cycles on this
// chip, so the fp32 rate needs three or more wavefronts per SIMD; the kernels are split by mode
// (final / stream, one chunk / several) so that each keeps its register count low.
//
// Time.  A path's K = L-1 increments are cut into `segments` (one workgroup each) times `chunks`
// (side by side inside a workgroup) pieces of `chunk_steps` increments.  Every piece is folded from
// the identity with the fused step of Eq. 3; pieces are joined with the product of Eq. 4, which
// is associative, in LDS (pairwise tree for the final signature, left-to-right scan for stream
// mode, where every piece is then folded a second time from its carry-in while emitting each prefix).
//
// Loader.  Increments are staged through LDS one tile of `tile_steps` steps at a time: the
// workgroup reads the path with consecutive lanes on consecutive floats, subtracts neighbouring
// points and stores one row per step.
#ifndef SIG_ONCHIP_H
#define SIG_ONCHIP_H

#include <type_traits>

#include "sig_internal.h"

// Wavefront priority of the phases that wait on HBM (staging increments, writing results).  The SIMD's
// arbiter favours older wavefronts, so a freshly started workgroup would otherwise issue its loads only in
// the gaps its neighbours' arithmetic leaves; with the priority raised the loads go out at once and the
// arithmetic of the other wavefronts fills the time they are in flight.
#ifndef SIG_FLAT_BATCH
#define SIG_FLAT_BATCH 3  // vectors per thread whose loads are in flight together in the straight-copy loader
#endif
#ifndef SIG_MEMORY_PHASE_PRIORITY
#define SIG_MEMORY_PHASE_PRIORITY 3
#endif
#define SIG_PRIO_MEMORY() __builtin_amdgcn_s_setprio(SIG_MEMORY_PHASE_PRIORITY)
#define SIG_PRIO_COMPUTE() __builtin_amdgcn_s_setprio(0)

namespace sig {
namespace onchip {

typedef float vec4f __attribute__((ext_vector_type(4)));  // plain 16-byte vector for LDS -> HBM row copies

constexpr int cpow(int b, int e)
{
    int r = 1;
    for (int i = 0; i < e; ++i) r *= b;
    return r;
}

constexpr int geom(int d, int terms)  // 1 + d + ... + d^(terms-1)
{
    int s = 0, p = 1;
    for (int i = 0; i < terms; ++i) { s += p; p *= d; }
    return s;
}

template <int d, int N, int P>
struct Shape {
    static_assert(P >= 0 && P < N, "prefix depth must leave at least one level to the lane");
    static constexpr int R = N - P;       // levels below the prefix word
    static constexpr int Q = cpow(d, P);  // lanes per (path, chunk)
    static constexpr int sub_off(int r) { return geom(d, r); }  // start of sub-level r (level P + r) in the lane's state
    static constexpr int SZ = geom(d, R + 1);
    static constexpr int NPRE = P > 1 ? P - 1 : 1;
    static constexpr int row_off(int n) { return geom(d, n) - 1; }  // start of level n >= 1 in an output row
    static constexpr int D = geom(d, N + 1) - 1;
};

// compile-time loop: f(std::integral_constant<int, I>) for I in [B, E)
template <int I, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// registers of one lane: s = the sub-tree below its prefix word u (sub-level r at sub_off(r)),
// pre[m-1] = S[u_{1:m}] for m = 1 .. P-1
template <int d, int N, int P>
struct Lane {
    float s[Shape<d, N, P>::SZ];
    float pre[Shape<d, N, P>::NPRE];
};

// ------------------------------------------------------------------------------------------
// Fused step  S <- S (x) exp^N(v)  on one lane's sub-tree (Eq. 3 with Eqs. 2 and 4 expanded, Horner form).
//   row[a] = v[a] (LDS);  dls[c-1][a] = v[a] / c;  du[m-1] = v[u_m]
// Level n is updated from g_{n-1}, where g_0 = 1 and g_m[w a] = S_m[w a] + g_{m-1}[w] v[a] / (n - m + 1).
// Levels go from N down to 1 so that the old lower levels are still in place when needed.
template <int d, int N, int P, int n, int r>
struct Descend {
    using Sh = Shape<d, N, P>;
    // g belongs to the word (u, v) where v has index idx in sub-level r
    static __device__ __forceinline__ void run(float (&s)[Sh::SZ], const float (&dls)[Sh::R][d], float g, int idx)
    {
        constexpr int tgt = n - P;  // sub-level being updated
#pragma unroll
        for (int a = 0; a < d; ++a) {
            const int child = idx * d + a;
            if constexpr (r + 1 == tgt) {
                s[Sh::sub_off(tgt) + child] = fmaf(g, dls[0][a], s[Sh::sub_off(tgt) + child]);
            } else if constexpr (r == 0) {
                // a single parent: scale it once (hoisted out of the loop over a) instead of scaling v
                float g2 = fmaf(g * (1.0f / (float)(tgt - r)), dls[0][a], s[Sh::sub_off(r + 1) + child]);
                Descend<d, N, P, n, r + 1>::run(s, dls, g2, child);
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
                                               const float (&dls)[Sh::R][d], const float (&du)[P > 0 ? P : 1])
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

// one staged increment as a lane needs it: all d components and the components at its own prefix letters
template <int d, int P>
struct Inc {
    float v[d];
    float du[P > 0 ? P : 1];
};

template <int d, int P>
__device__ __forceinline__ void load_inc(Inc<d, P> &inc, const float *row, const int *letter)
{
#pragma unroll
    for (int a = 0; a < d; ++a) inc.v[a] = row[a];
    inc.du[0] = 0.0f;
#pragma unroll
    for (int m = 0; m < P; ++m) inc.du[m] = row[letter[m]];
}

template <int d, int N, int P>
__device__ __forceinline__ void fused_step(Lane<d, N, P> &ln, const Inc<d, P> &inc)
{
    using Sh = Shape<d, N, P>;
    float dls[Sh::R][d];
    // the scaled copies v/2 .. v/R cost a multiply each, which is cheaper than reading them from LDS
    // (one LDS serves four SIMDs)
#pragma unroll
    for (int a = 0; a < d; ++a) dls[0][a] = inc.v[a];
#pragma unroll
    for (int c = 1; c < Sh::R; ++c)
#pragma unroll
        for (int a = 0; a < d; ++a) dls[c][a] = inc.v[a] * (1.0f / (float)(c + 1));
    Level<d, N, P, N>::run(ln.s, ln.pre, dls, inc.du);
}

// 16- and 8-byte vectors that are only 4-byte aligned: a lane's blocks start at multiples of d^r floats, so
// their alignment varies from lane to lane, and the hardware takes dword-aligned vector accesses
typedef float vec4f_u __attribute__((ext_vector_type(4), aligned(4)));
typedef float vec2f_u __attribute__((ext_vector_type(2), aligned(4)));

// copy CNT consecutive registers s[OFF ..] to dst[0 ..] with the widest stores
template <int OFF, int CNT, int SZ>
__device__ __forceinline__ void store_run(float *dst, const float (&s)[SZ])
{
    if constexpr (CNT >= 4) {
        vec4f_u v = {s[OFF], s[OFF + 1], s[OFF + 2], s[OFF + 3]};
        *reinterpret_cast<vec4f_u *>(dst) = v;
        store_run<OFF + 4, CNT - 4, SZ>(dst + 4, s);
    } else if constexpr (CNT >= 2) {
        vec2f_u v = {s[OFF], s[OFF + 1]};
        *reinterpret_cast<vec2f_u *>(dst) = v;
        store_run<OFF + 2, CNT - 2, SZ>(dst + 2, s);
    } else if constexpr (CNT == 1) {
        dst[0] = s[OFF];
    }
}

// write / read a lane's state to / from a row laid out like an output row
template <int d, int N, int P>
__device__ __forceinline__ void store_state(float *row, unsigned u, const Lane<d, N, P> &ln)
{
    using Sh = Shape<d, N, P>;
    static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) __attribute__((always_inline)) {
        constexpr int r = decltype(rc)::value;
        constexpr int cnt = cpow(d, r);
        store_run<Sh::sub_off(r), cnt, Sh::SZ>(row + Sh::row_off(P + r) + u * cnt, ln.s);
    });
    static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
        constexpr int m = decltype(mc)::value;
        constexpr unsigned span = cpow(d, P - m);
        if (u % span == 0) row[Sh::row_off(m) + u / span] = ln.pre[m - 1];
    });
}

template <int d, int N, int P>
__device__ __forceinline__ void load_state(const float *row, unsigned u, Lane<d, N, P> &ln)
{
    using Sh = Shape<d, N, P>;
    static_for<(P == 0 ? 1 : 0), Sh::R + 1>([&](auto rc) __attribute__((always_inline)) {
        constexpr int r = decltype(rc)::value;
        constexpr int cnt = cpow(d, r);
        const float *src = row + Sh::row_off(P + r) + u * cnt;
#pragma unroll
        for (int i = 0; i < cnt; ++i) ln.s[Sh::sub_off(r) + i] = src[i];
    });
    static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
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
// Product of Eq. 4 on rows of D floats:  c = a (x) b,  c not overlapping a or b.
//   c_n[w] = a_n[w] + b_n[w] + sum_{i=1}^{n-1} a_i[w_{1:i}] * b_{n-i}[w_{i+1:n}]
// One work item is a parent word v of length n-1 (levels n = 1..N, geom(d, N) items in all); it
// produces the d children v.j: the a-factors depend on v only and the b-factors are contiguous in j.
template <int d, int N>
struct RowProduct {
    using Sh = Shape<d, N, 0>;
    static constexpr int ITEMS = geom(d, N);

    static __device__ __forceinline__ void item(const float *a, const float *b, float *c, int it)
    {
        static_for<1, N + 1>([&](auto nc) __attribute__((always_inline)) {
            constexpr int n = decltype(nc)::value;
            constexpr int start = geom(d, n - 1);
            constexpr int cnt = cpow(d, n - 1);
            if (it >= start && it < start + cnt) {
                const int v = it - start;
                float acc[d];
#pragma unroll
                for (int j = 0; j < d; ++j) acc[j] = a[Sh::row_off(n) + v * d + j] + b[Sh::row_off(n) + v * d + j];
                static_for<1, n>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int i = decltype(ic)::value;
                    constexpr int tail = cpow(d, n - 1 - i);  // words of length n-1-i between the prefix and j
                    const float ai = a[Sh::row_off(i) + v / tail];
                    const float *bs = b + Sh::row_off(n - i) + (v % tail) * d;
#pragma unroll
                    for (int j = 0; j < d; ++j) acc[j] = fmaf(ai, bs[j], acc[j]);
                });
#pragma unroll
                for (int j = 0; j < d; ++j) c[Sh::row_off(n) + v * d + j] = acc[j];
            }
        });
    }
};


// Pairwise tree over `rows` consecutive rows of each of G groups in LDS, ping-pong between two buffers;
// the left-to-right order of the factors is kept.  On return src / src_stride address the results
// (row 0 of every group).  Every thread of the workgroup must call it (it contains barriers).
template <int d, int N>
__device__ __forceinline__ void lds_tree_reduce(float *&src, float *&dst, int G, int rows, int &src_stride,
                                                int &dst_stride, int tid, int nthr)
{
    using RP = RowProduct<d, N>;
    constexpr int D = Shape<d, N, 0>::D;
    while (rows > 1) {
        const int pairs = rows / 2;
        const int total = G * pairs * RP::ITEMS;
        for (int x = tid; x < total; x += nthr) {
            const int pq = x / RP::ITEMS;
            const int it = x - pq * RP::ITEMS;
            const int g2 = pq / pairs;
            const int q = pq - g2 * pairs;
            const float *a = src + (g2 * src_stride + 2 * q) * D;
            RP::item(a, a + D, dst + (g2 * dst_stride + q) * D, it);
        }
        if (rows & 1) {  // odd row out: carried to the next round unchanged
            for (int x = tid; x < G * D; x += nthr) {
                const int g2 = x / D;
                const int pos = x - g2 * D;
                dst[(g2 * dst_stride + pairs) * D + pos] = src[(g2 * src_stride + rows - 1) * D + pos];
            }
        }
        __syncthreads();
        rows = (rows + 1) / 2;
        float *tmp = src; src = dst; dst = tmp;
        const int ts = src_stride; src_stride = dst_stride; dst_stride = ts;
    }
}


// ------------------------------------------------------------------------------------------
// Product of Eq. 4 with the left factor in registers:  ln <- ln (x) b,  b a row of D floats (LDS).
// A lane holds the left factor's coefficients of the words below its prefix u and of u's own prefixes, which
// are exactly the a-factors its words need:
//   c[u v] = a[u v] + b[u v] + sum_{i=1}^{P} a[u_{1:i}] b[(u_{i+1:P}, v)] + sum_{j=1}^{r-1} a[u v_{1:j}] b[v_{j+1:r}]
// for a word (u, v), |v| = r >= 1, and for the prefix words u_{1:n}, n <= P,
//   c[u_{1:n}] = a[u_{1:n}] + b[u_{1:n}] + sum_{i=1}^{n-1} a[u_{1:i}] b[u_{i+1:n}].
// The b-factors are suffix words: runs of d^r consecutive floats at lane-dependent offsets.  Levels go from
// N down to 1 so that the result can replace the left factor in place.
// BATCH: every run of b is read into registers in one go and only then used (a scheduling fence keeps the loads
// together).  That costs about a dozen registers; it pays in the join kernel, which runs one workgroup per path
// with nothing else to hide the LDS latency (the compiler's own order waits once per handful of reads), and
// loses in the fold kernels, where the registers are worth a wavefront of occupancy.
#ifndef SIG_TREE_BATCH
#define SIG_TREE_BATCH false
#endif
template <int d, int N, int P, bool BATCH = false>
__device__ __forceinline__ void reg_product(Lane<d, N, P> &ln, const float *b, unsigned u)
{
    using Sh = Shape<d, N, P>;
    // a[u_{1:i}] for i = 1..P (old values, kept while the prefix words are updated last)
    float apre[P > 0 ? P : 1];
    apre[0] = 0.0f;
    static_for<1, P + 1>([&](auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        apre[i - 1] = (i < P) ? ln.pre[i - 1] : ln.s[0];
    });
    // sub-tree levels, deepest first
    static_for<0, Sh::R>([&](auto qc) __attribute__((always_inline)) {
        constexpr int r = Sh::R - decltype(qc)::value;  // R .. 1
        constexpr int n = P + r;
        constexpr int cnt = cpow(d, r);
        float acc[cnt];
        float tmp[cnt];
        const float *bn = b + Sh::row_off(n) + u * cnt;
#pragma unroll
        for (int v = 0; v < cnt; ++v) tmp[v] = bn[v];
        if constexpr (BATCH) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int v = 0; v < cnt; ++v) acc[v] = ln.s[Sh::sub_off(r) + v] + tmp[v];
        // a-factors that are prefixes of u: b-factor (u_{i+1:P}, v) is a run of cnt floats of level n - i
        static_for<1, P + 1>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            const float *bs = b + Sh::row_off(n - i) + (u % (unsigned)cpow(d, P - i)) * cnt;
#pragma unroll
            for (int v = 0; v < cnt; ++v) tmp[v] = bs[v];
            if constexpr (BATCH) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int v = 0; v < cnt; ++v) acc[v] = fmaf(apre[i - 1], tmp[v], acc[v]);
        });
        // a-factors inside the sub-tree: a[u v_{1:j}] times b[v_{j+1:r}]
        static_for<1, r>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            constexpr int tail = cpow(d, r - j);
            const float *bs = b + Sh::row_off(r - j);
#pragma unroll
            for (int v = 0; v < cnt; ++v) acc[v] = fmaf(ln.s[Sh::sub_off(j) + v / tail], bs[v % tail], acc[v]);
        });
#pragma unroll
        for (int v = 0; v < cnt; ++v) ln.s[Sh::sub_off(r) + v] = acc[v];
    });
    // prefix words u_{1:n}, n = P .. 1 (every lane keeps its own copy)
    static_for<0, P>([&](auto qc) __attribute__((always_inline)) {
        constexpr int n = P - decltype(qc)::value;  // P .. 1
        float acc = apre[n - 1] + b[Sh::row_off(n) + u / (unsigned)cpow(d, P - n)];
        static_for<1, n>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            // suffix u_{i+1:n}: letters i+1..n of u
            const unsigned suffix = (u / (unsigned)cpow(d, P - n)) % (unsigned)cpow(d, n - i);
            acc = fmaf(apre[i - 1], b[Sh::row_off(n - i) + suffix], acc);
        });
        if constexpr (n < P) ln.pre[n - 1] = acc;
        else ln.s[0] = acc;
    });
}

extern __shared__ __align__(16) float sig_onchip_smem[];

// per (group, chunk) of a workgroup: where its increments start in the path and how many it has
struct ChunkDesc {
    int64_t base;      // float offset of x[b][k_begin][0] in the path array
    int64_t out_row0;  // stream mode: float offset of out[b][k_begin][0]
    int32_t steps;     // valid increments of this chunk (0 for chunks beyond the path or the batch)
    int32_t pad[3];
};

constexpr int kStage = kLoaderStage;  // floats of the next tile a thread holds in registers (PIPE kernels)

// floats of LDS in front of the increment tiles (descriptors, 32 bytes each)
__host__ __device__ constexpr int desc_floats(int ngc) { return 8 * ngc; }
__host__ __device__ constexpr int round4(int x) { return (x + 3) / 4 * 4; }

// CHUNKED: several time chunks per group, joined in LDS.  STREAM: every prefix is emitted.
// PIPE: the chunk spans several LDS tiles; the next tile's global loads are kept in flight in
// registers while the current tile is consumed (one barrier per tile).
// largest workgroup a kernel is built for (512 threads leave 256 registers per lane)
template <int d, int N, int P, bool CHUNKED>
constexpr int max_threads() { return (CHUNKED && Shape<d, N, P>::SZ <= 64) ? 512 : 256; }

// Workgroups of the CHUNKED kernels may have up to 512 threads (when the lane state is small enough): only chunks * Q lanes fold, but every
// thread takes part in the LDS products, which are latency bound with one wavefront per SIMD.
template <int d, int N, int P, bool CHUNKED, bool STREAM, bool PIPE, bool FLAT = false>
__global__ __launch_bounds__((max_threads<d, N, P, CHUNKED>())) void sig_on_chip_kernel(OnChipArgs A)
{
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;

    SIG_PRIO_MEMORY();
    // Skewed start.  All workgroups of a launch would otherwise load, fold and store in lock-step, and
    // the HBM phases would not overlap the arithmetic.  The workgroups that are resident first are delayed by
    // their residency slot (about blockIdx / number of CUs) times a fraction of one workgroup's lifetime;
    // later workgroups start when earlier ones retire and inherit the skew.  The wait ends by the clock.
    if (!CHUNKED && A.stagger_ticks > 0 && (int)blockIdx.x < A.resident_workgroups) {
        const unsigned long long until =
            wall_clock64() + (unsigned long long)(blockIdx.x / (unsigned)A.num_cus) * (unsigned long long)A.stagger_ticks;
        while (wall_clock64() < until) __builtin_amdgcn_s_sleep(32);
    }
    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int64_t K = A.L - 1;
    const int C = CHUNKED ? A.chunks : 1;
    const int W = A.segments, T = A.chunk_steps, TT = A.tile_steps;
    const unsigned ngroups = (unsigned)(A.B * W);  // (path, segment) pairs; fits 31 bits (checked on the host)

    // ---- lane -> (group, chunk, prefix word)
    const bool big = Q > nthr;  // one chunk's lanes span several workgroups (then C == 1)
    int G, gi, c;
    unsigned u, group0;  // group0: first group of this workgroup
    bool active;
    // Stream kernels with Q <= 64 keep every (group, chunk) slot inside one wavefront (64 / Q slots per
    // wavefront, the remaining lanes idle) so that a wavefront can gather its slots' rows in LDS and write
    // them out with consecutive lanes on consecutive addresses, without a workgroup barrier per step.
    constexpr bool WAVE_SLOTS = STREAM && Q <= kWave;
    constexpr int SPW = WAVE_SLOTS ? kWave / Q : 1;  // slots per wavefront
    if constexpr (WAVE_SLOTS) {
        const int wave = tid / kWave, lw = tid - wave * kWave;
        const int sw = lw / Q;
        const int slot = wave * SPW + sw;
        G = A.groups;
        u = (unsigned)(lw - sw * Q);
        gi = slot / C;
        c = slot - gi * C;
        group0 = blockIdx.x * (unsigned)G;
        active = sw < SPW && gi < G && group0 + gi < ngroups;
        if (sw >= SPW || gi >= G) { gi = 0; c = 0; }
    } else if (!big) {
        const int LG = C * Q;
        G = A.groups;
        gi = tid / LG;
        const int rem = tid - gi * LG;
        c = CHUNKED ? rem / Q : 0;
        u = (unsigned)(rem - c * Q);
        group0 = blockIdx.x * (unsigned)G;
        active = gi < G && group0 + gi < ngroups;
        if (gi >= G) { gi = 0; c = 0; }
    } else {
        const unsigned NB = (Q + nthr - 1) / nthr;
        G = 1;
        gi = 0;
        c = 0;
        group0 = blockIdx.x / NB;
        u = (blockIdx.x % NB) * nthr + tid;
        active = u < (unsigned)Q;
        if (!active) u = 0;
    }
    const int NGC = G * C;
    const int mygc = gi * C + c;

    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    }

    // ---- LDS: chunk descriptors, one or two increment tiles, then (CHUNKED) the chunk signatures
    ChunkDesc *desc = reinterpret_cast<ChunkDesc *>(sig_onchip_smem);
    const int row_floats = TT * d;                      // one chunk's part of a tile, rows of d floats, unpadded
    const int tile_floats = round4(NGC * row_floats);
    float *tile0 = sig_onchip_smem + desc_floats(NGC);
    // [NGC][D]: chunk signatures, and the rows staged for emission; behind the tile(s) (the straight-copy tile
    // holds rows of L * d floats plus up to three floats of alignment)
    float *sigA = tile0 + (FLAT ? round4(G * (int)A.L * d + 3) : (PIPE ? 2 : 1) * tile_floats);
    (void)sigA;

    if (tid < NGC) {
        const unsigned g2 = (unsigned)tid / (unsigned)C;
        const unsigned c2 = (unsigned)tid - g2 * C;
        const unsigned grp = group0 + g2;
        ChunkDesc dsc;
        dsc.base = 0;
        dsc.out_row0 = 0;
        dsc.steps = 0;
        dsc.pad[0] = dsc.pad[1] = dsc.pad[2] = 0;
        if (grp < ngroups) {
            const unsigned b2 = grp / (unsigned)W;
            const int64_t k0 = (int64_t)((grp - b2 * W) * C + c2) * T;
            int64_t left = K - k0;
            if (left > T) left = T;
            if (left > 0) {
                dsc.steps = (int)left;
                dsc.base = ((int64_t)b2 * A.L + k0) * d;
                dsc.out_row0 = ((int64_t)b2 * K + k0) * D;
            }
        }
        desc[tid] = dsc;
    }

    // Loader.  A tile is addressed as [chunk][r] with r < row_floats padded to a power of two
    // (A.row_shift), so consecutive threads read consecutive floats of one chunk's stretch of the path.
    const int rshift = A.row_shift;
    const int rmask = (1 << rshift) - 1;
    const int flat = NGC << rshift;
    auto fetch_one = [&](int idx, int t0) -> float {
        const int gc = idx >> rshift;
        const int r = idx & rmask;
        float v = 0.0f;
        if (idx < flat && r < row_floats) {
            const ChunkDesc dsc = desc[gc];
            if (r < (dsc.steps - t0) * d) {
                const float *x = A.path + dsc.base + (int64_t)t0 * d + r;
                v = x[d] - x[0];
            }
        }
        return v;
    };
    auto put_one = [&](float *tile, int idx, float v) {
        const int gc = idx >> rshift;
        const int r = idx & rmask;
        if (idx < flat && r < row_floats) tile[gc * row_floats + r] = v;
    };

    const bool vec_ok = (reinterpret_cast<uintptr_t>(A.out) & 15) == 0;  // rows of D floats, D % 4 == 0, stay 16-byte aligned
    (void)vec_ok;
    Lane<d, N, P> ln;
    int64_t b = 0, k_begin = 0;
    unsigned mygroup = 0;
    if (active) {
        mygroup = group0 + gi;
        const unsigned bb = mygroup / (unsigned)W;
        b = bb;
        k_begin = (int64_t)((mygroup - bb * W) * C + c) * T;
    }

    // fold this lane's chunk, optionally emitting every prefix (stream mode)
    auto fold_chunk = [&](auto emit_tag) __attribute__((always_inline)) {
        constexpr bool emit = decltype(emit_tag)::value;
        // Emission through LDS (WAVE_SLOTS): the rows of a wavefront's slots form one flat range of
        // vectors; lane lw copies elements lw, lw + 64, ...  Which slot and column an element belongs to
        // does not change from step to step, so the output address at step 0 of the chunk, the LDS offset
        // and the number of valid steps are worked out once per lane (NIT elements).
        constexpr int VEC = (D % 4 == 0) ? 4 : 1;
        constexpr int ROWV = D / VEC;
        constexpr int NIT = (SPW * ROWV + kWave - 1) / kWave;
        constexpr bool FAST_EMIT = emit && WAVE_SLOTS && NIT <= 8;
        using V = std::conditional_t<VEC == 4, vec4f, float>;
        V *eptr[FAST_EMIT ? NIT : 1];  // output address of the element at step 0 of its chunk
        int eoff[FAST_EMIT ? NIT : 1];  // offset (in vectors) into the staged rows
        int elim[FAST_EMIT ? NIT : 1];  // steps for which the element is written (0: never)
        const bool use_vec = VEC == 1 || vec_ok;
        if constexpr (FAST_EMIT) {
            const int wave = tid / kWave, lw = tid - wave * kWave;
#pragma unroll
            for (int j = 0; j < NIT; ++j) {
                const int i = lw + j * kWave;
                const int sw = i / ROWV;
                const int col = i - sw * ROWV;
                const int slot = wave * SPW + sw;
                eptr[j] = reinterpret_cast<V *>(A.out);
                eoff[j] = 0;
                elim[j] = 0;
                if (use_vec && i < SPW * ROWV && slot < NGC) {
                    eptr[j] = reinterpret_cast<V *>(A.out + desc[slot].out_row0) + col;
                    eoff[j] = slot * ROWV + col;
                    elim[j] = desc[slot].steps;
                }
            }
        }
        auto consume = [&](const float *tile, int t0, int row_stride) {
            const int steps = (T - t0 < TT) ? T - t0 : TT;
            const float *row = tile + mygc * row_stride;
            Inc<d, P> inc;
            int t = 0;
            if constexpr (!emit && Sh::SZ <= 40) {
                // small lane states, final mode: two steps per round, both increments read first (one wait and one set of
                // address updates per pair; the seven extra registers cost no occupancy at these state sizes)
                Inc<d, P> inc2;
                for (; t + 1 < steps; t += 2, row += 2 * d) {
                    load_inc<d, P>(inc, row, letter);
                    load_inc<d, P>(inc2, row + d, letter);
                    fused_step<d, N, P>(ln, inc);
                    fused_step<d, N, P>(ln, inc2);
                }
            }
            for (; t < steps; ++t, row += d) {
                load_inc<d, P>(inc, row, letter);
                fused_step<d, N, P>(ln, inc);
                if constexpr (emit && WAVE_SLOTS) {
                    // gather this wavefront's rows in LDS, then write them with consecutive lanes on
                    // consecutive addresses (LDS operations of one wavefront execute in order)
                    if (active) store_state<d, N, P>(sigA + mygc * D, u, ln);
                    if (FAST_EMIT && use_vec) {
                        if constexpr (FAST_EMIT) {
                            V val[NIT];
#pragma unroll
                            for (int j = 0; j < NIT; ++j) val[j] = reinterpret_cast<const V *>(sigA)[eoff[j]];
#pragma unroll
                            for (int j = 0; j < NIT; ++j)
                                if (t0 + t < elim[j]) eptr[j][(int64_t)(t0 + t) * ROWV] = val[j];
                        }
                    } else {
                        // rows too long for the per-lane element table: slot by slot (both loop bounds are the
                        // same for the whole wavefront), consecutive lanes on consecutive vectors of the row
                        const int wave = tid / kWave, lw = tid - wave * kWave;
                        for (int sw = 0; sw < SPW; ++sw) {
                            const int slot = wave * SPW + sw;
                            if (slot >= NGC) break;
                            if (t0 + t >= desc[slot].steps) continue;
                            float *dst = A.out + desc[slot].out_row0 + (int64_t)(t0 + t) * D;
                            const float *src = sigA + slot * D;
                            if (VEC == 4 && use_vec) {
                                for (int col = lw; col < ROWV; col += kWave)
                                    reinterpret_cast<vec4f *>(dst)[col] = reinterpret_cast<const vec4f *>(src)[col];
                            } else {
                                for (int col = lw; col < D; col += kWave) dst[col] = src[col];
                            }
                        }
                    }
                } else if constexpr (emit) {
                    const int64_t k = k_begin + t0 + t;
                    if (active && k < K) store_state<d, N, P>(A.out + (b * K + k) * D, u, ln);
                }
            }
        };
        if constexpr (!PIPE) {
            if constexpr (FLAT) {
                // One tile, whole paths, one segment: the groups of this workgroup are one contiguous range of
                // the path array.  Thread i takes vectors i, i + nthr, ... of that range (from the 16-byte
                // boundary below its start), loads each and the one d floats further on, and writes their
                // difference to the same place in the tile, so row g of the tile starts at g * L * d floats
                // and its last d entries (differences across two paths) are never consumed.  No index
                // arithmetic per vector and all loads of a batch in flight together.  The last vectors of
                // the array are taken from the last position that can be read in full.
                constexpr int LB = SIG_FLAT_BATCH;
                const int64_t NF = A.B * A.L * d;
                const int row_stride = (int)A.L * d;
                const int64_t F0 = (int64_t)group0 * row_stride;
                const int mis = (int)(F0 & 3);
                const int64_t F0a = F0 - mis;
                int64_t nfl = (int64_t)G * row_stride + mis;
                if (nfl > NF - F0a) nfl = NF - F0a;
                const int nvec = (int)((nfl + 3) >> 2);
                // last float offset from which both vectors can be read in full; taken in 64 bits (the path array may
                // hold 2^31 floats or more) and clamped to the tile before narrowing.  >= 0: checked on the host
                const int64_t qlast = NF - d - 4 - F0a;
                const int qmax = (int)(qlast < (int64_t)4 * nvec ? qlast : (int64_t)4 * nvec);
                const float *src = A.path + F0a;
                __syncthreads();
                SIG_PRIO_MEMORY();
                for (int base = 0; base < nvec; base += LB * nthr) {
                    vec4f_u lo[LB], hi[LB];
                    int off[LB];
#pragma unroll
                    for (int e = 0; e < LB; ++e) {
                        int i = base + e * nthr + tid;
                        if (i > nvec - 1) i = nvec - 1;
                        int q = 4 * i;
                        if (q > qmax) q = qmax;
                        off[e] = q;
                        lo[e] = *reinterpret_cast<const vec4f_u *>(src + q);
                        hi[e] = *reinterpret_cast<const vec4f_u *>(src + q + d);
                    }
#pragma unroll
                    for (int e = 0; e < LB; ++e) *reinterpret_cast<vec4f_u *>(tile0 + off[e]) = hi[e] - lo[e];
                }
                __syncthreads();
                SIG_PRIO_COMPUTE();
                consume(tile0 + mis, 0, row_stride);
            } else {
            for (int t0 = 0; t0 < T; t0 += TT) {
                __syncthreads();
                SIG_PRIO_MEMORY();
                // One element = four consecutive increments of one chunk's row (dword-aligned 16-byte loads of
                // the points and of the points d floats on).  The loads of a batch of elements are issued
                // together and nothing waits inside a branch.  The last element of a row is taken from the
                // last position that lies in the row in full (valid - 4), so no load is split; what a tile
                // row holds beyond the chunk's end is zero (an increment of zero leaves the state unchanged).
                // (the lane state is live here: with a small state one more element in flight costs a whole
                // wavefront of occupancy, and measured slower even on the shapes bound by reading the path; with a
                // large state the occupancy is low anyway)
                constexpr int LB = Sh::SZ <= 64 ? 1 : 3;
                const int vshift = rshift > 2 ? rshift - 2 : 0;  // vectors per chunk row, padded to a power of two
                const int vmask = (1 << vshift) - 1;
                const int vflat = NGC << vshift;
                for (int base = 0; base < vflat; base += LB * nthr) {
                    vec4f_u lo[LB], hi[LB];
                    int qv[LB];  // position of the loaded vector in its row, or -1 if none was loaded
#pragma unroll
                    for (int e = 0; e < LB; ++e) {
                        const int idx = base + e * nthr + tid;
                        const int gc = idx >> vshift;
                        const int r = (idx & vmask) * 4;
                        qv[e] = -1;
                        lo[e] = vec4f_u{0.0f, 0.0f, 0.0f, 0.0f};
                        hi[e] = lo[e];
                        if (idx < vflat && r < row_floats) {
                            const ChunkDesc dsc = desc[gc];
                            int valid = (dsc.steps - t0) * d;  // floats of this chunk still inside the path
                            if (valid > row_floats) valid = row_floats;
                            if (valid >= 4 && r < valid) {
                                const int q = r < valid - 4 ? r : valid - 4;
                                const float *x = A.path + dsc.base + (int64_t)t0 * d + q;
                                lo[e] = *reinterpret_cast<const vec4f_u *>(x);
                                hi[e] = *reinterpret_cast<const vec4f_u *>(x + d);
                                qv[e] = q;
                            }
                        }
                    }
#pragma unroll
                    for (int e = 0; e < LB; ++e) {
                        const int idx = base + e * nthr + tid;
                        const int gc = idx >> vshift;
                        const int r = (idx & vmask) * 4;
                        if (idx < vflat && r < row_floats) {
                            float *trow = tile0 + gc * row_floats;
                            if (qv[e] >= 0) *reinterpret_cast<vec4f_u *>(trow + qv[e]) = hi[e] - lo[e];
                            const ChunkDesc dsc = desc[gc];
                            int valid = (dsc.steps - t0) * d;
                            if (valid > row_floats) valid = row_floats;
                            if (valid < 0) valid = 0;
                            if (r + 4 > valid) {
                                // the end of the row: zeros beyond the chunk, and rows shorter than one vector float by float
                                const float *x = A.path + dsc.base + (int64_t)t0 * d;
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const int pos = r + j;
                                    if (pos < row_floats) {
                                        if (pos >= valid) trow[pos] = 0.0f;
                                        else if (valid < 4) trow[pos] = x[pos + d] - x[pos];
                                    }
                                }
                            }
                        }
                    }
                }
                __syncthreads();
                SIG_PRIO_COMPUTE();
                consume(tile0, t0, row_floats);
            }
            }
        } else {
            float stage[kStage];  // flat <= kStage * nthr (checked on the host)
            __syncthreads();
#pragma unroll
            for (int e = 0; e < kStage; ++e) stage[e] = fetch_one(tid + e * nthr, 0);
#pragma unroll
            for (int e = 0; e < kStage; ++e) put_one(tile0, tid + e * nthr, stage[e]);
            __syncthreads();
            SIG_PRIO_COMPUTE();
            int buf = 0;
            for (int t0 = 0; t0 < T; t0 += TT, buf ^= 1) {
                const bool more = t0 + TT < T;
                if (more) {
#pragma unroll
                    for (int e = 0; e < kStage; ++e) stage[e] = fetch_one(tid + e * nthr, t0 + TT);
                }
                consume(tile0 + buf * tile_floats, t0, row_floats);
                if (more) {
#pragma unroll
                    for (int e = 0; e < kStage; ++e) put_one(tile0 + (buf ^ 1) * tile_floats, tid + e * nthr, stage[e]);
                }
                __syncthreads();
            }
        }
    };

    identity_state<d, N, P>(ln);
    __syncthreads();  // descriptors visible

    if constexpr (!CHUNKED) {
        fold_chunk(std::integral_constant<bool, STREAM>{});
        SIG_PRIO_MEMORY();
        if constexpr (!STREAM) {
            if (active) {
                float *dst = (W == 1) ? A.out + b * D : A.partial + (int64_t)mygroup * D;
                store_state<d, N, P>(dst, u, ln);
            }
        }
    } else {
        using RP = RowProduct<d, N>;
        fold_chunk(std::false_type{});
        if constexpr (!STREAM && Sh::SZ <= 64) {
            // pairwise tree with the left factor in registers: in the round with stride st chunk c (a multiple
            // of 2 st) absorbs chunk c + st, which has put its row into LDS; the result stays in c's lanes.
            // Only every other surviving chunk writes a row per round, so a group needs (C + 1) / 2 rows,
            // and they take the place of the increment tiles, which are dead by now.
            __syncthreads();  // every lane is done with the tiles
            float *rows = tile0;
            const int HC = (C + 1) / 2;
            for (int st = 1; st < C; st <<= 1) {
                float *slot = rows + (gi * HC + c / (2 * st)) * D;  // of the pair (c, c + st)
                if (active && (c & (2 * st - 1)) == st) store_state<d, N, P>(slot, u, ln);
                __syncthreads();
                if (active && (c & (2 * st - 1)) == 0 && c + st < C) reg_product<d, N, P, SIG_TREE_BATCH>(ln, slot, u);
                if (2 * st < C) __syncthreads();  // the slots are rewritten in the next round
            }
            if (active && c == 0) {
                float *o = (W == 1) ? A.out + (int64_t)mygroup * D : A.partial + (int64_t)mygroup * D;
                store_state<d, N, P>(o, u, ln);
            }
        } else {
        if (active) store_state<d, N, P>(sigA + mygc * D, u, ln);
        float *sigB = sigA + NGC * D;  // second buffer: [G][(C+1)/2][D] (final) or [NGC][D] (stream)
        __syncthreads();
        if constexpr (!STREAM) {
            float *src = sigA, *dst = sigB;
            int src_stride = C, dst_stride = (C + 1) / 2;
            lds_tree_reduce<d, N>(src, dst, G, C, src_stride, dst_stride, tid, nthr);
            for (int x = tid; x < G * D; x += nthr) {
                const int g2 = x / D;
                const int pos = x - g2 * D;
                const unsigned grp = group0 + g2;
                if (grp < ngroups) {
                    float *o = (W == 1) ? A.out + (int64_t)grp * D : A.partial + (int64_t)grp * D;
                    o[pos] = src[(g2 * src_stride) * D + pos];
                }
            }
        } else {
            // inclusive scan left to right into the second buffer: B[0] = A[0], B[c] = B[c-1] (x) A[c]
            float *scanned = sigB;  // where the inclusive prefixes end up
            if constexpr (Sh::SZ <= 64 && WAVE_SLOTS) {
                // Scan in log2(C) rounds with the left factor in registers: in the round with stride st the lanes
                // of chunk c multiply their value by the row of chunk c + st and leave the product as that chunk's
                // new row; then every chunk reads its own new row back.  Rows alternate between the two buffers.
                // B[C-1] is nobody's carry and is not computed.
                float *cur = sigA, *nxt = sigB;
                for (int st = 1; st < C - 1; st <<= 1) {
                    if (active) {
                        if (c < st) store_state<d, N, P>(nxt + mygc * D, u, ln);  // already the full prefix
                        if (c + st < C - 1) {
                            reg_product<d, N, P, SIG_TREE_BATCH>(ln, cur + (mygc + st) * D, u);
                            store_state<d, N, P>(nxt + (mygc + st) * D, u, ln);
                        }
                    }
                    __syncthreads();
                    if (active && c < C - 1) load_state<d, N, P>(nxt + mygc * D, u, ln);
                    float *t = cur; cur = nxt; nxt = t;
                }
                scanned = cur;
            } else {
                for (int x = tid; x < G * D; x += nthr) {
                    const int g2 = x / D;
                    const int pos = x - g2 * D;
                    sigB[(g2 * C) * D + pos] = sigA[(g2 * C) * D + pos];
                }
                __syncthreads();
                for (int c2 = 1; c2 < C; ++c2) {
                    const int total = G * RP::ITEMS;
                    for (int x = tid; x < total; x += nthr) {
                        const int g2 = x / RP::ITEMS;
                        const int it = x - g2 * RP::ITEMS;
                        const int rowi = g2 * C + c2;
                        RP::item(sigB + (rowi - 1) * D, sigA + rowi * D, sigB + rowi * D, it);
                    }
                    __syncthreads();
                }
            }
            // every chunk restarts from the signature of everything before it and emits its prefixes
            if (c == 0) identity_state<d, N, P>(ln);
            else load_state<d, N, P>(scanned + (mygc - 1) * D, u, ln);
            fold_chunk(std::true_type{});
        }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Fold with the prefix part of the Horner chains shared by the workgroup (final signature, one time chunk per
// (path, segment), shapes whose Q = d^P lanes per path exceed a workgroup; P >= 2).
//
// In the kernel above every lane carries the coefficients of the proper prefixes of its word u (levels 1 .. P-1)
// and re-evaluates, for each target level n = P .. N, the chain g_m = S[u_{1:m}] + g_{m-1} v[u_m] / (n - m + 1)
// up to m = P: for d = 10, depth 6, P = 4 that is 46 of a step's 170 vector instructions, repeated by all
// 10^4 lanes of a path although the chain up to m = P-1 depends on the first P-1 letters only.  Here the lanes of
// a workgroup own consecutive words u, so they share about (threads / d) + 1 prefixes q = u / d of length P-1.
// Before a tile of increments is consumed, the workgroup builds
//     table[step][q][n - P] = g_{P-1}^{(n)}(q) / (n - P + 1)
// in LDS (see the kernel for how).  A lane of the fold then needs per step one multiply-add per target level,
//     g_P^{(n)}(u) = S_P[u] + table[step][u / d][n - P] * v[u_P],
// before it descends into its own sub-tree; it keeps no prefix coefficients at all (127 vector instructions per
// step instead of 170 for d = 10, depth 6).
template <int d, int N, int P>
struct SharedChain {
    using Sh = Shape<d, N, P>;
    static constexpr int R = Sh::R;
    static constexpr int E = N - P + 1;                       // target levels P .. N: floats per (step, prefix) of the table
    // prefixes q = u / d that the words of one workgroup can have
    static __host__ __device__ constexpr int nq(int threads) { return (threads - 1) / d + 2; }
    // LDS of one tile: shared_chain_lds_floats (the kernel lays its arrays out in that order)

    // sub-levels r >= 2 below the child `a` of u (local index idx in sub-level r - 1), target sub-level tgt
    template <int tgt, int r>
    static __device__ __forceinline__ void deeper(float (&s)[Sh::SZ], const float (&v)[d], float g, int idx)
    {
#pragma unroll
        for (int a = 0; a < d; ++a) {
            const int child = idx * d + a;
            if constexpr (r == tgt) {
                s[Sh::sub_off(tgt) + child] = fmaf(g, v[a], s[Sh::sub_off(tgt) + child]);
            } else {
                const float g2 = fmaf(g, v[a] * (1.0f / (float)(tgt - r + 1)), s[Sh::sub_off(r) + child]);
                deeper<tgt, r + 1>(s, v, g2, child);
            }
        }
    }

    // One step S <- S (x) exp(v) on the sub-tree below u, given the chain values G at u's parent from the table and
    // duP = v[u_P] (Eq. 3 with Eqs. 2 and 4 in Horner form; deeper levels first, they read the old upper ones).
    static __device__ __forceinline__ void step(float (&s)[Sh::SZ], const float (&v)[d], const float (&G)[E], float duP)
    {
        // chain values at u for the target levels P + 1 .. N, then S[u] itself
        float gu[E];
#pragma unroll
        for (int e = 1; e < E; ++e) gu[e] = fmaf(G[e], duP, s[0]);
        s[0] = fmaf(G[0], duP, s[0]);
        // per child a of u: the chain values below it for the target sub-levels 2 .. R (from the old S[u a]), S[u a]
        // itself, then everything below it, deepest target first (one child at a time keeps few chain values live)
#pragma unroll
        for (int a = 0; a < d; ++a) {
            float g2[R > 1 ? R - 1 : 1];
#pragma unroll
            for (int tg = 2; tg <= R; ++tg) g2[tg - 2] = fmaf(gu[tg] * (1.0f / (float)tg), v[a], s[Sh::sub_off(1) + a]);
            s[Sh::sub_off(1) + a] = fmaf(gu[1], v[a], s[Sh::sub_off(1) + a]);
            static_for<2, R + 1>([&](auto tc) __attribute__((always_inline)) {
                constexpr int tg = R + 2 - decltype(tc)::value;   // R .. 2
                deeper<tg, 2>(s, v, g2[tg - 2], a);
            });
        }
    }
};

// wavefronts per SIMD the kernel is built for: what the lane state and about 45 more registers allow, and no more
// than four when the table's build holds three levels of 16 steps in registers (five spilled ten registers of it)
template <int d, int N, int P>
constexpr int shared_chain_min_waves()
{
    constexpr int sz = Shape<d, N, P>::SZ;
    constexpr int by_state = sz <= 60 ? 5 : sz <= 84 ? 4 : sz <= 124 ? 3 : 2;
    return P >= 4 && by_state > 4 ? 4 : by_state;
}

constexpr int kSharedChainChunk = 16;   // steps of the table one thread builds (held in registers)

template <int d, int N, int P>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(shared_chain_min_waves<d, N, P>())))
void sig_shared_chain_kernel(OnChipArgs A)
{
    static_assert(P >= 2, "needs at least one prefix level to share");
    using Sh = Shape<d, N, P>;
    using SC = SharedChain<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr int E = SC::E;
    constexpr int QP = cpow(d, P - 1);      // prefixes of length P-1 per path
    constexpr int CL = kSharedChainChunk;

    SIG_PRIO_MEMORY();
    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int64_t K = A.L - 1;
    const int W = A.segments, T = A.chunk_steps;
    const unsigned NB = (Q + nthr - 1) / nthr;
    const unsigned group = blockIdx.x / NB;              // (path, segment)
    const unsigned u0 = (blockIdx.x % NB) * (unsigned)nthr;   // first word of this workgroup
    const bool active = u0 + tid < (unsigned)Q;
    const unsigned u = active ? u0 + tid : 0;            // the word of length P this lane works below
    const unsigned b = group / (unsigned)W;
    const int64_t k0 = (int64_t)(group - b * W) * T;
    int64_t left = K - k0;
    if (left > T) left = T;
    const int steps = left > 0 ? (int)left : 0;          // increments of this segment: one tile (checked on the host)
    const float *x0 = A.path + ((int64_t)b * A.L + k0) * d;

    // prefixes q = u / d of this workgroup's words
    unsigned u_last = u0 + nthr - 1;
    if (u_last > (unsigned)Q - 1) u_last = Q - 1;
    const unsigned q0 = u0 / d;
    const int nq = (int)(u_last / d - q0) + 1;           // <= SC::nq(nthr)
    const int NQ = SC::nq(nthr);
    // wavefronts without a word (the tail of a path's last workgroup) only keep the barriers company
    const bool wave_active = (u0 + (unsigned)(tid & ~(kWave - 1))) < (unsigned)Q;

    float *inc = sig_onchip_smem;                        // [T][d]
    float *table = inc + round4(T * d);                  // [T][NQ][E]
    float *ctot = table + round4(T * NQ * E);            // [P-1][chunks][NQ]: chunk totals, at most one float per thread and level
    float *total = ctot + (P - 1) * round4(nthr);        // [P-1][NQ]: S[q_{1:m}] at the end of the segment

    for (int i = tid; i < steps * d; i += nthr) inc[i] = x0[i + d] - x0[i];

    // ---- the table.  Thread -> (prefix bq, chunk bc of CL consecutive steps); the prefixes take a power of two of slots.
    // Level by level (Eq. 3 restricted to the words q_{1:m}, summed over time): the term of step t at level m is
    // h_{m-1}(t) v_t[q_m], with h the Horner chain over the lower levels before step t.  A thread holds its chunk's
    // increments and running sums in registers, leaves its chunk's total per level in LDS, and after a barrier adds up
    // the totals of the chunks before it.  This happens before the fold's lane state exists, so the registers are free.
    int qslots = 1;
    while (qslots < NQ) qslots <<= 1;
    const int nchk = nthr / qslots;                      // >= 1 and nchk * CL >= steps (checked on the host)
    const int bq = tid & (qslots - 1), bc = tid / qslots;
    const bool builder = bq < nq && bc < nchk;
    const int cl = (steps + nchk - 1) / nchk;            // steps per chunk, <= CL
    const int t_begin = bc * cl < steps ? bc * cl : steps;
    const int cnt = builder ? (t_begin + cl < steps ? cl : steps - t_begin) : 0;
    __syncthreads();
    {
        int blet[P - 1];                                 // the letters of this thread's prefix
        unsigned rest = q0 + (builder ? bq : 0);
#pragma unroll
        for (int m = P - 2; m >= 0; --m) { blet[m] = (int)(rest % d); rest /= d; }
        float dv[CL][P - 1];                             // v_t[q_m] of the chunk's steps
        float loc[P - 1][CL];                            // the chunk's own running sums before each of its steps
        float cc[P - 1];                                 // totals of the chunks before this one
#pragma unroll
        for (int i = 0; i < CL; ++i) {
            const float *row = inc + (t_begin + (i < cnt ? i : 0)) * d;
#pragma unroll
            for (int m = 0; m < P - 1; ++m) dv[i][m] = row[blet[m]];
        }
        static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value;
            float run = 0.0f;
#pragma unroll
            for (int i = 0; i < CL; ++i) {
                if (i < cnt) {
                    float hh = 1.0f;
#pragma unroll
                    for (int mm = 1; mm <= m - 1; ++mm) hh = fmaf(hh, dv[i][mm - 1] * (1.0f / (float)(m - mm + 1)), loc[mm - 1][i] + cc[mm - 1]);
                    loc[m - 1][i] = run;
                    run = fmaf(hh, dv[i][m - 1], run);
                }
            }
            float *lvl = ctot + (m - 1) * round4(nthr);
            if (builder) lvl[bc * NQ + bq] = run;
            __syncthreads();
            float sum = 0.0f;
            if (builder) {
                for (int c2 = 0; c2 < bc; ++c2) sum += lvl[c2 * NQ + bq];
                if (bc == nchk - 1) total[(m - 1) * NQ + bq] = sum + run;
            }
            cc[m - 1] = sum;
        });
        // from S[q_{1:m}] before step t to the chain values the fold needs: g_{P-1}^{(n)}(q) / (n - P + 1), n = P .. N
#pragma unroll
        for (int i = 0; i < CL; ++i) {
            if (i < cnt) {
                float *cell = table + ((t_begin + i) * NQ + bq) * E;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    float gg = 1.0f;
#pragma unroll
                    for (int mm = 1; mm <= P - 1; ++mm) gg = fmaf(gg, dv[i][mm - 1] * (1.0f / (float)(P + e - mm + 1)), loc[mm - 1][i] + cc[mm - 1]);
                    cell[e] = gg * (1.0f / (float)(e + 1));
                }
            }
        }
    }
    __syncthreads();

    // ---- the fold: the sub-tree below u
    SIG_PRIO_COMPUTE();
    const int myql = (int)(u / d - q0);
    const int letterP = (int)(u % d);
    float st[Sh::SZ];
#pragma unroll
    for (int i = 0; i < Sh::SZ; ++i) st[i] = 0.0f;
    if (wave_active) {
        // operands of a step: the increment (all lanes of a wavefront read the same row: a broadcast), its component at
        // u's last letter and the table's entries for u's parent
        const float *row = inc;
        const float *tab = table + myql * E;
        for (int t = 0; t < steps; ++t, row += d, tab += NQ * E) {
            float v[d], G[E];
#pragma unroll
            for (int a = 0; a < d; ++a) v[a] = row[a];
            const float duP = row[letterP];
#pragma unroll
            for (int e = 0; e < E; ++e) G[e] = tab[e];
            SC::step(st, v, G, duP);
        }
    }

    // ---- results: the lanes' sub-trees, and the prefix words from the threads that hold their totals
    SIG_PRIO_MEMORY();
    float *dst = (W == 1) ? A.out + (int64_t)b * D : A.partial + (int64_t)group * D;
    if (active) {
        static_for<0, Sh::R + 1>([&](auto rcst) __attribute__((always_inline)) {
            constexpr int r = decltype(rcst)::value;
            constexpr int cnt_r = cpow(d, r);
            store_run<Sh::sub_off(r), cnt_r, Sh::SZ>(dst + Sh::row_off(P + r) + u * cnt_r, st);
        });
    }
    if (tid < nq && q0 + tid < (unsigned)QP) {
        // the word q_{1:m} is written by the workgroup that holds the first word u below it (an empty segment has no
        // totals: its words are zero)
        const unsigned q_s = q0 + tid;
        static_for<1, P>([&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value;
            constexpr unsigned span = cpow(d, P - 1 - m);
            if (q_s % span == 0 && q_s * d >= u0) dst[Sh::row_off(m) + q_s / span] = total[(m - 1) * NQ + tid];
        });
    }
}

template <int d, int N, int P>
constexpr bool shared_chain_compiled() { return P >= 2 && Shape<d, N, P>::Q > 256; }

// ------------------------------------------------------------------------------------------
// Fold kernel for plans with one time chunk per (path, segment): independent wavefronts.
//
// A work item is a batch of `groups` (path, segment) pairs (or, when a chunk's Q lanes exceed the
// workgroup, one workgroup-sized slice of one pair's lanes).  A workgroup walks items blockIdx.x,
// blockIdx.x + gridDim.x, ...  Inside it every wavefront works on its own: it stages the increments of
// the groups its 64 lanes belong to in a private LDS region (groups that straddle two wavefronts are
// staged by both), so there is no workgroup barrier anywhere and wavefronts drift apart in time.  The
// stall of one wavefront on its tile loads is then covered by the arithmetic of the others on the same
// SIMD, and the final stores of an item drain while the next item is folded.  (With workgroup-wide tiles
// all workgroups of a launch load, fold and store in lock-step and the HBM phases are not overlapped.)
template <int d, int N, int P, bool STREAM>
struct FoldGeom {
    using Sh = Shape<d, N, P>;
    static constexpr bool WAVE_SLOTS = STREAM && Sh::Q <= kWave;
    static constexpr int SPW = WAVE_SLOTS ? kWave / Sh::Q : 1;
    // groups a wavefront can touch: all of them aligned (stream), one (Q >= workgroup) or straddling
    static constexpr int NGW = WAVE_SLOTS ? SPW : (Sh::Q >= kWave ? 2 : (kWave + Sh::Q - 2) / Sh::Q + 1);
};

template <int d, int N, int P, bool STREAM>
__global__ __launch_bounds__(256) void sig_fold_kernel(OnChipArgs A)
{
    using Sh = Shape<d, N, P>;
    using Geo = FoldGeom<d, N, P, STREAM>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    constexpr bool WAVE_SLOTS = Geo::WAVE_SLOTS;
    constexpr int SPW = Geo::SPW;
    constexpr int NGW = Geo::NGW;

    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int wave = tid / kWave, lw = tid - wave * kWave;
    const int64_t K = A.L - 1;
    const int W = A.segments, T = A.chunk_steps, TT = A.tile_steps;
    const unsigned ngroups = (unsigned)(A.B * W);
    const bool big = Q > nthr;
    const unsigned NB = big ? (Q + nthr - 1) / nthr : 1;
    const int G = big ? 1 : A.groups;  // groups (slots) per item
    const unsigned nitems = big ? ngroups * NB : (ngroups + G - 1) / G;

    // ---- lane -> (slot in the item, prefix word); fixed, except the prefix word in `big` mode
    int gi;
    unsigned u = 0;
    bool lane_ok;
    int g_lo, ng;  // slots this wavefront stages: g_lo .. g_lo + ng - 1
    if constexpr (WAVE_SLOTS) {
        const int sw = lw / Q;
        gi = wave * SPW + sw;
        u = (unsigned)(lw - sw * Q);
        lane_ok = sw < SPW && gi < G;
        g_lo = wave * SPW;
        ng = G - g_lo < SPW ? G - g_lo : SPW;
    } else if (!big) {
        gi = tid / Q;
        u = (unsigned)(tid - gi * Q);
        lane_ok = gi < G;
        g_lo = (wave * kWave) / Q;
        int g_hi = (wave * kWave + kWave - 1) / Q;
        if (g_hi > G - 1) g_hi = G - 1;
        ng = g_hi - g_lo + 1;
    } else {
        gi = 0;
        lane_ok = true;
        g_lo = 0;
        ng = 1;
    }
    if (ng < 0) ng = 0;
    if (!lane_ok) gi = g_lo < G ? g_lo : 0;
    const int gl = lane_ok ? gi - g_lo : 0;  // my slot inside the set this wavefront stages
    int letter[P > 0 ? P : 1];
    letter[0] = 0;
    auto set_letters = [&]() {
        unsigned rest = u;
#pragma unroll
        for (int m = P - 1; m >= 0; --m) { letter[m] = (int)(rest % d); rest /= d; }
    };
    set_letters();

    // ---- LDS, private to the wavefront: NGW descriptors, one tile [NGW][TT*d], staged rows (stream)
    const int row_floats = TT * d;
    const int wave_floats = desc_floats(NGW) + round4(NGW * row_floats) + (WAVE_SLOTS ? SPW * D : 0);
    float *wbase = sig_onchip_smem + wave * wave_floats;
    ChunkDesc *desc = reinterpret_cast<ChunkDesc *>(wbase);
    float *tile = wbase + desc_floats(NGW);
    float *rows = tile + round4(NGW * row_floats);  // [SPW][D], WAVE_SLOTS only
    (void)rows;

    const int rshift = A.row_shift;
    const int rmask = (1 << rshift) - 1;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(A.out) & 15) == 0;
    (void)vec_ok;
    Lane<d, N, P> ln;

    for (unsigned item = blockIdx.x; item < nitems; item += gridDim.x) {
        const unsigned group0 = big ? item / NB : item * (unsigned)G;
        if (big) {
            u = (item % NB) * nthr + tid;
            lane_ok = u < (unsigned)Q;
            if (!lane_ok) u = 0;
            set_letters();
        }
        const unsigned grp = group0 + gi;
        const bool active = lane_ok && grp < ngroups;

        // descriptors of the groups this wavefront stages (LDS operations of one wavefront execute in order,
        // so the other lanes may read them right after)
        if (lw < ng) {
            const unsigned g2 = group0 + g_lo + lw;
            ChunkDesc dsc;
            dsc.base = 0;
            dsc.out_row0 = 0;
            dsc.steps = 0;
            dsc.pad[0] = dsc.pad[1] = dsc.pad[2] = 0;
            if (g2 < ngroups) {
                const unsigned b2 = g2 / (unsigned)W;
                const int64_t k0 = (int64_t)(g2 - b2 * W) * T;
                int64_t left = K - k0;
                if (left > T) left = T;
                if (left > 0) {
                    dsc.steps = (int)left;
                    dsc.base = ((int64_t)b2 * A.L + k0) * d;
                    dsc.out_row0 = ((int64_t)b2 * K + k0) * D;
                }
            }
            desc[lw] = dsc;
        }
        __builtin_amdgcn_wave_barrier();
        identity_state<d, N, P>(ln);

        // emission through LDS (stream): per-lane copy descriptors, see the chunked kernel
        constexpr int VEC = (D % 4 == 0) ? 4 : 1;
        constexpr int ROWV = D / VEC;
        constexpr int NIT = (SPW * ROWV + kWave - 1) / kWave;
        constexpr bool FAST_EMIT = WAVE_SLOTS && NIT <= 8;
        using V = std::conditional_t<VEC == 4, vec4f, float>;
        V *eptr[FAST_EMIT ? NIT : 1];
        int eoff[FAST_EMIT ? NIT : 1];
        int elim[FAST_EMIT ? NIT : 1];
        const bool use_vec = VEC == 1 || vec_ok;
        if constexpr (FAST_EMIT) {
            static_for<0, NIT>([&](auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                const int i = lw + j * kWave;
                const int sw = i / ROWV;
                const int col = i - sw * ROWV;
                eptr[j] = reinterpret_cast<V *>(A.out);
                eoff[j] = 0;
                elim[j] = 0;
                if (use_vec && i < SPW * ROWV && sw < ng) {
                    eptr[j] = reinterpret_cast<V *>(A.out + desc[sw].out_row0) + col;
                    eoff[j] = sw * ROWV + col;
                    elim[j] = desc[sw].steps;
                }
            });
        }
        int64_t my_out_row0 = 0;
        int my_steps = 0;
        if (STREAM && !WAVE_SLOTS && active) {
            my_out_row0 = desc[gl].out_row0;
            my_steps = desc[gl].steps;
        }

        for (int t0 = 0; t0 < T; t0 += TT) {
            // ---- stage this wavefront's tile: consecutive lanes on consecutive floats of a group's stretch
            // (eight elements per lane and trip, so that their global loads are in flight together)
            const int flat = ng << rshift;
            for (int base = 0; base < flat; base += 8 * kWave) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int idx = base + e * kWave + lw;
                    const int g = idx >> rshift;
                    const int r = idx & rmask;
                    v[e] = 0.0f;
                    if (idx < flat && r < (desc[g].steps - t0) * d && r < row_floats) {
                        const float *x = A.path + desc[g].base + (int64_t)t0 * d + r;
                        v[e] = x[d] - x[0];
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int idx = base + e * kWave + lw;
                    const int g = idx >> rshift;
                    const int r = idx & rmask;
                    if (idx < flat && r < row_floats) tile[g * row_floats + r] = v[e];
                }
            }
            __builtin_amdgcn_wave_barrier();
            // ---- consume it
            const int steps = (T - t0 < TT) ? T - t0 : TT;
            const float *row = tile + gl * row_floats;
            Inc<d, P> inc;
            for (int t = 0; t < steps; ++t, row += d) {
                load_inc<d, P>(inc, row, letter);
                fused_step<d, N, P>(ln, inc);
                if constexpr (WAVE_SLOTS) {
                    if (active) store_state<d, N, P>(rows + gl * D, u, ln);
                    if (FAST_EMIT && use_vec) {
                        if constexpr (FAST_EMIT) {
                            V val[NIT];
                            static_for<0, NIT>([&](auto jc) __attribute__((always_inline)) {
                                constexpr int j = decltype(jc)::value;
                                val[j] = reinterpret_cast<const V *>(rows)[eoff[j]];
                            });
                            static_for<0, NIT>([&](auto jc) __attribute__((always_inline)) {
                                constexpr int j = decltype(jc)::value;
                                if (t0 + t < elim[j]) eptr[j][(int64_t)(t0 + t) * ROWV] = val[j];
                            });
                        }
                    } else {
                        for (int i = lw; i < SPW * D; i += kWave) {
                            const int sw = i / D;
                            const int col = i - sw * D;
                            if (sw < ng && t0 + t < desc[sw].steps)
                                A.out[desc[sw].out_row0 + (int64_t)(t0 + t) * D + col] = rows[sw * D + col];
                        }
                    }
                } else if constexpr (STREAM) {
                    if (active && t0 + t < my_steps)
                        store_state<d, N, P>(A.out + my_out_row0 + (int64_t)(t0 + t) * D, u, ln);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (!STREAM && active) {
            float *dst = (W == 1) ? A.out + (int64_t)grp * D : A.partial + (int64_t)grp * D;
            store_state<d, N, P>(dst, u, ln);
        }
    }
}

// LDS bytes of the fold kernel (same layout as in the kernel)
template <int d, int N, int P>
int64_t fold_lds_bytes(const OnChipArgs &A)
{
    using Sh = Shape<d, N, P>;
    const int waves = A.threads / kWave;
    int64_t per_wave;
    if (A.stream_flag) {
        using Geo = FoldGeom<d, N, P, true>;
        per_wave = desc_floats(Geo::NGW) + round4(Geo::NGW * A.tile_steps * d) + (Geo::WAVE_SLOTS ? Geo::SPW * Sh::D : 0);
    } else {
        using Geo = FoldGeom<d, N, P, false>;
        per_wave = desc_floats(Geo::NGW) + round4(Geo::NGW * A.tile_steps * d);
    }
    return per_wave * waves * (int64_t)sizeof(float);
}

// LDS bytes of a launch (same layout as in the kernel)
template <int d, int N, int P>
int64_t on_chip_lds_bytes(const OnChipArgs &A)
{
    using Sh = Shape<d, N, P>;
    if constexpr (shared_chain_compiled<d, N, P>()) {
        if (A.shared_chain) return shared_chain_lds_floats(d, N, P, A.threads, A.chunk_steps) * (int64_t)sizeof(float);
    }
    if (A.chunks == 1 && !A.cooperative) return fold_lds_bytes<d, N, P>(A);
    const int64_t NGC = (int64_t)A.groups * A.chunks;
    const bool pipe = A.pipe != 0;
    int64_t floats = desc_floats((int)NGC) + (pipe ? 2 : 1) * (int64_t)round4((int)(NGC * A.tile_steps * d));
    if (A.flat_tile) floats = desc_floats((int)NGC) + round4((int)(A.groups * A.L * d) + 3);
    if (A.chunks > 1 && !A.stream_flag && Sh::SZ <= 64) {
        // register tree: (chunks + 1) / 2 rows per group, in the place of the tiles
        const int64_t rows = (int64_t)A.groups * ((A.chunks + 1) / 2) * Sh::D;
        const int64_t tiles = floats - desc_floats((int)NGC);
        if (rows > tiles) floats += rows - tiles;
    } else if (A.chunks > 1) {
        floats += NGC * Sh::D;
        // second buffer: the scan's prefixes (stream) or the ping-pong half of the LDS tree (final, large state)
        if (A.stream_flag) floats += NGC * Sh::D;
        else floats += (int64_t)A.groups * ((A.chunks + 1) / 2) * Sh::D;
    } else if (A.stream_flag && Sh::Q <= kWave) {
        floats += NGC * Sh::D;  // rows staged for emission
    }
    return floats * (int64_t)sizeof(float);
}

template <int d, int N, int P, bool CHUNKED, bool STREAM>
void on_chip_launch_pipe(const OnChipArgs &A, dim3 g, dim3 blk, size_t lds, hipStream_t st)
{
    if (A.pipe) {
        hipLaunchKernelGGL((sig_on_chip_kernel<d, N, P, CHUNKED, STREAM, true>), g, blk, lds, st, A);
        return;
    }
    if constexpr (!CHUNKED) {
        if (A.flat_tile) {
            hipLaunchKernelGGL((sig_on_chip_kernel<d, N, P, false, STREAM, false, true>), g, blk, lds, st, A);
            return;
        }
    }
    hipLaunchKernelGGL((sig_on_chip_kernel<d, N, P, CHUNKED, STREAM, false>), g, blk, lds, st, A);
}

template <int d, int N, int P>
hipError_t on_chip_launch(const OnChipArgs &A, hipStream_t st)
{
    using Sh = Shape<d, N, P>;
    const int64_t ngroups = A.B * A.segments;
    if (Sh::Q <= A.threads) {
        if (A.groups < 1) return hipErrorInvalidValue;
        if (A.stream_flag && Sh::Q <= kWave) {
            if ((int64_t)A.groups * A.chunks > (int64_t)(A.threads / kWave) * (kWave / Sh::Q)) return hipErrorInvalidValue;
        } else if ((int64_t)A.groups * A.chunks * Sh::Q > A.threads) {
            return hipErrorInvalidValue;
        }
    }
    const int64_t grid = on_chip_workgroups(Sh::Q, A);
    if (grid <= 0 || on_chip_work_items(Sh::Q, A) > INT32_MAX || ngroups > INT32_MAX) return hipErrorInvalidValue;
    if (A.threads > (A.chunks > 1 ? max_threads<d, N, P, true>() : 256)) return hipErrorInvalidValue;
    // loader geometry the kernel relies on
    const int64_t NGC = (int64_t)A.groups * A.chunks;
    if (A.row_shift < 0 || A.row_shift > 20 || (1 << A.row_shift) < A.tile_steps * d) return hipErrorInvalidValue;
    if ((A.chunks > 1 || A.cooperative) && A.pipe && (NGC << A.row_shift) > (int64_t)kStage * A.threads)
        return hipErrorInvalidValue;
    const int64_t lds = on_chip_lds_bytes<d, N, P>(A);
    if (lds > kMaxLdsBytes) return hipErrorInvalidValue;
    const dim3 blk(A.threads);
    if (A.shared_chain) {
        if constexpr (shared_chain_compiled<d, N, P>()) {
            if (A.stream_flag || A.chunks != 1 || Sh::Q <= A.threads || A.tile_steps != A.chunk_steps ||
                !shared_chain_fits(d, N, P, A.threads, A.chunk_steps)) return hipErrorInvalidValue;
            hipLaunchKernelGGL((sig_shared_chain_kernel<d, N, P>), dim3((unsigned)grid), blk, (size_t)lds, st, A);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (A.chunks > 1) {
        const dim3 g((unsigned)grid);
        if (A.stream_flag) on_chip_launch_pipe<d, N, P, true, true>(A, g, blk, (size_t)lds, st);
        else on_chip_launch_pipe<d, N, P, true, false>(A, g, blk, (size_t)lds, st);
    } else if (A.cooperative) {
        const dim3 g((unsigned)grid);
        if (A.stream_flag) on_chip_launch_pipe<d, N, P, false, true>(A, g, blk, (size_t)lds, st);
        else on_chip_launch_pipe<d, N, P, false, false>(A, g, blk, (size_t)lds, st);
    } else {
        // persistent: no more workgroups than stay resident, each walking the same number of work items
        const dim3 g((unsigned)grid);
        if (A.stream_flag) hipLaunchKernelGGL((sig_fold_kernel<d, N, P, true>), g, blk, (size_t)lds, st, A);
        else hipLaunchKernelGGL((sig_fold_kernel<d, N, P, false>), g, blk, (size_t)lds, st, A);
    }
    return hipGetLastError();
}

// Join the partial signatures of the W time segments of each path: out[b] = partial[b][0] (x) ... (x) partial[b][W-1].
// One workgroup handles G paths: all their partial rows are read into LDS in one go, then reduced by the tree.
template <int d, int N>
__global__ __launch_bounds__(256) void sig_join_kernel(const float *partial, float *out, int B, int W, int G)
{
    constexpr int D = Shape<d, N, 0>::D;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int b0 = blockIdx.x * G;
    const int nb = (B - b0 < G) ? B - b0 : G;
    float *bufA = sig_onchip_smem;               // [G][W][D]
    float *bufB = bufA + G * W * D;              // [G][(W+1)/2][D]
    const float *srcg = partial + (int64_t)b0 * W * D;
    for (int x = tid; x < nb * W * D; x += nthr) bufA[x] = srcg[x];
    __syncthreads();
    float *src = bufA, *dst = bufB;
    int src_stride = W, dst_stride = (W + 1) / 2;
    lds_tree_reduce<d, N>(src, dst, G, W, src_stride, dst_stride, tid, nthr);
    for (int x = tid; x < nb * D; x += nthr) {
        const int g2 = x / D;
        const int pos = x - g2 * D;
        out[(int64_t)(b0 + g2) * D + pos] = src[(g2 * src_stride) * D + pos];
    }
}

template <int d, int N>
hipError_t on_chip_join(const float *partial, float *out, int64_t B, int W, hipStream_t st)
{
    constexpr int D = Shape<d, N, 0>::D;
    if (B <= 0 || B > INT32_MAX || W < 2) return hipErrorInvalidValue;
    const int64_t per_path = (int64_t)(W + (W + 1) / 2) * D * (int64_t)sizeof(float);
    int64_t G = kMaxLdsBytes / 2 / per_path;  // half of the LDS limit keeps two workgroups on a CU
    if (G < 1) G = kMaxLdsBytes / per_path;
    if (G < 1) return hipErrorInvalidValue;
    if (G > 8) G = 8;
    if (G > B) G = B;
    const int64_t grid = (B + G - 1) / G;
    hipLaunchKernelGGL((sig_join_kernel<d, N>), dim3((unsigned)grid), dim3(256), (size_t)(G * per_path), st, partial, out,
                       (int)B, W, (int)G);
    return hipGetLastError();
}

// Join with the running product in registers (lane state small enough).  One workgroup per path: all of its
// W partial rows are copied to LDS in one go (every thread helps, loads batched), then the Q lanes that own the
// sub-trees multiply them left to right; no barrier is needed between the products.
template <int d, int N, int P>
__global__ __launch_bounds__(256) void sig_join_reg_kernel(const float *partial, float *out, int W)
{
    using Sh = Shape<d, N, P>;
    constexpr int Q = Sh::Q;
    constexpr int D = Sh::D;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t b = blockIdx.x;
    float *rows = sig_onchip_smem;  // [W][D]
    const float *src = partial + b * W * D;
    const int total = W * D;
    for (int base = 0; base < total; base += 8 * nthr) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int x = base + e * nthr + tid;
            v[e] = x < total ? src[x] : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int x = base + e * nthr + tid;
            if (x < total) rows[x] = v[e];
        }
    }
    __syncthreads();
    if (tid < Q) {
        const unsigned u = (unsigned)tid;
        Lane<d, N, P> ln;
        load_state<d, N, P>(rows, u, ln);
        for (int w = 1; w < W; ++w) reg_product<d, N, P, true>(ln, rows + w * D, u);
        store_state<d, N, P>(out + b * D, u, ln);
    }
}

template <int d, int N, int P>
hipError_t on_chip_join_reg(const float *partial, float *out, int64_t B, int W, hipStream_t st)
{
    using Sh = Shape<d, N, P>;
    if (B <= 0 || B > INT32_MAX || W < 2 || Sh::Q > 256) return hipErrorInvalidValue;
    const int64_t lds = (int64_t)W * Sh::D * (int64_t)sizeof(float);
    if (lds > kMaxLdsBytes) return hipErrorInvalidValue;
    hipLaunchKernelGGL((sig_join_reg_kernel<d, N, P>), dim3((unsigned)B), dim3(256), (size_t)lds, st, partial, out, W);
    return hipGetLastError();
}

// the join a table entry uses: in registers when the lane state is small, else the LDS tree
template <int d, int N, int P>
hipError_t on_chip_join_any(const float *partial, float *out, int64_t B, int W, hipStream_t st)
{
    if constexpr (Shape<d, N, P>::SZ <= 64 && Shape<d, N, P>::Q <= 256) return on_chip_join_reg<d, N, P>(partial, out, B, W, st);
    else return on_chip_join<d, N>(partial, out, B, W, st);
}

#define SIG_ON_CHIP_ENTRY(d, N, P)                                                              \
    {                                                                                           \
        d, N, P, ::sig::onchip::Shape<d, N, P>::Q, ::sig::onchip::Shape<d, N, P>::SZ,           \
            d, &::sig::onchip::on_chip_launch<d, N, P>,         \
            &::sig::onchip::on_chip_lds_bytes<d, N, P>, &::sig::onchip::on_chip_join_any<d, N, P> \
    }

}  // namespace onchip
}  // namespace sig
#endif

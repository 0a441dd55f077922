// Gradient of the signature with respect to the path for ANY (d, depth): the fallback of sig_backward for shapes
// without a compiled register kernel, and for paths too long for those kernels' LDS staging.
//
// Same reverse sweep as sig_backward.hip (the derivative of the paper's Eqs. 2-5, needed because the layer is
// trained between other layers, Section 4.2, Eq. 11), but with run-time d and depth, so nothing lives in
// registers: one workgroup per path keeps the prefix signature S, its adjoint A = d(loss)/dS and the Horner
// chain values in LDS when they fit and in device scratch otherwise, and sweeps every level with one thread per
// coefficient.  Per increment k = K-1 .. 0, with v = dX_k:
//   1. (stream mode) A += upstream gradient of row k;
//   2. S <- S (x) exp(-v): the fused Horner step with the negated increment, levels depth .. 1 in place
//      (g_0 = 1, g_m[w a] = S_m[w a] + g_{m-1}[w] (-v[a]) / (n-m+1), S_n[w a] += g_{n-1}[w] (-v[a])); k = 0: S = 1;
//   3. the transpose of the forward step S_{k-1} -> S_k, target levels n = 1 .. depth in this order so that A can
//      be updated in place.  Chain values G_m = g_{n,m} of all levels m < n are kept; then, with gb the adjoint of g,
//        gb_{n-1}[w] = sum_a A_n[w a] v[a],                      dv[a] += sum_w A_n[w a] G_{n-1}[w],
//        for m = n-1 .. 1:  A_m[w a] += gb_m[w a],               dv[a] += sum_w gb_m[w a] G_{m-1}[w] / (n-m+1),
//                           gb_{m-1}[w] = sum_a gb_m[w a] v[a] / (n-m+1).
// Sums over the children of a word are taken by one thread per parent; sums over all words of a level (the dv
// terms) by threads that each stay on one letter (the thread stride is a multiple of d) and a final ordered sum
// over the threads of a letter: deterministic.  d(loss)/dv of every step goes to device scratch and the
// workgroup forms d(loss)/dX_j = d/d(dX_{j-1}) - d/d(dX_j) at the end.
#include "sig_internal.h"

namespace sig {

namespace {

constexpr int kGenThreads = 256;
constexpr int kGenLdsFloats = 12288;   // S, A and the chain buffers of one path stay in LDS up to this many floats

struct GeneralBackwardArgs {
    const float *path;      // [B][L][d]
    const float *sig;       // [B][D] or [B][K][D]
    const float *grad_out;  // same shape as sig
    float *grad_path;       // [B][L][d]
    float *work;            // per path: [K][d] sums over the increments, then (unless in LDS) S, A, G, two gb buffers
    int64_t work_stride;    // floats of `work` per path
    int64_t B, L, D;
    int32_t d, depth, stream_flag, in_lds;
    int64_t pw[kMaxDepth + 1];   // d^n
    int64_t off[kMaxDepth + 2];  // start of level n (n >= 1) in a row
    int64_t goff[kMaxDepth + 1]; // start of chain level m in G: 1 + d + ... + d^{m-1}
    int64_t chain_floats;        // 1 + d + ... + d^{depth-1}
};

extern __shared__ float gen_smem[];

__global__ __launch_bounds__(kGenThreads) void sig_backward_general_kernel(GeneralBackwardArgs P)
{
    const int d = P.d, N = P.depth;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t b = blockIdx.x;
    const int64_t K = P.L - 1, D = P.D;
    const float *X = P.path + b * P.L * d;
    float *gdx = P.work + b * P.work_stride;   // [K][d]

    // LDS: v[d], per-thread partial sums [nthr], then (if they fit) the per-path arrays
    float *vs = gen_smem;
    float *part = vs + (d + 3) / 4 * 4;
    float *arrays = P.in_lds ? part + nthr : gdx + K * d;
    float *S = arrays;                    // levels 1 .. N at off[n]
    float *A = S + D;
    float *G = A + D;                     // chain values of levels 0 .. N-1 at goff[m]
    float *cur = G + P.chain_floats;      // two buffers of d^{N-1} floats: chain of step 2, gb of step 3
    float *nxt = cur + P.pw[N - 1];

    // a thread that walks the words of a level with this stride keeps its letter and advances its parent evenly
    const int stride = nthr / d * d;
    const int pstride = stride / d;
    const bool walker = tid < stride;
    const int my_letter = tid % d;
    const int my_parent = tid / d;

    {
        const float *srow = P.stream_flag ? P.sig + (b * K + (K - 1)) * D : P.sig + b * D;
        for (int64_t i = tid; i < D; i += nthr) {
            S[i] = srow[i];
            A[i] = P.stream_flag ? 0.0f : P.grad_out[b * D + i];
        }
    }
    __syncthreads();

    for (int64_t k = K - 1; k >= 0; --k) {
        if (tid < d) vs[tid] = X[(k + 1) * d + tid] - X[k * d + tid];
        if (P.stream_flag) {
            const float *up = P.grad_out + (b * K + k) * D;
            for (int64_t i = tid; i < D; i += nthr) A[i] += up[i];
        }
        __syncthreads();
        const float v_mine = vs[my_letter];

        // 2. undo the increment
        if (k == 0) {
            for (int64_t i = tid; i < D; i += nthr) S[i] = 0.0f;
            __syncthreads();
        } else {
            for (int n = N; n >= 1; --n) {
                if (tid == 0) cur[0] = 1.0f;
                __syncthreads();
                for (int m = 1; m < n; ++m) {
                    const float scale = -v_mine / (float)(n - m + 1);
                    if (walker) {
                        int64_t par = my_parent;
                        for (int64_t c = tid; c < P.pw[m]; c += stride, par += pstride)
                            nxt[c] = fmaf(cur[par], scale, S[P.off[m] + c]);
                    }
                    __syncthreads();
                    float *t = cur; cur = nxt; nxt = t;
                }
                if (walker) {
                    int64_t par = my_parent;
                    for (int64_t c = tid; c < P.pw[n]; c += stride, par += pstride)
                        S[P.off[n] + c] = fmaf(cur[par], -v_mine, S[P.off[n] + c]);
                }
                __syncthreads();
            }
        }

        // 3. transposed step
        float acc = 0.0f;   // this thread's share of d(loss)/dv[my_letter]
        for (int n = 1; n <= N; ++n) {
            if (tid == 0) G[0] = 1.0f;
            __syncthreads();
            for (int m = 1; m < n; ++m) {
                const float scale = v_mine / (float)(n - m + 1);
                if (walker) {
                    int64_t par = my_parent;
                    for (int64_t c = tid; c < P.pw[m]; c += stride, par += pstride)
                        G[P.goff[m] + c] = fmaf(G[P.goff[m - 1] + par], scale, S[P.off[m] + c]);
                }
                __syncthreads();
            }
            // top of the chain: level n against G_{n-1}
            const float *An = A + P.off[n];
            for (int64_t w = tid; w < P.pw[n - 1]; w += nthr) {
                float s = 0.0f;
                for (int a = 0; a < d; ++a) s = fmaf(An[w * d + a], vs[a], s);
                cur[w] = s;
            }
            if (walker) {
                int64_t par = my_parent;
                const float *Gt = G + P.goff[n - 1];
                for (int64_t c = tid; c < P.pw[n]; c += stride, par += pstride) acc = fmaf(An[c], Gt[par], acc);
            }
            __syncthreads();
            for (int m = n - 1; m >= 1; --m) {   // cur holds gb_m
                const float scale = 1.0f / (float)(n - m + 1);
                if (walker) {
                    int64_t par = my_parent;
                    const float *Gp = G + P.goff[m - 1];
                    float *Am = A + P.off[m];
                    for (int64_t c = tid; c < P.pw[m]; c += stride, par += pstride) {
                        const float gb = cur[c];
                        Am[c] += gb;
                        acc = fmaf(gb * scale, Gp[par], acc);
                    }
                }
                if (m > 1) {
                    for (int64_t w = tid; w < P.pw[m - 1]; w += nthr) {
                        float s = 0.0f;
                        for (int a = 0; a < d; ++a) s = fmaf(cur[w * d + a], vs[a], s);
                        nxt[w] = s * scale;
                    }
                }
                __syncthreads();
                float *t = cur; cur = nxt; nxt = t;
            }
        }

        // d(loss)/dv[a]: the threads of letter a, in order
        part[tid] = walker ? acc : 0.0f;
        __syncthreads();
        if (tid < d) {
            float s = 0.0f;
            for (int j = tid; j < stride; j += d) s += part[j];
            gdx[k * d + tid] = s;
        }
        __syncthreads();
    }

    // d(loss)/dX_j = d/d(dX_{j-1}) - d/d(dX_j)
    const int64_t out_row = P.L * d, row_floats = K * d;
    float *out = P.grad_path + b * out_row;
    for (int64_t r = tid; r < out_row; r += nthr) {
        const float before = r >= d ? gdx[r - d] : 0.0f;
        const float after = r < row_floats ? gdx[r] : 0.0f;
        out[r] = before - after;
    }
}

int64_t per_path_arrays(const RowShape &rs)
{
    int64_t chain = 0;
    for (int m = 0; m < rs.depth; ++m) chain += rs.pow[m];
    return 2 * rs.D + chain + 2 * rs.pow[rs.depth - 1];
}

}  // namespace

bool backward_general_available(int d) { return d >= 1 && d <= kGenThreads; }

int64_t backward_general_scratch_floats(int64_t B, int64_t L, const RowShape &rs)
{
    const int64_t arrays = per_path_arrays(rs);
    const int64_t steps = (L - 1) * rs.d;
    return B * (steps + (arrays <= kGenLdsFloats ? 0 : arrays));
}

hipError_t launch_backward_general(const float *path, const float *sig, const float *grad_out, float *grad_path,
                                   float *scratch, int64_t B, int64_t L, const RowShape &rs, int stream_flag,
                                   hipStream_t st)
{
    if (!backward_general_available(rs.d) || !scratch || B <= 0 || B > INT32_MAX) return hipErrorInvalidValue;
    GeneralBackwardArgs P{};
    P.path = path;
    P.sig = sig;
    P.grad_out = grad_out;
    P.grad_path = grad_path;
    P.work = scratch;
    P.B = B;
    P.L = L;
    P.D = rs.D;
    P.d = rs.d;
    P.depth = rs.depth;
    P.stream_flag = stream_flag;
    const int64_t arrays = per_path_arrays(rs);
    P.in_lds = arrays <= kGenLdsFloats ? 1 : 0;
    P.work_stride = (L - 1) * rs.d + (P.in_lds ? 0 : arrays);
    int64_t g = 0;
    for (int n = 0; n <= rs.depth; ++n) {
        P.pw[n] = rs.pow[n];
        if (n < rs.depth) { P.goff[n] = g; g += rs.pow[n]; }
    }
    P.chain_floats = g;
    for (int n = 1; n <= rs.depth + 1; ++n) P.off[n] = rs.off[n];
    const size_t lds = (size_t)((rs.d + 3) / 4 * 4 + kGenThreads + (P.in_lds ? arrays : 0)) * sizeof(float);
    hipLaunchKernelGGL(sig_backward_general_kernel, dim3((unsigned)B), dim3(kGenThreads), lds, st, P);
    return hipGetLastError();
}

}  // namespace sig

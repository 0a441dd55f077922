// Measurement anchors declared in include/sig_probe.h: a plain copy, write-only kernels and an fp32 FMA loop.
#include "sig_internal.h"
#include "sig_probe.h"

namespace {

// every workgroup copies one contiguous 16 KB piece (four vectors per thread, all four loads in flight together)
__global__ __launch_bounds__(256) void sig_probe_copy_kernel(float4 *dst, const float4 *src, int64_t n4)
{
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    float4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t i = base + j * 256;
        if (i < n4) v[j] = src[i];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t i = base + j * 256;
        if (i < n4) dst[i] = v[j];
    }
}

// every workgroup writes one contiguous 16 KB piece (four vectors per thread, 4 KB apart), pieces in grid order
__global__ __launch_bounds__(256) void sig_probe_fill_kernel(float4 *dst, int64_t n4)
{
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    const float4 one = {1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t i = base + j * 256;
        if (i < n4) dst[i] = one;
    }
}

// one wavefront per region of region4 vectors, written front to back 1 KB at a time
__global__ __launch_bounds__(256) void sig_probe_streams_kernel(float4 *dst, int64_t region4, int64_t streams)
{
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / 64;
    const int lane = threadIdx.x & 63;
    if (wave >= streams) return;
    float4 *base = dst + wave * region4;
    const float4 one = {1.0f, 1.0f, 1.0f, 1.0f};
    for (int64_t i = lane; i < region4; i += 64) base[i] = one;
}

extern __shared__ float sig_probe_smem[];

// ILP independent FMA chains per lane; dynamic LDS is only there to limit how many workgroups share a CU
template <int ILP>
__global__ __launch_bounds__(256) void sig_probe_fma_kernel(float *out, int64_t iters)
{
    const int64_t lane = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    float a[ILP];
#pragma unroll
    for (int i = 0; i < ILP; ++i) a[i] = 1.0f + (float)((lane + i) & 7) * 0.125f;
    const float x = 0.999f, y = 0.001f + (float)(lane & 3) * 1e-6f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 16 / ILP; ++r)
#pragma unroll
            for (int i = 0; i < ILP; ++i) a[i] = fmaf(a[i], x, y);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < ILP; ++i) s += a[i];
    out[lane] = s;
}

// acc[a][b] += g[a] * v[b]: the three-register FMA form of the fused kernels' inner loops
__global__ __launch_bounds__(256) void sig_probe_fma_outer_kernel(float *out, const float *seed, int64_t iters)
{
    const int64_t lane = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    float acc[100], g[10], v[10];
    // operands the compiler cannot fold: they come from memory (the buffer is written before it is read back below)
    const float s0 = seed[lane & 63];
#pragma unroll
    for (int i = 0; i < 100; ++i) acc[i] = s0 + (float)i * 0.001f;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        g[i] = s0 * 0.01f + (float)i * 1e-4f;
        v[i] = s0 * 0.02f - (float)i * 1e-4f;
    }
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 10; ++a)
#pragma unroll
            for (int b = 0; b < 10; ++b) acc[a * 10 + b] = fmaf(g[a], v[b], acc[a * 10 + b]);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 100; ++i) s += acc[i];
    out[lane] = s;
}

}  // namespace

extern "C" {

int sig_probe_copy(float *dst, const float *src, int64_t n_floats, void *hip_stream)
{
    if (!dst || !src || n_floats < 0 || n_floats % 4 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return SIG_ERR_INVALID;
    if (n_floats == 0) return SIG_OK;
    const int64_t n4 = n_floats / 4;
    const int64_t blocks = (n4 + 1023) / 1024;
    if (blocks > INT32_MAX) return SIG_ERR_TOO_LARGE;
    hipLaunchKernelGGL(sig_probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<float4 *>(dst), reinterpret_cast<const float4 *>(src), n4);
    return hipGetLastError() == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int sig_probe_write(float *dst, int64_t n_floats, int64_t streams, void *hip_stream)
{
    if (!dst || n_floats < 0 || streams < 1 || ((uintptr_t)dst & 15) || n_floats % (4 * streams)) return SIG_ERR_INVALID;
    if (n_floats == 0) return SIG_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (streams == 1) {
        const int64_t n4 = n_floats / 4;
        const int64_t blocks = (n4 + 1023) / 1024;
        if (blocks > INT32_MAX) return SIG_ERR_TOO_LARGE;
        hipLaunchKernelGGL(sig_probe_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                           reinterpret_cast<float4 *>(dst), n4);
    } else {
        const int64_t blocks = (streams + 3) / 4;
        if (blocks > INT32_MAX) return SIG_ERR_TOO_LARGE;
        hipLaunchKernelGGL(sig_probe_streams_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                           reinterpret_cast<float4 *>(dst), n_floats / 4 / streams, streams);
    }
    return hipGetLastError() == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int sig_probe_fma(float *out, int64_t waves, int64_t iters, int ilp, int lds_bytes, void *hip_stream)
{
    if (!out || waves < 4 || waves % 4 || iters < 0 || waves / 4 > INT32_MAX) return SIG_ERR_INVALID;
    if (lds_bytes < 0 || lds_bytes > sig::kMaxLdsBytes) return SIG_ERR_INVALID;
    const dim3 grid((unsigned)(waves / 4)), block(256);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    switch (ilp) {
    case 1: hipLaunchKernelGGL(sig_probe_fma_kernel<1>, grid, block, (size_t)lds_bytes, st, out, iters); break;
    case 2: hipLaunchKernelGGL(sig_probe_fma_kernel<2>, grid, block, (size_t)lds_bytes, st, out, iters); break;
    case 4: hipLaunchKernelGGL(sig_probe_fma_kernel<4>, grid, block, (size_t)lds_bytes, st, out, iters); break;
    case 8: hipLaunchKernelGGL(sig_probe_fma_kernel<8>, grid, block, (size_t)lds_bytes, st, out, iters); break;
    case 16: hipLaunchKernelGGL(sig_probe_fma_kernel<16>, grid, block, (size_t)lds_bytes, st, out, iters); break;
    default: return SIG_ERR_INVALID;
    }
    return hipGetLastError() == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int sig_probe_fma_outer(float *out, int64_t waves, int64_t iters, int lds_bytes, void *hip_stream)
{
    if (!out || waves < 4 || waves % 4 || iters < 0 || waves / 4 > INT32_MAX) return SIG_ERR_INVALID;
    if (lds_bytes < 0 || lds_bytes > sig::kMaxLdsBytes) return SIG_ERR_INVALID;
    // the kernel reads its starting values from the first 64 floats of `out` (whatever they hold) and overwrites all of it
    hipLaunchKernelGGL(sig_probe_fma_outer_kernel, dim3((unsigned)(waves / 4)), dim3(256), (size_t)lds_bytes,
                       static_cast<hipStream_t>(hip_stream), out, out, iters);
    return hipGetLastError() == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

}  // extern "C"

// Abs-max / scale (Eq. 3, Section 4.1) and quantize (Eq. 1) kernels for gfx950.
// Both are single passes over fp32 data and are bound by HBM bandwidth:
// abs-max reads 4 B per element, quantize reads 4 B and writes 1 B.
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

constexpr int kEwThreads = 256;
constexpr int kEwUnroll = 4;  // float4 loads in flight per thread per trip

// Order of non-negative binary32 values equals the order of their bit patterns,
// so the reduction runs on integers and ends in one atomic max per workgroup.
__device__ __forceinline__ unsigned abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

__global__ void absmax_init_kernel(unsigned* amax_bits, unsigned* ticket)
{
    amax_bits[0] = 0u;
    if (ticket) ticket[0] = 0u;
}

// Empty tensor: behaves as all zeros.
__global__ void absmax_empty_kernel(float* amax, float* scale)
{
    amax[0] = 0.0f;
    if (scale) scale[0] = 1.0f;
}

// x is walked as aligned float4 vectors; `head` leading and the trailing scalars
// (fewer than 4 each) are taken by the first threads of block 0.
// `ticket` aliases the scale output: it counts finished workgroups and the last one
// overwrites it with S = 127 / amax, so scale and abs-max come out of one launch.
__global__ __launch_bounds__(kEwThreads) void absmax_kernel(const float* __restrict__ x, int64_t n, int head,
                                                             unsigned* amax_bits, unsigned* ticket)
{
    unsigned m = 0u;
    const float4* xv = reinterpret_cast<const float4*>(x + head);
    const int64_t nvec = (n - head) >> 2;
    const int64_t tail0 = head + (nvec << 2);
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x;
    for (; i + (kEwUnroll - 1) * stride < nvec; i += kEwUnroll * stride) {
        float4 v[kEwUnroll];
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) v[u] = xv[i + u * stride];
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) {
            unsigned a = max(abs_bits(v[u].x), abs_bits(v[u].y));
            unsigned b = max(abs_bits(v[u].z), abs_bits(v[u].w));
            m = max(m, max(a, b));
        }
    }
    for (; i < nvec; i += stride) {
        float4 v = xv[i];
        m = max(m, max(max(abs_bits(v.x), abs_bits(v.y)), max(abs_bits(v.z), abs_bits(v.w))));
    }
    if (blockIdx.x == 0) {
        if ((int)threadIdx.x < head) m = max(m, abs_bits(x[threadIdx.x]));
        int64_t t = tail0 + threadIdx.x;
        if (t < n) m = max(m, abs_bits(x[t]));
    }

    __shared__ unsigned wave_part[kEwThreads / 64];
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kEwThreads / 64; ++w) m = max(m, wave_part[w]);
        atomicMax(amax_bits, m);
        if (ticket) {
            __threadfence();
            unsigned done = atomicAdd(ticket, 1u);
            if (done == gridDim.x - 1) {
                float amax = __uint_as_float(atomicMax(amax_bits, 0u));  // read at the coherence point
                reinterpret_cast<float*>(ticket)[0] = scale_from_amax(amax);
            }
        }
    }
}

__global__ void scale_from_amax_kernel(const float* amax, float* scale) { scale[0] = scale_from_amax(amax[0]); }

__device__ __forceinline__ unsigned pack4(float4 v, float s)
{
    unsigned a = (unsigned)quantize_code(v.x, s) & 0xffu;
    unsigned b = (unsigned)quantize_code(v.y, s) & 0xffu;
    unsigned c = (unsigned)quantize_code(v.z, s) & 0xffu;
    unsigned d = (unsigned)quantize_code(v.w, s) & 0xffu;
    return a | (b << 8) | (c << 16) | (d << 24);
}

// Vector path: x 16-byte aligned, q 4-byte aligned.  Each lane turns one float4 into
// one packed dword, so a wave reads 1 KiB and writes 256 B, both contiguous.
__global__ __launch_bounds__(kEwThreads) void quantize_vec_kernel(const float* __restrict__ x, int64_t n,
                                                                   const float* __restrict__ scale,
                                                                   int8_t* __restrict__ q)
{
    const float s = scale[0];
    const float4* xv = reinterpret_cast<const float4*>(x);
    unsigned* qv = reinterpret_cast<unsigned*>(q);
    const int64_t nvec = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x;
    for (; i + (kEwUnroll - 1) * stride < nvec; i += kEwUnroll * stride) {
        float4 v[kEwUnroll];
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) v[u] = xv[i + u * stride];
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) qv[i + u * stride] = pack4(v[u], s);
    }
    for (; i < nvec; i += stride) qv[i] = pack4(xv[i], s);
    if (blockIdx.x == 0) {
        int64_t t = (nvec << 2) + threadIdx.x;
        if (t < n) q[t] = (int8_t)quantize_code(x[t], s);
    }
}

// Any alignment.
__global__ __launch_bounds__(kEwThreads) void quantize_scalar_kernel(const float* __restrict__ x, int64_t n,
                                                                      const float* __restrict__ scale,
                                                                      int8_t* __restrict__ q)
{
    const float s = scale[0];
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n; i += stride)
        q[i] = (int8_t)quantize_code(x[i], s);
}

static int ew_grid(int64_t work_items)
{
    int64_t per_block = (int64_t)kEwThreads * kEwUnroll;
    int64_t g = (work_items + per_block - 1) / per_block;
    const int64_t cap = 256 * 8;  // 8 workgroups per compute unit
    if (g < 1) g = 1;
    return (int)(g < cap ? g : cap);
}

int launch_absmax(const float* x, int64_t n, float* amax_out, float* scale_out, hipStream_t st)
{
    if (n == 0) {
        hipLaunchKernelGGL(absmax_empty_kernel, dim3(1), dim3(1), 0, st, amax_out, scale_out);
        return hipGetLastError() == hipSuccess ? 0 : 1;
    }
    unsigned* bits = reinterpret_cast<unsigned*>(amax_out);
    unsigned* ticket = reinterpret_cast<unsigned*>(scale_out);
    int head = (int)(((16 - (reinterpret_cast<uintptr_t>(x) & 15)) & 15) >> 2);
    if (head > n) head = (int)n;
    hipLaunchKernelGGL(absmax_init_kernel, dim3(1), dim3(1), 0, st, bits, ticket);
    hipLaunchKernelGGL(absmax_kernel, dim3(ew_grid((n - head) >> 2)), dim3(kEwThreads), 0, st, x, n, head, bits, ticket);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_scale_from_amax(const float* amax, float* scale_out, hipStream_t st)
{
    hipLaunchKernelGGL(scale_from_amax_kernel, dim3(1), dim3(1), 0, st, amax, scale_out);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_quantize(const float* x, int64_t n, const float* scale, int8_t* q, hipStream_t st)
{
    if (n == 0) return 0;
    bool vec = ((reinterpret_cast<uintptr_t>(x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(q) & 3) == 0);
    if (vec)
        hipLaunchKernelGGL(quantize_vec_kernel, dim3(ew_grid(n >> 2)), dim3(kEwThreads), 0, st, x, n, scale, q);
    else
        hipLaunchKernelGGL(quantize_scalar_kernel, dim3(ew_grid(n)), dim3(kEwThreads), 0, st, x, n, scale, q);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

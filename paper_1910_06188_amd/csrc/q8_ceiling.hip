// Measurement kernels behind the q8_debug_* entry points: what the chip itself sustains, measured next to
// the library's kernels by the benchmark (not part of the method).
//   - a register-resident loop of v_mfma_i32_32x32x32_i8 on caller-given int8 operands: the matrix pipes' own
//     ceiling on that data (operand bit toggling moves the clock the power management allows);
//   - a streaming copy and a streaming fill with 16-byte accesses: what the HBM sustains.
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

// Every wave runs iters x 8 independent MFMAs (128 accumulator registers) on 2 + 4 operand fragments it loads once.  One workgroup of
// 8 waves per compute unit keeps two waves on every SIMD.  sink is only written if an impossible sum shows up,
// which keeps the accumulators alive.
__global__ __launch_bounds__(512, 2) void mfma_rate_kernel(const v4i* __restrict__ ops, int iters, int* sink)
{
    v4i a[2], b[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = ops[(i * 512 + threadIdx.x) & 4095];
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = ops[((i + 2) * 512 + threadIdx.x) & 4095];
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i >> 2], b[i & 3], acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s ^= acc[i][e];
    if (s == 0x7fffffff && iters < 0) sink[0] = s;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void stream_fill_kernel(float4* __restrict__ dst, int64_t n16, float v)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const float4 f = make_float4(v, v, v, v);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = f;
}

int launch_mfma_rate(const int8_t* ops, int iters, int workgroups, int* sink, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(512), 0, st, reinterpret_cast<const v4i*>(ops), iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_stream_copy(const void* src, void* dst, int64_t nbytes, hipStream_t st)
{
    const int64_t n16 = nbytes / 16;
    if (n16 == 0) return 0;
    const int64_t want = (n16 + 256 * 8 - 1) / (256 * 8);
    const unsigned grid = (unsigned)(want < 8192 ? want : 8192);
    if (src)
        hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, st, reinterpret_cast<const float4*>(src),
                           reinterpret_cast<float4*>(dst), n16);
    else
        hipLaunchKernelGGL(stream_fill_kernel, dim3(grid), dim3(256), 0, st, reinterpret_cast<float4*>(dst), n16, 1.0f);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

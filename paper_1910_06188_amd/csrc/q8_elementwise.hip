// Abs-max / scale (Eq. 3, Section 4.1) and quantize (Eq. 1) kernels for gfx950, and the
// training-side twins: fake quantization (Section 2.2), the moving average of max|x| under
// Eq. 4 and the straight-through gradient (Eq. 5).  All are single passes over fp32 data and
// are bound by HBM bandwidth: abs-max reads 4 B per element, quantize reads 4 B and writes
// 1 B, fake quantization and the gradient copy read 4 B and write 4 B.
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

constexpr int kEwThreads = 256;
constexpr int kEwUnroll = 4;  // float4 loads in flight per thread per trip
constexpr int kMaxEwGrid = 2048;  // also the number of abs-max slots the fused path may use

// Order of non-negative binary32 values equals the order of their bit patterns,
// so the reduction runs on integers and ends in one atomic max per workgroup.
__device__ __forceinline__ unsigned abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// 16-byte load with the non-temporal hint.  The quantize pass is the quantizer's last read of the
// fp32 tensor: letting it stream past the Infinity Cache instead of being allocated there on its way
// through is worth 3.5 % of the whole dynamic layer step and 6.6 % of the stored-scale one (the
// abs-max pass in front keeps ordinary loads: the hint makes no difference there).
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_f4_nt(const float4* p)
{
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__global__ void absmax_init_kernel(unsigned* amax_bits) { amax_bits[0] = 0u; }

// Empty tensor: behaves as all zeros.
__global__ void absmax_empty_kernel(float* amax, float* scale)
{
    amax[0] = 0.0f;
    if (scale) scale[0] = 1.0f;
}

// Per-thread abs-max of this thread's share of x.  x is walked as aligned float4 vectors;
// `head` leading and the trailing scalars (fewer than 4 each) are taken by block 0.
// A maximum does not mind seeing an element twice, so the last trip clamps its indices to
// the final vector instead of branching: every trip has kAmUnroll loads in flight.
constexpr int kAmUnroll = 8;
__device__ __forceinline__ unsigned absmax_thread(const float* __restrict__ x, int64_t n, int head)
{
    unsigned m = 0u;
    const float4* xv = reinterpret_cast<const float4*>(x + head);
    const int64_t nvec = (n - head) >> 2;
    const int64_t tail0 = head + (nvec << 2);
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < nvec; i += kAmUnroll * stride) {
        float4 v[kAmUnroll];
#pragma unroll
        for (int u = 0; u < kAmUnroll; ++u) v[u] = xv[min(i + u * stride, nvec - 1)];
#pragma unroll
        for (int u = 0; u < kAmUnroll; ++u) {
            unsigned a = max(abs_bits(v[u].x), abs_bits(v[u].y));
            unsigned b = max(abs_bits(v[u].z), abs_bits(v[u].w));
            m = max(m, max(a, b));
        }
    }
    if (blockIdx.x == 0) {
        if ((int)threadIdx.x < head) m = max(m, abs_bits(x[threadIdx.x]));
        int64_t t = tail0 + threadIdx.x;
        if (t < n) m = max(m, abs_bits(x[t]));
    }
    return m;
}

// Max over the workgroup; valid in thread 0.
__device__ __forceinline__ unsigned block_max_u32(unsigned m)
{
    __shared__ unsigned wave_part[kEwThreads / 64];
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kEwThreads / 64; ++w) m = max(m, wave_part[w]);
    }
    return m;
}

// Stand-alone abs-max: one atomic max per workgroup into a zeroed word.  No fences and
// no "last block" ticket: device-scope fences cost an L2 write-back per workgroup on a
// chip whose eight L2s are not coherent with each other, so the scale is left to a
// follow-up launch (stream order makes the result visible).
__global__ __launch_bounds__(kEwThreads) void absmax_atomic_kernel(const float* __restrict__ x, int64_t n, int head,
                                                                    unsigned* amax_bits)
{
    unsigned m = block_max_u32(absmax_thread(x, n, head));
    // the maximum only grows: skip the serialising read-modify-write when there is nothing to add
    if (threadIdx.x == 0 && m > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(amax_bits, m);
}

// Fused path: each workgroup leaves its abs-max in its own slot; the quantize kernel that
// follows folds the slots.  No atomics at all.
__global__ __launch_bounds__(kEwThreads) void absmax_partial_kernel(const float* __restrict__ x, int64_t n, int head,
                                                                     unsigned* __restrict__ partials)
{
    unsigned m = block_max_u32(absmax_thread(x, n, head));
    if (threadIdx.x == 0) partials[blockIdx.x] = m;
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
        for (int u = 0; u < kEwUnroll; ++u) v[u] = load_f4_nt(&xv[i + u * stride]);
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) qv[i + u * stride] = pack4(v[u], s);
    }
    for (; i < nvec; i += stride) qv[i] = pack4(xv[i], s);
    if (blockIdx.x == 0) {
        int64_t t = (nvec << 2) + threadIdx.x;
        if (t < n) q[t] = (int8_t)quantize_code(x[t], s);
    }
}

// Scale from n_amax abs-max values (their maximum is the tensor's abs-max), Eq. 3; block 0
// also publishes the abs-max and the scale for the GEMM that follows.
__device__ __forceinline__ float scale_from_partials(const float* __restrict__ amax, int n_amax, float* amax_out,
                                                     float* scale_out, float* zero_slot)
{
    __shared__ unsigned folded;
    unsigned m = 0u;
    for (int i = threadIdx.x; i < n_amax; i += kEwThreads) m = max(m, abs_bits(amax[i]));
    m = block_max_u32(m);
    if (threadIdx.x == 0) folded = m;
    __syncthreads();
    const float a = __uint_as_float(folded);
    const float s = scale_from_amax(a);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (amax_out) amax_out[0] = a;
        scale_out[0] = s;
        if (zero_slot) zero_slot[0] = 0.0f;  // the abs-max slot the GEMM that follows accumulates into
    }
    return s;
}

template <bool kVec>
__global__ __launch_bounds__(kEwThreads) void quantize_amax_kernel(const float* __restrict__ x, int64_t n,
                                                                    const float* __restrict__ amax, int n_amax,
                                                                    float* amax_out, float* scale_out,
                                                                    int8_t* __restrict__ q, float* zero_slot)
{
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x;
    if (kVec) {
        const float4* xv = reinterpret_cast<const float4*>(x);
        unsigned* qv = reinterpret_cast<unsigned*>(q);
        const int64_t nvec = n >> 2;
        // The first trip's loads are requested before the partial maxima are folded: most workgroups
        // only make one or two trips, so the fold would otherwise sit in front of nearly all the work.
        float4 first[kEwUnroll];
        const bool full_first = i + (kEwUnroll - 1) * stride < nvec;
        if (full_first) {
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) first[u] = load_f4_nt(&xv[i + u * stride]);
        }
        const float s = scale_from_partials(amax, n_amax, amax_out, scale_out, zero_slot);
        if (full_first) {
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) qv[i + u * stride] = pack4(first[u], s);
            i += kEwUnroll * stride;
        }
        for (; i + (kEwUnroll - 1) * stride < nvec; i += kEwUnroll * stride) {
            float4 v[kEwUnroll];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) v[u] = load_f4_nt(&xv[i + u * stride]);
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) qv[i + u * stride] = pack4(v[u], s);
        }
        for (; i < nvec; i += stride) qv[i] = pack4(xv[i], s);
        if (blockIdx.x == 0) {
            int64_t t = (nvec << 2) + threadIdx.x;
            if (t < n) q[t] = (int8_t)quantize_code(x[t], s);
        }
    } else {
        const float s = scale_from_partials(amax, n_amax, amax_out, scale_out, zero_slot);
        for (; i < n; i += stride) q[i] = (int8_t)quantize_code(x[i], s);
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

// ---- training side ---------------------------------------------------------------------

// Section 2.2: Quantize(x | S, 127) / S, the code taken straight back to fp32 with one
// correctly rounded binary32 division.
__device__ __forceinline__ float fake_quantize_value(float x, float s)
{
    float r = round_half_away(__fmul_rn(x, s));
    r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return __fdiv_rn(r, s);
}

__device__ __forceinline__ float4 fake_quantize4(float4 v, float s)
{
    return make_float4(fake_quantize_value(v.x, s), fake_quantize_value(v.y, s), fake_quantize_value(v.z, s),
                       fake_quantize_value(v.w, s));
}

// x and xq 16-byte aligned (they may be the same buffer: every element is read before its
// own store and by no other thread).
template <bool kVec>
__global__ __launch_bounds__(kEwThreads) void fake_quantize_kernel(const float* x, int64_t n,
                                                                    const float* __restrict__ scale, float* xq)
{
    const float s = scale[0];
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x;
    if (kVec) {
        const float4* xv = reinterpret_cast<const float4*>(x);
        float4* yv = reinterpret_cast<float4*>(xq);
        const int64_t nvec = n >> 2;
        for (; i + (kEwUnroll - 1) * stride < nvec; i += kEwUnroll * stride) {
            float4 v[kEwUnroll];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) v[u] = xv[i + u * stride];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) yv[i + u * stride] = fake_quantize4(v[u], s);
        }
        for (; i < nvec; i += stride) yv[i] = fake_quantize4(xv[i], s);
        if (blockIdx.x == 0) {
            int64_t t = (nvec << 2) + threadIdx.x;
            if (t < n) xq[t] = fake_quantize_value(x[t], s);
        }
    } else {
        for (; i < n; i += stride) xq[i] = fake_quantize_value(x[i], s);
    }
}

// One step of the moving average under Eq. 4 (one workgroup): a = max of the n_amax values,
// state[0] <- a on the first call (state[1] == 0), else decay * state[0] + (1 - decay) * a,
// four binary32 operations in this order; state[1] <- 1; the scale is 127 over the average.
__global__ __launch_bounds__(kEwThreads) void ema_update_kernel(const float* __restrict__ amax, int n_amax,
                                                                 float decay, float* state, float* amax_out,
                                                                 float* scale_out)
{
    unsigned m = 0u;
    for (int i = threadIdx.x; i < n_amax; i += kEwThreads) m = max(m, abs_bits(amax[i]));
    m = block_max_u32(m);
    if (threadIdx.x == 0) {
        const float a = __uint_as_float(m);
        float e = a;
        if (state[1] != 0.0f) {
            const float keep = __fmul_rn(decay, state[0]);
            const float take = __fmul_rn(__fsub_rn(1.0f, decay), a);
            e = __fadd_rn(keep, take);
        }
        state[0] = e;
        state[1] = 1.0f;
        if (amax_out) amax_out[0] = a;
        if (scale_out) scale_out[0] = scale_from_amax(e);
    }
}

// Eq. 5: the gradient passes unchanged.  A plain streaming copy.
template <bool kVec>
__global__ __launch_bounds__(kEwThreads) void ste_backward_kernel(const float* __restrict__ g, int64_t n,
                                                                   float* __restrict__ gx)
{
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x;
    if (kVec) {
        const float4* gv = reinterpret_cast<const float4*>(g);
        float4* ov = reinterpret_cast<float4*>(gx);
        const int64_t nvec = n >> 2;
        for (; i + (kEwUnroll - 1) * stride < nvec; i += kEwUnroll * stride) {
            float4 v[kEwUnroll];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) v[u] = gv[i + u * stride];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) ov[i + u * stride] = v[u];
        }
        for (; i < nvec; i += stride) ov[i] = gv[i];
        if (blockIdx.x == 0) {
            int64_t t = (nvec << 2) + threadIdx.x;
            if (t < n) gx[t] = g[t];
        }
    } else {
        for (; i < n; i += stride) gx[i] = g[i];
    }
}

static int am_grid(int64_t nvec)
{
    int64_t per_block = (int64_t)kEwThreads * 6;  // 6 to 8 vectors per thread in one trip
    int64_t g = (nvec + per_block - 1) / per_block;
    if (g < 1) g = 1;
    return (int)(g < kMaxEwGrid ? g : kMaxEwGrid);
}

static int ew_grid(int64_t work_items)
{
    int64_t per_block = (int64_t)kEwThreads * kEwUnroll;
    int64_t g = (work_items + per_block - 1) / per_block;
    const int64_t cap = kMaxEwGrid;  // 4 workgroups per compute unit
    if (g < 1) g = 1;
    return (int)(g < cap ? g : cap);
}

static int head_of(const float* x, int64_t n)
{
    int head = (int)(((16 - (reinterpret_cast<uintptr_t>(x) & 15)) & 15) >> 2);
    return head > n ? (int)n : head;
}

int launch_absmax(const float* x, int64_t n, float* amax_out, float* scale_out, hipStream_t st)
{
    if (n == 0) {
        hipLaunchKernelGGL(absmax_empty_kernel, dim3(1), dim3(1), 0, st, amax_out, scale_out);
        return hipGetLastError() == hipSuccess ? 0 : 1;
    }
    unsigned* bits = reinterpret_cast<unsigned*>(amax_out);
    const int head = head_of(x, n);
    hipLaunchKernelGGL(absmax_init_kernel, dim3(1), dim3(1), 0, st, bits);
    // two workgroups per compute unit at most: every workgroup ends in a read or read-modify-write of one address
    const int g = am_grid((n - head) >> 2);
    hipLaunchKernelGGL(absmax_atomic_kernel, dim3(g < 512 ? g : 512), dim3(kEwThreads), 0, st, x, n, head, bits);
    if (scale_out) hipLaunchKernelGGL(scale_from_amax_kernel, dim3(1), dim3(1), 0, st, amax_out, scale_out);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_absmax_partial(const float* x, int64_t n, float* partials, int* n_partials, hipStream_t st)
{
    const int head = head_of(x, n);
    const int g = am_grid((n - head) >> 2);
    *n_partials = g;
    hipLaunchKernelGGL(absmax_partial_kernel, dim3(g), dim3(kEwThreads), 0, st, x, n, head,
                       reinterpret_cast<unsigned*>(partials));
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// Small tensors (latency-bound layers such as a 16-token batch): abs-max, scale and quantize in one launch of one
// workgroup that keeps its elements in registers between the two steps -- Eq. 3 then Eq. 1, same values as the
// two-kernel path, one launch less.
constexpr int kOnePassPerThread = 64;   // 256 threads x 64 = 16384 elements
constexpr int kOnePassMax = kEwThreads * kOnePassPerThread;
__global__ __launch_bounds__(kEwThreads) void quantize_onepass_kernel(const float* __restrict__ x, int n, float* amax_out,
                                                                       float* scale_out, int8_t* __restrict__ q,
                                                                       float* zero_slot)
{
    __shared__ unsigned folded;
    float v[kOnePassPerThread];
    unsigned m = 0u;
#pragma unroll
    for (int i = 0; i < kOnePassPerThread; ++i) {
        const int idx = i * kEwThreads + threadIdx.x;
        v[i] = idx < n ? x[idx] : 0.0f;
        m = max(m, abs_bits(v[i]));
    }
    m = block_max_u32(m);
    if (threadIdx.x == 0) folded = m;
    __syncthreads();
    const float a = __uint_as_float(folded);
    const float s = scale_from_amax(a);
    if (threadIdx.x == 0) {
        amax_out[0] = a;
        scale_out[0] = s;
        if (zero_slot) zero_slot[0] = 0.0f;
    }
#pragma unroll
    for (int i = 0; i < kOnePassPerThread; ++i) {
        const int idx = i * kEwThreads + threadIdx.x;
        if (idx < n) q[idx] = (int8_t)quantize_code(v[i], s);
    }
}

int quantize_onepass_max() { return kOnePassMax; }

int launch_quantize_onepass(const float* x, int64_t n, float* amax_out, float* scale_out, int8_t* q, float* zero_slot,
                            hipStream_t st)
{
    hipLaunchKernelGGL(quantize_onepass_kernel, dim3(1), dim3(kEwThreads), 0, st, x, (int)n, amax_out, scale_out, q, zero_slot);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_quantize_amax(const float* x, int64_t n, const float* amax, int n_amax, float* amax_out, float* scale_out,
                         int8_t* q, float* zero_slot, hipStream_t st)
{
    bool vec = ((reinterpret_cast<uintptr_t>(x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(q) & 3) == 0);
    if (vec)
        hipLaunchKernelGGL(quantize_amax_kernel<true>, dim3(ew_grid(n >> 2)), dim3(kEwThreads), 0, st, x, n, amax,
                           n_amax, amax_out, scale_out, q, zero_slot);
    else
        hipLaunchKernelGGL(quantize_amax_kernel<false>, dim3(ew_grid(n)), dim3(kEwThreads), 0, st, x, n, amax, n_amax,
                           amax_out, scale_out, q, zero_slot);
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

int launch_fake_quantize(const float* x, int64_t n, const float* scale, float* xq, hipStream_t st)
{
    if (n == 0) return 0;
    bool vec = ((reinterpret_cast<uintptr_t>(x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(xq) & 15) == 0);
    if (vec)
        hipLaunchKernelGGL(fake_quantize_kernel<true>, dim3(ew_grid(n >> 2)), dim3(kEwThreads), 0, st, x, n, scale, xq);
    else
        hipLaunchKernelGGL(fake_quantize_kernel<false>, dim3(ew_grid(n)), dim3(kEwThreads), 0, st, x, n, scale, xq);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_ema_update(const float* amax, int n_amax, float decay, float* state, float* amax_out, float* scale_out,
                      hipStream_t st)
{
    hipLaunchKernelGGL(ema_update_kernel, dim3(1), dim3(kEwThreads), 0, st, amax, n_amax, decay, state, amax_out,
                       scale_out);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_ste_backward(const float* g, int64_t n, float* gx, hipStream_t st)
{
    if (n == 0 || g == gx) return 0;
    bool vec = ((reinterpret_cast<uintptr_t>(g) & 15) == 0) && ((reinterpret_cast<uintptr_t>(gx) & 15) == 0);
    if (vec)
        hipLaunchKernelGGL(ste_backward_kernel<true>, dim3(ew_grid(n >> 2)), dim3(kEwThreads), 0, st, g, n, gx);
    else
        hipLaunchKernelGGL(ste_backward_kernel<false>, dim3(ew_grid(n)), dim3(kEwThreads), 0, st, g, n, gx);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

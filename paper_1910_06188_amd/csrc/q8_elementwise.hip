// Abs-max / scale (Eq. 3, Section 4.1) and quantize (Eq. 1) kernels for gfx950, and the
// training-side twins: fake quantization (Section 2.2), the moving average of max|x| under
// Eq. 4 and the straight-through gradient (Eq. 5).  All are single passes over fp32 data and
// are bound by HBM bandwidth: abs-max reads 4 B per element, quantize reads 4 B and writes
// 1 B, fake quantization and the gradient copy read 4 B and write 4 B.
#include <atomic>
#include <mutex>

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
    // A trip's kAmUnroll loads are neighbouring 4 KiB blocks, and block (trip * grid + b) goes to workgroup b: at any
    // time the whole grid reads one contiguous window of x.  With the loads of a trip a grid-stride apart instead
    // (every workgroup touching kAmUnroll distant pages at once) the same pass reads 5.0 TB/s instead of 6.2.
    const int64_t step = (int64_t)gridDim.x * (kAmUnroll * kEwThreads);
    for (int64_t i = (int64_t)blockIdx.x * (kAmUnroll * kEwThreads) + threadIdx.x; i < nvec; i += step) {
        float4 v[kAmUnroll];
#pragma unroll
        for (int u = 0; u < kAmUnroll; ++u) v[u] = xv[min(i + u * kEwThreads, nvec - 1)];
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
    // trips over blocks of kEwUnroll neighbouring 4 KiB pieces, block (trip * grid + b) to workgroup b (see absmax_thread)
    const int64_t step = (int64_t)gridDim.x * (kEwUnroll * kEwThreads);
    int64_t i = (int64_t)blockIdx.x * (kEwUnroll * kEwThreads) + threadIdx.x;
    for (; i + (kEwUnroll - 1) * kEwThreads < nvec; i += step) {
        float4 v[kEwUnroll];
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) v[u] = load_f4_nt(&xv[i + u * kEwThreads]);
#pragma unroll
        for (int u = 0; u < kEwUnroll; ++u) qv[i + u * kEwThreads] = pack4(v[u], s);
    }
    for (; i < nvec; i += step)  // the ragged last block
        for (int u = 0; u < kEwUnroll && i + u * kEwThreads < nvec; ++u) qv[i + u * kEwThreads] = pack4(xv[i + u * kEwThreads], s);
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
    if (kVec) {
        const float4* xv = reinterpret_cast<const float4*>(x);
        unsigned* qv = reinterpret_cast<unsigned*>(q);
        const int64_t nvec = n >> 2;
        // trips over blocks of kEwUnroll neighbouring 4 KiB pieces, block (trip * grid + b) to workgroup b (see absmax_thread)
        const int64_t step = (int64_t)gridDim.x * (kEwUnroll * kEwThreads);
        int64_t i = (int64_t)blockIdx.x * (kEwUnroll * kEwThreads) + threadIdx.x;
        // The first trip's loads are requested before the partial maxima are folded: most workgroups
        // only make one or two trips, so the fold would otherwise sit in front of nearly all the work.
        float4 first[kEwUnroll];
        const bool full_first = i + (kEwUnroll - 1) * kEwThreads < nvec;
        if (full_first) {
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) first[u] = load_f4_nt(&xv[i + u * kEwThreads]);
        }
        const float s = scale_from_partials(amax, n_amax, amax_out, scale_out, zero_slot);
        if (full_first) {
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) qv[i + u * kEwThreads] = pack4(first[u], s);
            i += step;
        }
        for (; i + (kEwUnroll - 1) * kEwThreads < nvec; i += step) {
            float4 v[kEwUnroll];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) v[u] = load_f4_nt(&xv[i + u * kEwThreads]);
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) qv[i + u * kEwThreads] = pack4(v[u], s);
        }
        for (; i < nvec; i += step)  // the ragged last block
            for (int u = 0; u < kEwUnroll && i + u * kEwThreads < nvec; ++u) qv[i + u * kEwThreads] = pack4(xv[i + u * kEwThreads], s);
        if (blockIdx.x == 0) {
            int64_t t = (nvec << 2) + threadIdx.x;
            if (t < n) q[t] = (int8_t)quantize_code(x[t], s);
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kEwThreads;
        const float s = scale_from_partials(amax, n_amax, amax_out, scale_out, zero_slot);
        for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n; i += stride) q[i] = (int8_t)quantize_code(x[i], s);
    }
}

// Large tensors with one scale known up front (a stored scale, or a single abs-max): one wave per workgroup and
// 4 KiB of x per wave.  Every lane turns four vectors 1 KiB apart into four packed dwords (each load instruction
// of the wave covers 1 KiB contiguous), the wave transposes the 256 dwords through LDS, and each lane stores 16
// consecutive codes with one 16-byte store: the wave writes its 1 KiB of codes with one instruction instead of four
// of 256 B.  Workgroups run in address order, so at any moment the chip reads one window of x and writes one window
// of q.  201 MB in, 50 MB out: 38.4 us (6.55 TB/s, what a streaming copy gets) against 40.5-41.3 us for 4-byte
// stores in any arrangement of workgroups and trips; 50 MB in: 10.9 against 11.3-11.5 us.
constexpr int kQwVec = 256;  // float4 per wave
template <bool kFromAmax>
__global__ __launch_bounds__(64) void quantize_wave_kernel(const float* __restrict__ x, int64_t n,
                                                           const float* __restrict__ src, float* amax_out,
                                                           float* scale_out, int8_t* __restrict__ q, float* zero_slot)
{
    __shared__ __attribute__((aligned(16))) unsigned codes[kQwVec];
    const int lane = threadIdx.x;
    const float4* xv = reinterpret_cast<const float4*>(x);
    const int64_t nvec = n >> 2;
    const int64_t base = (int64_t)blockIdx.x * kQwVec;
    const bool full = base + kQwVec <= nvec;
    float4 v[4];
    if (full) {
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = load_f4_nt(&xv[base + u * 64 + lane]);
    }
    float s;
    if (kFromAmax) {  // src[0] = the abs-max of the tensor: Eq. 3, and the scalars the GEMM that follows reads
        const float a = __uint_as_float(abs_bits(src[0]));
        s = scale_from_amax(a);
        if (blockIdx.x == 0 && lane == 0) {
            if (amax_out) amax_out[0] = a;
            scale_out[0] = s;
            if (zero_slot) zero_slot[0] = 0.0f;
        }
    } else {
        s = src[0];
    }
    if (full) {
#pragma unroll
        for (int u = 0; u < 4; ++u) codes[u * 64 + lane] = pack4(v[u], s);
        __syncthreads();  // one wave: orders its LDS writes before the read below
        const uint4 o = *reinterpret_cast<const uint4*>(&codes[4 * lane]);
        reinterpret_cast<uint4*>(q + 4 * base)[lane] = o;
    } else {
        for (int64_t i = base + lane; i < nvec; i += 64) reinterpret_cast<unsigned*>(q)[i] = pack4(xv[i], s);
    }
    if (blockIdx.x == 0) {
        const int64_t t = (nvec << 2) + lane;
        if (t < n) q[t] = (int8_t)quantize_code(x[t], s);
    }
}

// The wave kernel's shape: enough work to fill the chip, codes 16-byte aligned, a grid that fits 31 bits.
static bool quantize_wave_shape(const float* x, int64_t n, const int8_t* q)
{
    const int64_t nvec = n >> 2;
    return nvec >= 16384 && (nvec + kQwVec - 1) / kQwVec < ((int64_t)1 << 31) && (reinterpret_cast<uintptr_t>(x) & 15) == 0 &&
           (reinterpret_cast<uintptr_t>(q) & 15) == 0;
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
    if (kVec) {
        const float4* xv = reinterpret_cast<const float4*>(x);
        float4* yv = reinterpret_cast<float4*>(xq);
        const int64_t nvec = n >> 2;
        // trips over blocks of kEwUnroll neighbouring 4 KiB pieces, block (trip * grid + b) to workgroup b (see absmax_thread)
        const int64_t step = (int64_t)gridDim.x * (kEwUnroll * kEwThreads);
        int64_t i = (int64_t)blockIdx.x * (kEwUnroll * kEwThreads) + threadIdx.x;
        for (; i + (kEwUnroll - 1) * kEwThreads < nvec; i += step) {
            float4 v[kEwUnroll];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) v[u] = xv[i + u * kEwThreads];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) yv[i + u * kEwThreads] = fake_quantize4(v[u], s);
        }
        for (; i < nvec; i += step)  // the ragged last block
            for (int u = 0; u < kEwUnroll && i + u * kEwThreads < nvec; ++u) yv[i + u * kEwThreads] = fake_quantize4(xv[i + u * kEwThreads], s);
        if (blockIdx.x == 0) {
            int64_t t = (nvec << 2) + threadIdx.x;
            if (t < n) xq[t] = fake_quantize_value(x[t], s);
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kEwThreads;
        for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n; i += stride) xq[i] = fake_quantize_value(x[i], s);
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
    if (kVec) {
        const float4* gv = reinterpret_cast<const float4*>(g);
        float4* ov = reinterpret_cast<float4*>(gx);
        const int64_t nvec = n >> 2;
        // trips over blocks of kEwUnroll neighbouring 4 KiB pieces, block (trip * grid + b) to workgroup b (see absmax_thread)
        const int64_t step = (int64_t)gridDim.x * (kEwUnroll * kEwThreads);
        int64_t i = (int64_t)blockIdx.x * (kEwUnroll * kEwThreads) + threadIdx.x;
        for (; i + (kEwUnroll - 1) * kEwThreads < nvec; i += step) {
            float4 v[kEwUnroll];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) v[u] = gv[i + u * kEwThreads];
#pragma unroll
            for (int u = 0; u < kEwUnroll; ++u) ov[i + u * kEwThreads] = v[u];
        }
        for (; i < nvec; i += step)  // the ragged last block
            for (int u = 0; u < kEwUnroll && i + u * kEwThreads < nvec; ++u) ov[i + u * kEwThreads] = gv[i + u * kEwThreads];
        if (blockIdx.x == 0) {
            int64_t t = (nvec << 2) + threadIdx.x;
            if (t < n) gx[t] = g[t];
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kEwThreads;
        for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n; i += stride) gx[i] = g[i];
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
    // every workgroup ends in a read of one address and, while the maximum still grows, a read-modify-write of it
    const int g = am_grid((n - head) >> 2);
    hipLaunchKernelGGL(absmax_atomic_kernel, dim3(g < 256 ? g : 256), dim3(kEwThreads), 0, st, x, n, head, bits);
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

// ---- The dynamic quantizer in one pass over x (Section 4.1: abs-max of the incoming tensor, Eq. 3, then Eq. 1).
//
// The abs-max has to be complete before the first code can be formed, which is why the plain path reads x twice
// (9 bytes of traffic per element).  The register files of the chip (512 KiB per compute unit, 128 MiB in all)
// are larger than the activation tensors of an encoder layer (50 MB at 12288 tokens x 1024), so this kernel
// keeps the tensor in registers across the reduction: every workgroup loads its share (up to 48 floats per
// thread), leaves its maximum in a slot, waits at a grid-wide barrier, folds the slots, and quantizes from
// registers -- 5 bytes per element, x read once.
//
// The barrier needs every workgroup of the launch to be resident at once: the grid is one workgroup of 1024
// threads per compute unit, so it is whenever the chip is not held by something else; and no wait is unbounded --
// a workgroup that has polled `spin_limit` times stops waiting and reads the shares of the workgroups that have
// not published yet itself (same result, slower; what two such launches from different streams that each hold
// part of the chip fall back to).
//
// The barrier has no counter (256 read-modify-writes on one address serialise at the memory side, and the
// release/acquire fences around them write back and invalidate a whole L2 each: together 10 us): every workgroup
// publishes (ticket, maximum) as one 64-bit atomic store into its own slot, and one wave per workgroup polls all
// slots until each carries this launch's ticket.  Tickets come from a host-side counter, so a slot never carries
// the current ticket before its workgroup has written it; the slots are library-owned (zero when the code object
// is loaded, written by this kernel only), handed out round robin from a ring.  Should two launches in flight
// ever share a ring entry they overwrite each other's slots, which can only make a workgroup stop waiting and
// scan -- never use a maximum that is not its launch's.
constexpr int kRqThreads = 1024;
constexpr int kRqVec = 12;  // float4 per thread
constexpr int kRqMaxGroups = 256;
constexpr int kRqRing = 64;
static __device__ unsigned long long g_rq_slots[kRqRing][kRqMaxGroups];

__global__ __launch_bounds__(kRqThreads) void quantize_resident_kernel(const float4* __restrict__ x4, int n4,
                                                                        unsigned long long* slots, unsigned ticket,
                                                                        unsigned spin_limit, float* amax_out,
                                                                        float* scale_out, unsigned* __restrict__ q4,
                                                                        float* zero_slot)
{
    __shared__ unsigned wave_part[kRqThreads / 64];
    __shared__ unsigned folded;
    __shared__ unsigned long long missing[kRqMaxGroups / 64];
    const int G = (int)gridDim.x, w = (int)blockIdx.x, t = (int)threadIdx.x;
    // Workgroup w holds the 16 KiB blocks w, w + G, w + 2 G, ...: the k-th loads of all workgroups together are one
    // contiguous window of x, which is the order the memory system likes best (see absmax_thread).
    float4 v[kRqVec];
    unsigned m = 0u;
#pragma unroll
    for (int k = 0; k < kRqVec; ++k) {
        const int idx = (k * G + w) * kRqThreads + t;
        v[k] = idx < n4 ? load_f4_nt(&x4[idx]) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
#pragma unroll
    for (int k = 0; k < kRqVec; ++k)
        m = max(m, max(max(abs_bits(v[k].x), abs_bits(v[k].y)), max(abs_bits(v[k].z), abs_bits(v[k].w))));
    m = wave_max_u32(m);
    if ((t & 63) == 0) wave_part[t >> 6] = m;
    __syncthreads();
    if (t < 64) {
        const unsigned wm = wave_max_u32(t < kRqThreads / 64 ? wave_part[t] : 0u);
        if (t == 0)
            __hip_atomic_store(&slots[w], ((unsigned long long)ticket << 32) | wm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned a = 0u;
        for (unsigned polls = 0;; ++polls) {
            a = 0u;
            bool all_here = true;
#pragma unroll
            for (int r = 0; r < kRqMaxGroups / 64; ++r) {
                const int i = r * 64 + t;
                bool here = true;  // slots past the grid count as arrived
                if (i < G) {
                    const unsigned long long sv = __hip_atomic_load(&slots[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    here = (unsigned)(sv >> 32) == ticket;
                    if (here) a = max(a, (unsigned)sv);
                }
                const unsigned long long absent = __ballot(!here);
                if (t == 0) missing[r] = absent;
                all_here = all_here && absent == 0ull;
            }
            if (all_here || polls >= spin_limit) break;  // bounded: after spin_limit polls the absent ones are scanned below
            __builtin_amdgcn_s_sleep(8);
        }
        a = wave_max_u32(a);
        if (t == 0) folded = a;
    }
    __syncthreads();
    // Workgroups that had not published their maximum when this one stopped waiting: their shares of x are read
    // here instead (each element's maximum is the same whoever takes it), so the result never depends on the wait.
    unsigned extra = 0u;
    bool scanned = false;
#pragma unroll 1
    for (int r = 0; r < kRqMaxGroups / 64; ++r) {
        unsigned long long absent = missing[r];
        while (absent) {
            const int g = r * 64 + __builtin_ctzll(absent);
            absent &= absent - 1ull;
            scanned = true;
            for (int k = 0; k < kRqVec; ++k) {
                const int i = (k * G + g) * kRqThreads + t;
                if (i < n4) {
                    const float4 u = x4[i];
                    extra = max(extra, max(max(abs_bits(u.x), abs_bits(u.y)), max(abs_bits(u.z), abs_bits(u.w))));
                }
            }
        }
    }
    if (scanned) {  // uniform over the workgroup: `missing` is shared
        extra = wave_max_u32(extra);
        if ((t & 63) == 0) wave_part[t >> 6] = extra;  // its first contents were read before the barrier above
        __syncthreads();
        if (t == 0) {
            for (int i = 0; i < kRqThreads / 64; ++i) folded = max(folded, wave_part[i]);
        }
        __syncthreads();
    }
    const float a = __uint_as_float(folded);
    const float s = scale_from_amax(a);
    if (w == 0 && t == 0) {
        amax_out[0] = a;
        scale_out[0] = s;
        if (zero_slot) zero_slot[0] = 0.0f;
    }
#pragma unroll
    for (int k = 0; k < kRqVec; ++k) {
        const int idx = (k * G + w) * kRqThreads + t;
        if (idx < n4) q4[idx] = pack4(v[k], s);
    }
}

static std::atomic<unsigned> g_rq_next{0};
static std::atomic<unsigned> g_rq_spin_limit{64u};   // about 80 us of polling
static std::atomic<bool> g_rq_enabled{true};
static std::mutex g_rq_lock;
static unsigned long long* g_rq_slots_ptr[64] = {};
static int g_rq_groups[64] = {};

void set_quantize_resident(bool enabled, unsigned polls)
{
    g_rq_enabled.store(enabled);
    g_rq_spin_limit.store(polls);
}

// 0: launched.  1: the runtime refused the launch.  2: not a case for this kernel (the caller takes the two-pass path):
// shape or alignment, a tensor larger than the registers of the grid, a stream under graph capture (a replay would
// carry the ticket of the capture), or a device the slot ring cannot be looked up on.
int launch_quantize_resident(const float* x, int64_t n, float* amax_out, float* scale_out, int8_t* q, float* zero_slot,
                             hipStream_t st)
{
    if (!g_rq_enabled.load()) return 2;
    if (n % 4 != 0 || (reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(q) & 3)) return 2;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 2;
    unsigned long long* ring = nullptr;
    int groups = 0;
    {
        std::lock_guard<std::mutex> hold(g_rq_lock);
        if (!g_rq_slots_ptr[dev]) {
            void* p = nullptr;
            int cus = 0;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_rq_slots)) != hipSuccess ||
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
                (void)hipGetLastError();
                return 2;
            }
            g_rq_slots_ptr[dev] = static_cast<unsigned long long*>(p);
            g_rq_groups[dev] = cus < kRqMaxGroups ? cus : kRqMaxGroups;
        }
        ring = g_rq_slots_ptr[dev];
        groups = g_rq_groups[dev];
    }
    const int64_t n4 = n >> 2;
    if (n4 < (int64_t)groups * kRqThreads || n4 > (int64_t)groups * kRqThreads * kRqVec) return 2;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
        (void)hipGetLastError();
        return 2;
    }
    if (cap != hipStreamCaptureStatusNone) return 2;
    unsigned seq = g_rq_next.fetch_add(1u);
    const unsigned ticket = seq + 1u == 0u ? g_rq_next.fetch_add(1u) + 1u : seq + 1u;   // never 0: the slots start as zeros
    unsigned long long* slots = ring + (size_t)(seq % kRqRing) * kRqMaxGroups;
    hipLaunchKernelGGL(quantize_resident_kernel, dim3(groups), dim3(kRqThreads), 0, st, reinterpret_cast<const float4*>(x),
                       (int)n4, slots, ticket, g_rq_spin_limit.load(), amax_out, scale_out,
                       reinterpret_cast<unsigned*>(q), zero_slot);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_quantize_amax(const float* x, int64_t n, const float* amax, int n_amax, float* amax_out, float* scale_out,
                         int8_t* q, float* zero_slot, hipStream_t st)
{
    bool vec = ((reinterpret_cast<uintptr_t>(x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(q) & 3) == 0);
    // one abs-max value, and no slot to clear that later workgroups still have to read
    if (n_amax == 1 && zero_slot != amax && quantize_wave_shape(x, n, q))
        hipLaunchKernelGGL(quantize_wave_kernel<true>, dim3((unsigned)(((n >> 2) + kQwVec - 1) / kQwVec)), dim3(64), 0, st, x, n,
                           amax, amax_out, scale_out, q, zero_slot);
    else if (vec)
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
    if (quantize_wave_shape(x, n, q))
        hipLaunchKernelGGL(quantize_wave_kernel<false>, dim3((unsigned)(((n >> 2) + kQwVec - 1) / kQwVec)), dim3(64), 0, st, x, n,
                           scale, nullptr, nullptr, q, nullptr);
    else if (vec)
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

// The dynamic-quantization FC layer for a handful of tokens in ONE launch (Section 4.1 + Section 3): abs-max of x,
// S_x = 127 / max (Eq. 3), codes (Eq. 1), Int8 GEMM onto the Int32 bias, dequantize and the optional epilogue.
//
// At 16 tokens the layer is bound by launch latency, not by arithmetic: the two-launch path (quantizer, GEMM)
// spends most of its 12-13 us between the launches.  Here every workgroup repeats the small quantizer on its own
// (x is at most 16384 elements: 64 KiB out of L2) and keeps the codes in LDS as the A operand of its MFMAs, so no
// workgroup waits for another and nothing goes through memory between the two halves of the layer.
//
//   workgroup = 4 waves, owns 64 output columns and all (at most 32) rows
//   wave w    = the quarter [w K/4, (w+1) K/4) of the reduction for both 32x32 blocks; its share of the weights goes
//               straight from global memory into MFMA operand registers (a weight row is K-contiguous, 16 bytes of it
//               are one lane's operand), requested before the quantizer runs so that their latency hides behind it
//   the four partial accumulators are summed through LDS (exact: Int32), then the common per-element epilogue.
//
// Same device functions as the two-launch path for every rounding step, hence the same bits.
#include "q8_device.h"
#include "q8_epilogue.h"
#include "q8_launch.h"

namespace q8 {

typedef int v4i_s __attribute__((ext_vector_type(4)));
typedef int v16i_s __attribute__((ext_vector_type(16)));

constexpr int kFsThreads = 256;
constexpr int kFsRows = 32;        // rows of the A operand (tokens, zero-padded)
constexpr int kFsCols = 64;        // output columns per workgroup
constexpr int kFsMaxK = 1024;
constexpr int kFsMaxElems = 16384;  // elements of x a workgroup keeps in registers between abs-max and quantize
constexpr int kFsPerThread = kFsMaxElems / kFsThreads / 4;  // float4 per thread
static_assert(kFsMaxK == 8 * 128, "one kernel instance per K / 128 up to 8");

// kSteps = K / 128: 32-byte k-steps in a wave's quarter of K, fixed at compile time so that the weight loads and the
// fragment reads of all steps are issued back to back (a run-time trip count leaves a branch and a wait between them).
template <int kSteps>
__global__ __launch_bounds__(kFsThreads) void fc_small_kernel(const float* __restrict__ x, const int8_t* __restrict__ W,
                                                              int M, int N, int8_t* __restrict__ xq_out,
                                                              float* __restrict__ scal_out, Epilogue ep)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // A operand: row r at r * (K + 16) bytes -- the 16 bytes of padding put the 32 rows a fragment read touches on
    // different banks.  The partial accumulators reuse the space afterwards.
    __shared__ __attribute__((aligned(16))) char lds[kFsRows * (kFsMaxK + 16)];
    __shared__ unsigned wave_part[kFsThreads / 64];
    static_assert(sizeof(lds) >= 4 * 2 * 16 * 64 * 4, "room for the four waves' partial accumulators");
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int n0 = blockIdx.x * kFsCols;
    constexpr int K = kSteps * 128, stride = K + 16;

    // this wave's weight fragments: rows n0 + 32 b + l32 (clamped inside W: such columns are never stored)
    v4i_s fb[2][kSteps];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int n = min(n0 + 32 * b + l32, N - 1);
        const int8_t* wr = W + (int64_t)n * K + wave * (K / 4) + 16 * hi;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) fb[b][s] = *reinterpret_cast<const v4i_s*>(wr + 32 * s);
    }

    // the quantizer: x into registers, abs-max, S, codes into LDS
    const int n4 = (M * K) >> 2;  // K % 128 == 0, so rows are whole float4s
    float4 v[kFsPerThread];
    unsigned m = 0u;
#pragma unroll
    for (int j = 0; j < kFsPerThread; ++j) {
        const int i4 = j * kFsThreads + t;
        v[j] = i4 < n4 ? reinterpret_cast<const float4*>(x)[i4] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        m = max(m, max(max(__float_as_uint(v[j].x) & 0x7fffffffu, __float_as_uint(v[j].y) & 0x7fffffffu),
                       max(__float_as_uint(v[j].z) & 0x7fffffffu, __float_as_uint(v[j].w) & 0x7fffffffu)));
    }
    m = wave_max_u32(m);
    if (lane == 0) wave_part[wave] = m;
    __syncthreads();  // rows >= M of the A operand are left as they are: an output row depends on its own A row only
    m = max(max(wave_part[0], wave_part[1]), max(wave_part[2], wave_part[3]));
    const float amax = __uint_as_float(m);
    const float sx = scale_from_amax(amax);
    if (blockIdx.x == 0 && t == 0) {
        scal_out[0] = amax;
        scal_out[1] = sx;
    }
    constexpr int k4 = K >> 2;  // float4 per row
#pragma unroll
    for (int j = 0; j < kFsPerThread; ++j) {
        const int i4 = j * kFsThreads + t;
        if (i4 < n4) {
            const unsigned a = (unsigned)quantize_code(v[j].x, sx) & 0xffu, b = (unsigned)quantize_code(v[j].y, sx) & 0xffu;
            const unsigned c = (unsigned)quantize_code(v[j].z, sx) & 0xffu, d = (unsigned)quantize_code(v[j].w, sx) & 0xffu;
            const unsigned packed = a | (b << 8) | (c << 16) | (d << 24);
            const int row = i4 / k4, col4 = i4 - row * k4;  // k4 is a constant: a multiply and a shift
            *reinterpret_cast<unsigned*>(lds + row * stride + 4 * col4) = packed;
            if (blockIdx.x == 0) reinterpret_cast<unsigned*>(xq_out)[i4] = packed;  // the codes, for the caller
        }
    }
    __syncthreads();

    // Int8 GEMM: acc[b] register e of lane (l32, hi) = row 8 (e/4) + 4 hi + e%4, column n0 + 32 b + l32
    v16i_s acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0;
    const char* arow = lds + l32 * stride + wave * (K / 4) + 16 * hi;
    v4i_s fa[kSteps];
#pragma unroll
    for (int s = 0; s < kSteps; ++s) fa[s] = *reinterpret_cast<const v4i_s*>(arow + 32 * s);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
        acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[s], fb[0][s], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[s], fb[1][s], acc[1], 0, 0, 0);
    }
    __syncthreads();  // every wave is done reading the A operand
    int* part = reinterpret_cast<int*>(lds);  // [wave][b][e][lane]
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) part[((wave * 2 + b) * 16 + e) * 64 + lane] = acc[b][e];
    __syncthreads();

    // 2 x 16 x 64 outputs over 256 threads: thread (wave, lane) takes column 32 b + lane % 32 of both blocks b and the
    // registers e = wave + 4 i of each, so the per-column constants (Int32 bias, 1 / (S_x S_W)) are formed twice per thread
    const float next_scale = (ep.flags & 4u) ? ep.next_scale[0] : 0.0f;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int n = n0 + 32 * b + l32;
        if (n < N) {
            const ColConst cc = col_const(ep, n, sx);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = wave + 4 * i;
                const int sum = part[((0 * 2 + b) * 16 + e) * 64 + lane] + part[((1 * 2 + b) * 16 + e) * 64 + lane] +
                                part[((2 * 2 + b) * 16 + e) * 64 + lane] + part[((3 * 2 + b) * 16 + e) * 64 + lane];
                const int row = 8 * (e >> 2) + 4 * hi + (e & 3);
                if (row < M) epilogue_store(ep, (int64_t)row * N + n, sum + cc.bq, cc.r, next_scale);
            }
        }
    }
#endif
}

bool fc_small_eligible(const float* x, const int8_t* wq, int64_t M, int64_t N, int64_t K, unsigned flags)
{
    if (M < 1 || M > kFsRows || N < 1 || K < 128 || K > kFsMaxK || K % 128 != 0 || M * K > kFsMaxElems) return false;
    if (N > ((int64_t)1 << 30) || (flags & 2u)) return false;  // the abs-max slot would have to be cleared by an earlier launch
    return ((reinterpret_cast<uintptr_t>(x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(wq) & 15) == 0);
}

int launch_fc_small(const float* x, const int8_t* wq, int64_t M, int64_t N, int64_t K, int8_t* xq_out, float* scal_out,
                    const Epilogue& ep, hipStream_t st)
{
    const dim3 grid((unsigned)((N + kFsCols - 1) / kFsCols)), block(kFsThreads);
#define Q8_FS_LAUNCH(S) \
    case S: hipLaunchKernelGGL(fc_small_kernel<S>, grid, block, 0, st, x, wq, (int)M, (int)N, xq_out, scal_out, ep); break
    switch ((int)(K / 128)) {
        Q8_FS_LAUNCH(1);
        Q8_FS_LAUNCH(2);
        Q8_FS_LAUNCH(3);
        Q8_FS_LAUNCH(4);
        Q8_FS_LAUNCH(5);
        Q8_FS_LAUNCH(6);
        Q8_FS_LAUNCH(7);
        Q8_FS_LAUNCH(8);
        default: return 1;
    }
#undef Q8_FS_LAUNCH
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

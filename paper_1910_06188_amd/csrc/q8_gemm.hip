// Int8 x Int8 -> Int32 GEMM with the fused Int32-bias / dequantize epilogue of the
// quantized FC layer (Section 3), for gfx950.
//
//   acc[m,n] = bq[n] + sum_k xq[m,k] * wq[n,k]          y[m,n] = acc[m,n] / (S_x S_W)
//
// Both operands are K-contiguous ("NT" GEMM), so a 16-byte vector of either one is
// 16 consecutive k of one row -- exactly one lane's share of an i8 MFMA operand.
//
// MFMA kernel: a workgroup owns a BM x BN tile of y and walks K in steps of 128 bytes.
// Operand tiles go HBM/L2 -> LDS directly (buffer_load ... lds, 16 B per lane), double
// buffered; waves read 16-byte fragments back (ds_read_b128) and issue
// v_mfma_i32_32x32x32_i8.  LDS rows are 128 B (8 chunks of 16 B); chunk c of row r is
// kept at slot c ^ ((r ^ (r >> 3)) & 7), which spreads the 32 rows a fragment read
// touches over all banks.  The swizzle costs nothing on the way in because each lane of
// a direct-to-LDS load picks its own global address while the LDS side stays linear.
#include <type_traits>

#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

constexpr int kBK = 128;  // bytes (= int8 elements) of K per LDS row and per pipeline stage

__device__ __forceinline__ unsigned f32_abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

struct ColConst {
    int bq;    // quantized bias of this column
    float r;   // 1 / (S_x * S_W[group])
};

__device__ __forceinline__ ColConst col_const(const Epilogue& ep, int n, float sx)
{
    float sw = ep.sw[n / ep.cols_per_group];
    ColConst c;
    c.bq = ep.bias ? quantize_bias(ep.bias[n], sx, sw) : 0;
    c.r = dequant_factor(sx, sw);
    return c;
}

// One output element: dequantize, optional GELU, optional requantize; returns the
// bit pattern of |y| for the optional abs-max.
__device__ __forceinline__ unsigned epilogue_store(const Epilogue& ep, int64_t idx, int acc, float r, float next_scale)
{
    if (ep.acc_out) ep.acc_out[idx] = acc;
    float y = (float)acc * r;
    if (ep.flags & 1u) y = gelu_erf(y);
    if (ep.flags & 4u)
        reinterpret_cast<int8_t*>(ep.y)[idx] = (int8_t)quantize_code(y, next_scale);
    else
        reinterpret_cast<float*>(ep.y)[idx] = y;
    return f32_abs_bits(y);
}

__device__ __forceinline__ int swizzle_of_row(int r) { return (r ^ (r >> 3)) & 7; }

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of
// tile ids so that the tiles sharing operand rows meet in the same L2.
__device__ __forceinline__ int xcd_remap(int b, int g)
{
    int per = g >> 3, rem = g & 7;
    int xcd = b & 7, idx = b >> 3;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Compile-time loop: the body sees its index as a constant, so accumulator registers
// are always addressed statically.
template <int I, int E, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// kPlain: fp32 output with no optional epilogue stage and no accumulator dump -- the
// common case gets a kernel of its own so the optional stages cost it nothing.
template <int BM, int BN, int WGM, int WGN, bool kPlain>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_mfma_kernel(const int8_t* __restrict__ X,
                                                                   const int8_t* __restrict__ W, int M, int N, int K,
                                                                   int tiles_n, int group_m, Epilogue ep)
{
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    constexpr int NW = WGM * WGN;
    constexpr int TM = BM / WGM, TN = BN / WGN;  // wave tile
    constexpr int FM = TM / 32, FN = TN / 32;    // 32x32 MFMA blocks per wave tile
    constexpr int A_BYTES = BM * kBK, B_BYTES = BN * kBK, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LOADS = BM / 8 / NW, B_LOADS = BN / 8 / NW;  // 1 KiB wave loads per stage
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split over the waves");
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");

    __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    // tile id -> (tm, tn): panels of group_m tile rows, column-major inside a panel
    int pid = xcd_remap(blockIdx.x, gridDim.x);
    const int tiles_m = gridDim.x / tiles_n;
    {
        int panel = pid / (group_m * tiles_n);
        int first = panel * group_m;
        int rows = min(group_m, tiles_m - first);
        int in_panel = pid - panel * group_m * tiles_n;
        pid = (first + in_panel % rows) * tiles_n + in_panel / rows;
    }
    const int m0 = (pid / tiles_n) * BM;
    const int n0 = (pid % tiles_n) * BN;

    const __amdgpu_buffer_rsrc_t rsrc_a =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(X), 0, (int)((unsigned)M * (unsigned)K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(W), 0, (int)((unsigned)N * (unsigned)K), 0x00020000);

    // Per-lane global byte offsets of this lane's chunk in each wave load (k-step 0).
    // Rows beyond the matrix edge re-read the last row; their products are never stored.
    unsigned a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        int r = (wave * A_LOADS + i) * 8 + (lane >> 3);
        int c = (lane & 7) ^ swizzle_of_row(r);
        a_off[i] = (unsigned)min(m0 + r, M - 1) * (unsigned)K + (unsigned)(c * 16);
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        int r = (wave * B_LOADS + i) * 8 + (lane >> 3);
        int c = (lane & 7) ^ swizzle_of_row(r);
        b_off[i] = (unsigned)min(n0 + r, N - 1) * (unsigned)K + (unsigned)(c * 16);
    }

    auto issue_loads = [&](int kt, int stage) {
        char* base = lds + stage * STAGE;
        const int koff = kt * kBK;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(base + (wave * A_LOADS + i) * 1024), 16,
                                                     a_off[i], koff, 0, 0);
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(base + A_BYTES + (wave * B_LOADS + i) * 1024),
                                                     16, b_off[i], koff, 0, 0);
    };

    // Fragment addressing: lane l of a 32x32x32 MFMA supplies row (l % 32) and the
    // 16 k-bytes numbered (l / 32) of a 32-byte k-step, for both operands.
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, hi = lane >> 5;
    int a_row_off[FM], a_swz[FM], b_row_off[FN], b_swz[FN];
#pragma unroll
    for (int f = 0; f < FM; ++f) {
        int r = wm * TM + f * 32 + l32;
        a_row_off[f] = r * kBK;
        a_swz[f] = swizzle_of_row(r);
    }
#pragma unroll
    for (int f = 0; f < FN; ++f) {
        int r = wn * TN + f * 32 + l32;
        b_row_off[f] = A_BYTES + r * kBK;
        b_swz[f] = swizzle_of_row(r);
    }

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int KT = K / kBK;
    issue_loads(0, 0);
    for (int kt = 0; kt < KT; ++kt) {
        // this wave's share of stage kt has landed; after the barrier everyone's has, and
        // every wave is done reading the other stage, which the next loads overwrite
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 1 < KT) issue_loads(kt + 1, (kt + 1) & 1);
        const char* base = lds + (kt & 1) * STAGE;
#pragma unroll
        for (int ks = 0; ks < kBK / 32; ++ks) {
            v4i a[FM], b[FN];
#pragma unroll
            for (int f = 0; f < FM; ++f)
                a[f] = *reinterpret_cast<const v4i*>(base + a_row_off[f] + (((ks * 2 + hi) ^ a_swz[f]) << 4));
#pragma unroll
            for (int f = 0; f < FN; ++f)
                b[f] = *reinterpret_cast<const v4i*>(base + b_row_off[f] + (((ks * 2 + hi) ^ b_swz[f]) << 4));
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

    // Epilogue.  Accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4 and
    // column l%32 of its 32x32 block: 32 lanes store 128 contiguous bytes of one row.
    const float sx = ep.sx[0];
    float next_scale = 0.0f;
    if constexpr (!kPlain) next_scale = (ep.flags & 4u) ? ep.next_scale[0] : 0.0f;
    unsigned amax = 0u;
    static_for<0, FN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int n = n0 + wn * TN + j * 32 + l32;
        if (n < N) {
            const ColConst cc = col_const(ep, n, sx);
            static_for<0, FM>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                const int mb = m0 + wm * TM + i * 32 + 4 * hi;
                if constexpr (kPlain) {
                    float* yp = reinterpret_cast<float*>(ep.y) + (int64_t)mb * N + n;
                    static_for<0, 16>([&](auto ec) {
                        constexpr int e = decltype(ec)::value;
                        constexpr int dm = 8 * (e >> 2) + (e & 3);
                        if (mb + dm < M) yp[(int64_t)dm * N] = (float)(acc[i][j][e] + cc.bq) * cc.r;
                    });
                } else {
                    static_for<0, 16>([&](auto ec) {
                        constexpr int e = decltype(ec)::value;
                        const int m = mb + 8 * (e >> 2) + (e & 3);
                        if (m < M) {
                            unsigned ab =
                                epilogue_store(ep, (int64_t)m * N + n, acc[i][j][e] + cc.bq, cc.r, next_scale);
                            amax = max(amax, ab);
                        }
                    });
                }
            });
        }
    });
    if constexpr (!kPlain) {
        if (ep.flags & 2u) {
            amax = wave_max_u32(amax);
            if (lane == 0) atomicMax(reinterpret_cast<unsigned*>(ep.out_amax), amax);
        }
    }
#endif
}

// Any shape and alignment: one thread per output element.  Slow; same results.
__global__ __launch_bounds__(256) void gemm_generic_kernel(const int8_t* __restrict__ X, const int8_t* __restrict__ W,
                                                            int64_t M, int64_t N, int64_t K, Epilogue ep)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool valid = idx < M * N;
    unsigned ab = 0u;
    if (valid) {
        const int64_t m = idx / N;
        const int n = (int)(idx - m * N);
        const int8_t* xr = X + m * K;
        const int8_t* wr = W + (int64_t)n * K;
        int acc = 0;
        for (int64_t k = 0; k < K; ++k) acc += (int)xr[k] * (int)wr[k];
        const float sx = ep.sx[0];
        const ColConst cc = col_const(ep, n, sx);
        const float next_scale = (ep.flags & 4u) ? ep.next_scale[0] : 0.0f;
        ab = epilogue_store(ep, idx, acc + cc.bq, cc.r, next_scale);
    }
    if (ep.flags & 2u) {
        ab = wave_max_u32(ab);
        if ((threadIdx.x & 63) == 0) atomicMax(reinterpret_cast<unsigned*>(ep.out_amax), ab);
    }
}

static int g_variant = 0;
void set_gemm_variant(int v) { g_variant = v; }
int get_gemm_variant() { return g_variant; }

bool gemm_mfma_eligible(const int8_t* xq, const int8_t* wq, int64_t M, int64_t N, int64_t K)
{
    if (K < kBK || K % kBK != 0) return false;
    if ((reinterpret_cast<uintptr_t>(xq) & 15) || (reinterpret_cast<uintptr_t>(wq) & 15)) return false;
    const int64_t lim = (int64_t)1 << 31;  // buffer offsets and sizes stay in 31 bits
    if (M * K >= lim || N * K >= lim || M * N >= ((int64_t)1 << 40)) return false;
    return M > 0 && N > 0;
}

template <int BM, int BN, int WGM, int WGN>
static int launch_tile(const int8_t* xq, const int8_t* wq, int M, int N, int K, int group_m, const Epilogue& ep,
                       hipStream_t st)
{
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const dim3 grid(tiles_m * tiles_n), block(WGM * WGN * 64);
    if (ep.flags == 0u && ep.acc_out == nullptr)
        hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WGM, WGN, true>), grid, block, 0, st, xq, wq, M, N, K, tiles_n,
                           group_m, ep);
    else
        hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WGM, WGN, false>), grid, block, 0, st, xq, wq, M, N, K, tiles_n,
                           group_m, ep);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_gemm_mfma(const int8_t* xq, const int8_t* wq, int64_t M64, int64_t N64, int64_t K64, const Epilogue& ep,
                     hipStream_t st)
{
    const int M = (int)M64, N = (int)N64, K = (int)K64;
    int v = g_variant;
    if (v == 0) {
        // large tiles once there is enough work to fill 256 compute units with them
        const int64_t t256 = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
        v = t256 >= 256 ? 1 : 3;
    }
    const int group_m = 8;
    switch (v) {
        case 1: return launch_tile<256, 256, 2, 2>(xq, wq, M, N, K, group_m, ep, st);
        case 2: return launch_tile<256, 256, 2, 4>(xq, wq, M, N, K, group_m, ep, st);
        case 3: return launch_tile<128, 128, 2, 2>(xq, wq, M, N, K, group_m, ep, st);
        case 4: return launch_tile<256, 128, 2, 2>(xq, wq, M, N, K, group_m, ep, st);
        default: return 1;
    }
}

int launch_gemm_generic(const int8_t* xq, const int8_t* wq, int64_t M, int64_t N, int64_t K, const Epilogue& ep,
                        hipStream_t st)
{
    const int64_t blocks = (M * N + 255) / 256;
    hipLaunchKernelGGL(gemm_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, st, xq, wq, M, N, K, ep);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

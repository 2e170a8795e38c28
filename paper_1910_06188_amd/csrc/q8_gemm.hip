// Int8 x Int8 -> Int32 GEMM with the fused Int32-bias / dequantize epilogue of the
// quantized FC layer (Section 3), for gfx950.
//
//   acc[m,n] = bq[n] + sum_k xq[m,k] * wq[n,k]          y[m,n] = acc[m,n] / (S_x S_W)
//
// Both operands are K-contiguous ("NT" GEMM), so a 16-byte vector of either one is
// 16 consecutive k of one row -- exactly one lane's share of an i8 MFMA operand.
//
// MFMA kernel: a workgroup owns a BM x BN tile of y and walks K in stages of 64 bytes.
// Operand tiles go HBM/L2 -> LDS directly (buffer_load ... lds, 16 B per lane) into a
// ring of stage buffers; waves read 16-byte fragments back (ds_read_b128) and issue
// v_mfma_i32_32x32x32_i8.  LDS rows are swizzled so fragment reads are free of bank
// conflicts; the swizzle costs nothing on the way in because each lane of a
// direct-to-LDS load picks its own global address while the LDS side stays linear.
#include "q8_device.h"
#include "q8_epilogue.h"
#include "q8_launch.h"

namespace q8 {

constexpr int kBK = 128;  // the MFMA kernel's K granularity (see q8_gemm_kernel.h)

// One translation unit per tile shape.
int launch_tile_256x256_w4(const int8_t*, const int8_t*, int, int, int, int, const Epilogue&, hipStream_t);
int launch_tile_256x256_w8(const int8_t*, const int8_t*, int, int, int, int, const Epilogue&, hipStream_t);
int launch_tile_128x128_w4(const int8_t*, const int8_t*, int, int, int, int, const Epilogue&, hipStream_t);
int launch_tile_192x256_w4(const int8_t*, const int8_t*, int, int, int, int, const Epilogue&, hipStream_t);

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

int launch_gemm_mfma(const int8_t* xq, const int8_t* wq, int64_t M64, int64_t N64, int64_t K64, const Epilogue& ep,
                     hipStream_t st)
{
    const int M = (int)M64, N = (int)N64, K = (int)K64;
    int v = g_variant;
    if (v == 0) {
        // Pick the tile whose launch leaves the 256 compute units least idle: large tiles
        // once they fill the chip, else the 192-row tile if it divides the work evenly,
        // else small tiles.
        auto tiles = [&](int bm, int bn) { return (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
        auto idle = [&](int64_t t) { return (double)(((t + 255) / 256) * 256 - t) / (double)(((t + 255) / 256) * 256); };
        const int64_t t256 = tiles(256, 256), t192 = tiles(192, 256);
        if (t256 >= 256 && idle(t256) <= 0.10)
            v = 2;
        else if (t192 >= 192 && idle(t192) <= idle(t256))
            v = 4;
        else if (t256 >= 512)
            v = 2;
        else
            v = 3;
    }
    const int group_m = 8;
    switch (v) {
        case 1: return launch_tile_256x256_w4(xq, wq, M, N, K, group_m, ep, st);
        case 2: return launch_tile_256x256_w8(xq, wq, M, N, K, group_m, ep, st);
        case 3: return launch_tile_128x128_w4(xq, wq, M, N, K, group_m, ep, st);
        case 4: return launch_tile_192x256_w4(xq, wq, M, N, K, group_m, ep, st);
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

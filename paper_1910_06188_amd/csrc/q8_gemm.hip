// Int8 x Int8 -> Int32 GEMM with the fused Int32-bias / dequantize epilogue of the
// quantized FC layer (Section 3), for gfx950.
//
//   acc[m,n] = bq[n] + sum_k xq[m,k] * wq[n,k]          y[m,n] = acc[m,n] / (S_x S_W)
//
// Both operands are K-contiguous ("NT" GEMM), so a 16-byte vector of either one is
// 16 consecutive k of one row -- exactly one lane's share of an i8 MFMA operand.
//
// MFMA kernel: a workgroup owns a BM x BN tile of y and walks K in stages of 128 bytes.
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
int launch_tile_192x256_w8(const int8_t*, const int8_t*, int, int, int, int, const Epilogue&, hipStream_t);
int launch_tile_192x128_w4(const int8_t*, const int8_t*, int, int, int, int, const Epilogue&, hipStream_t);

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
    const int64_t lim = (int64_t)1 << 31;  // M, N and the tile count are ints in the kernel; buffers are addressed per tile
    if (M >= lim || N >= lim || ((M + 127) / 128) * ((N + 127) / 128) >= lim) return false;
    return M > 0 && N > 0;
}

int launch_gemm_mfma(const int8_t* xq, const int8_t* wq, int64_t M64, int64_t N64, int64_t K64, const Epilogue& ep,
                     hipStream_t st)
{
    const int M = (int)M64, N = (int)N64, K = (int)K64;
    int v = g_variant;
    if (v == 0) {
        // Pick the tile shape with the best expected use of the chip: the fraction of the launch's
        // workgroup slots that hold work (256 compute units; tiles whose rings take half of the
        // LDS run two workgroups per unit, one's epilogue under the other's main loop), times the
        // fraction of each tile that lies inside y, times a prior of the shape itself.  The priors
        // come from timing each FC of a BERT-Large layer inside the whole layer step, where the
        // outputs of the neighbouring kernels keep the HBM busy (timings of a GEMM run alone, its
        // operands and output warm in the caches, rank the shapes differently and do not carry
        // over): long reductions favour the 192x256 tiles (most MFMAs per byte staged); short ones
        // the paired tiles -- 128x128 with its three-deep w ring when the output is fp32, 192x128
        // when the epilogue writes int8.
        struct Cand { int variant, bm, bn, per_cu; double prior_long, prior_short_f32, prior_short_i8; };
        static const Cand cands[] = {
            {5, 192, 256, 1, 1.00, 0.97, 0.90}, {4, 192, 256, 1, 0.99, 0.90, 0.85}, {2, 256, 256, 1, 0.96, 0.97, 0.95},
            {6, 192, 128, 2, 0.95, 0.93, 1.00}, {3, 128, 128, 2, 0.90, 1.00, 0.97},
        };
        const bool int8_out = (ep.flags & 4u) != 0;
        double best = -1.0;
        for (const Cand& c : cands) {
            const int64_t tm = (M + c.bm - 1) / c.bm, tn = (N + c.bn - 1) / c.bn, tiles = tm * tn;
            const double inside = ((double)M * N) / ((double)tiles * c.bm * c.bn);
            // rounds of the launch: a last round that fills at most one workgroup per unit of a paired
            // shape runs unshared and ends early
            const int64_t slots = 256 * c.per_cu, full = tiles / slots, rem = tiles % slots;
            // a short reduction whose fp32 epilogue carries the GELU: inside the BERT-Large layer step the paired
            // 192x128 tile wins it (314 us for the whole dynamic step against 320 with 256x256 and 321 with 128x128);
            // at BERT-Base size (4096 x 3072 x 768) one three-quarter-full round of 256x256 tiles beats one and a
            // half rounds of 128x128 by 7 us of the 147 us layer: the epilogue of the half-empty last round of a
            // paired shape has nothing to hide under, so it is counted as a whole round here
            const bool gelu_f32_short = K < 2048 && !int8_out && (ep.flags & 1u);
            const double rounds =
                (double)full + (rem == 0 ? 0.0 : (c.per_cu == 2 && rem <= 256 && !gelu_f32_short) ? 0.6 : 1.0);
            const double slots_used = ((double)tiles / (double)slots) / rounds;
            double prior = K >= 2048 ? c.prior_long : (int8_out ? c.prior_short_i8 : c.prior_short_f32);
            if (gelu_f32_short && c.variant == 6) prior = 1.05;
            if (gelu_f32_short && c.variant == 2) prior = 1.04;
            const double score = prior * slots_used * inside;
            if (score > best) {
                best = score;
                v = c.variant;
            }
        }
    }
    // tile rows per raster panel: 4 is 1-2 us faster than 8 over the 317 us layer step but re-reads the weight tiles more
    // often (FFN1: 282 MB of HBM-side traffic against 248); 16 is 4 us slower
    const int group_m = 8;
    switch (v) {
        case 1: return launch_tile_256x256_w4(xq, wq, M, N, K, group_m, ep, st);
        case 2: return launch_tile_256x256_w8(xq, wq, M, N, K, group_m, ep, st);
        case 3: return launch_tile_128x128_w4(xq, wq, M, N, K, group_m, ep, st);
        case 4: return launch_tile_192x256_w4(xq, wq, M, N, K, group_m, ep, st);
        case 5: return launch_tile_192x256_w8(xq, wq, M, N, K, group_m, ep, st);
        case 6: return launch_tile_192x128_w4(xq, wq, M, N, K, group_m, ep, st);
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

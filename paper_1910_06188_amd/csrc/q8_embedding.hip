// Int8 embedding lookup (Section 3: the quantized Embedding layer returns Int8
// vectors) with optional dequantisation for the FP32 consumers.  Pure gather,
// bound by HBM/L2: per token H bytes read and H (int8) or 4H (fp32) bytes written.
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

__device__ __forceinline__ float4 dequant4(unsigned packed, float r)
{
    float4 o;
    o.x = (float)(int)(int8_t)(packed & 0xff) * r;
    o.y = (float)(int)(int8_t)((packed >> 8) & 0xff) * r;
    o.z = (float)(int)(int8_t)((packed >> 16) & 0xff) * r;
    o.w = (float)(int)(int8_t)(packed >> 24) * r;
    return o;
}

// A workgroup takes kEmbRows token rows per trip, one thread per 4 codes: the ids are wave-uniform
// (scalar loads) and fetched first, then the rows; a wave reads 256 contiguous table bytes and writes
// 1 KiB of contiguous fp32 (or 256 B of int8).  Needs H % 4 == 0.
constexpr int kEmbRows = 4;
template <bool kInt8Out>
__global__ __launch_bounds__(256) void embedding_vec_kernel(const unsigned* __restrict__ table,
                                                             const float* __restrict__ scale, int64_t V, int H4,
                                                             const int32_t* __restrict__ ids, int64_t T,
                                                             void* __restrict__ out, int32_t* err_flag)
{
    float r = 0.0f;
    if (!kInt8Out) r = __fdiv_rn(1.0f, scale[0]);
    for (int64_t t0 = (int64_t)blockIdx.x * kEmbRows; t0 < T; t0 += (int64_t)gridDim.x * kEmbRows) {
        const unsigned* row[kEmbRows];
        bool ok[kEmbRows];
#pragma unroll
        for (int k = 0; k < kEmbRows; ++k) {
            const int64_t id = ids[min(t0 + k, T - 1)];
            ok[k] = id >= 0 && id < V;
            if (!ok[k] && err_flag && threadIdx.x == 0) err_flag[0] = 1;
            row[k] = table + (ok[k] ? id : 0) * H4;
        }
        for (int j = threadIdx.x; j < H4; j += 256) {
            unsigned packed[kEmbRows];
#pragma unroll
            for (int k = 0; k < kEmbRows; ++k) packed[k] = ok[k] ? row[k][j] : 0u;
#pragma unroll
            for (int k = 0; k < kEmbRows; ++k) {
                if (t0 + k < T) {
                    if (kInt8Out)
                        reinterpret_cast<unsigned*>(out)[(t0 + k) * H4 + j] = packed[k];
                    else
                        reinterpret_cast<float4*>(out)[(t0 + k) * H4 + j] = dequant4(packed[k], r);
                }
            }
        }
    }
}

// Any H and alignment: one thread per element.
template <bool kInt8Out>
__global__ __launch_bounds__(256) void embedding_scalar_kernel(const int8_t* __restrict__ table,
                                                                const float* __restrict__ scale, int64_t V, int64_t H,
                                                                const int32_t* __restrict__ ids, int64_t T,
                                                                void* __restrict__ out, int32_t* err_flag)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= T * H) return;
    const int64_t t = w / H;
    const int64_t h = w - t * H;
    const int64_t id = ids[t];
    int q = 0;
    if (id >= 0 && id < V)
        q = table[id * H + h];
    else if (err_flag && h == 0)
        err_flag[0] = 1;
    if (kInt8Out)
        reinterpret_cast<int8_t*>(out)[w] = (int8_t)q;
    else
        reinterpret_cast<float*>(out)[w] = (float)q * __fdiv_rn(1.0f, scale[0]);
}

// word + position + token-type rows, each dequantised with its own scale, summed as
// (word + position) + type in fp32.  A workgroup takes kRows token rows per trip: their ids are
// fetched first, then all their table rows, then the sums are stored -- one row at a time the
// kernel was bound by the id -> row -> store latency chain, not by bandwidth.  Needs H % 4 == 0.
__global__ __launch_bounds__(256) void embedding_sum3_kernel(const unsigned* __restrict__ word, int64_t Vw,
                                                              const unsigned* __restrict__ pos, int64_t Vp,
                                                              const unsigned* __restrict__ typ, int64_t Vt,
                                                              const float* __restrict__ scales, int H4,
                                                              const int32_t* __restrict__ wid,
                                                              const int32_t* __restrict__ pid,
                                                              const int32_t* __restrict__ tid, int64_t T,
                                                              float4* __restrict__ out, int32_t* err_flag)
{
    const float r0 = __fdiv_rn(1.0f, scales[0]), r1 = __fdiv_rn(1.0f, scales[1]), r2 = __fdiv_rn(1.0f, scales[2]);
    for (int64_t t0 = (int64_t)blockIdx.x * kEmbRows; t0 < T; t0 += (int64_t)gridDim.x * kEmbRows) {
        const unsigned *wr[kEmbRows], *pr[kEmbRows], *tr[kEmbRows];
        bool ok[kEmbRows];
#pragma unroll
        for (int r = 0; r < kEmbRows; ++r) {  // ids are wave-uniform: scalar loads
            const int64_t t = min(t0 + r, T - 1);
            const int64_t a = wid[t], b = pid[t], c = tid[t];
            ok[r] = a >= 0 && a < Vw && b >= 0 && b < Vp && c >= 0 && c < Vt;
            if (!ok[r] && err_flag && threadIdx.x == 0) err_flag[0] = 1;
            wr[r] = word + (ok[r] ? a : 0) * H4;
            pr[r] = pos + (ok[r] ? b : 0) * H4;
            tr[r] = typ + (ok[r] ? c : 0) * H4;
        }
        for (int j = threadIdx.x; j < H4; j += 256) {
            unsigned cw[kEmbRows], cp[kEmbRows], ct[kEmbRows];
#pragma unroll
            for (int r = 0; r < kEmbRows; ++r) {  // a token with a bad id reads nothing (a table may be empty or null)
                cw[r] = ok[r] ? wr[r][j] : 0u;
                cp[r] = ok[r] ? pr[r][j] : 0u;
                ct[r] = ok[r] ? tr[r][j] : 0u;
            }
#pragma unroll
            for (int r = 0; r < kEmbRows; ++r) {
                if (t0 + r < T) {
                    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (ok[r]) {
                        const float4 x = dequant4(cw[r], r0);
                        const float4 y = dequant4(cp[r], r1);
                        const float4 z = dequant4(ct[r], r2);
                        o.x = (x.x + y.x) + z.x;
                        o.y = (x.y + y.y) + z.y;
                        o.z = (x.z + y.z) + z.z;
                        o.w = (x.w + y.w) + z.w;
                    }
                    out[(t0 + r) * H4 + j] = o;
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void embedding_sum3_scalar_kernel(const int8_t* __restrict__ word, int64_t Vw,
                                                                     const int8_t* __restrict__ pos, int64_t Vp,
                                                                     const int8_t* __restrict__ typ, int64_t Vt,
                                                                     const float* __restrict__ scales, int64_t H,
                                                                     const int32_t* __restrict__ wid,
                                                                     const int32_t* __restrict__ pid,
                                                                     const int32_t* __restrict__ tid, int64_t T,
                                                                     float* __restrict__ out, int32_t* err_flag)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= T * H) return;
    const int64_t t = w / H;
    const int64_t h = w - t * H;
    const int64_t a = wid[t], b = pid[t], c = tid[t];
    float o = 0.f;
    if (a >= 0 && a < Vw && b >= 0 && b < Vp && c >= 0 && c < Vt) {
        float x = (float)(int)word[a * H + h] * __fdiv_rn(1.0f, scales[0]);
        float y = (float)(int)pos[b * H + h] * __fdiv_rn(1.0f, scales[1]);
        float z = (float)(int)typ[c * H + h] * __fdiv_rn(1.0f, scales[2]);
        o = (x + y) + z;
    } else if (err_flag && h == 0) {
        err_flag[0] = 1;
    }
    out[w] = o;
}

static bool aligned(const void* p, unsigned a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int launch_embedding(const int8_t* table, const float* scale, int64_t V, int64_t H, const int32_t* ids, int64_t T,
                     void* out, int out_is_int8, int32_t* err_flag, hipStream_t st)
{
    if (T == 0 || H == 0) return 0;
    const bool vec = (H % 4 == 0) && aligned(table, 4) && aligned(out, out_is_int8 ? 4 : 16);
    if (vec) {
        const int H4 = (int)(H / 4);
        const int64_t groups = (T + kEmbRows - 1) / kEmbRows;
        const unsigned blocks = (unsigned)(groups < 8192 ? groups : 8192);  // kEmbRows token rows per workgroup trip, grid-stride
        const unsigned* tab = reinterpret_cast<const unsigned*>(table);
        if (out_is_int8)
            hipLaunchKernelGGL(embedding_vec_kernel<true>, dim3(blocks), dim3(256), 0, st, tab, scale, V, H4, ids, T,
                               out, err_flag);
        else
            hipLaunchKernelGGL(embedding_vec_kernel<false>, dim3(blocks), dim3(256), 0, st, tab, scale, V, H4, ids, T,
                               out, err_flag);
    } else {
        const unsigned blocks = (unsigned)((T * H + 255) / 256);
        if (out_is_int8)
            hipLaunchKernelGGL(embedding_scalar_kernel<true>, dim3(blocks), dim3(256), 0, st, table, scale, V, H, ids,
                               T, out, err_flag);
        else
            hipLaunchKernelGGL(embedding_scalar_kernel<false>, dim3(blocks), dim3(256), 0, st, table, scale, V, H, ids,
                               T, out, err_flag);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_embedding_sum3(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp, const int8_t* type,
                          int64_t Vt, const float* scales, int64_t H, const int32_t* wid, const int32_t* pid,
                          const int32_t* tid, int64_t T, float* out, int32_t* err_flag, hipStream_t st)
{
    if (T == 0 || H == 0) return 0;
    const bool vec = (H % 4 == 0) && aligned(word, 4) && aligned(pos, 4) && aligned(type, 4) && aligned(out, 16);
    if (vec) {
        const int H4 = (int)(H / 4);
        const int64_t groups = (T + kEmbRows - 1) / kEmbRows;
        const unsigned blocks = (unsigned)(groups < 8192 ? groups : 8192);  // kEmbRows token rows per workgroup trip, grid-stride
        hipLaunchKernelGGL(embedding_sum3_kernel, dim3(blocks), dim3(256), 0, st,
                           reinterpret_cast<const unsigned*>(word), Vw, reinterpret_cast<const unsigned*>(pos), Vp,
                           reinterpret_cast<const unsigned*>(type), Vt, scales, H4, wid, pid, tid, T,
                           reinterpret_cast<float4*>(out), err_flag);
    } else {
        const unsigned blocks = (unsigned)((T * H + 255) / 256);
        hipLaunchKernelGGL(embedding_sum3_scalar_kernel, dim3(blocks), dim3(256), 0, st, word, Vw, pos, Vp, type, Vt,
                           scales, H, wid, pid, tid, T, out, err_flag);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

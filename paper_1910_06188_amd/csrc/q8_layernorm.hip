// FP32 glue next to the quantized FC layers: Layer Normalization (Section 3 keeps it in FP32)
// fused with what surrounds it on the dynamic-quantization path -- the residual addition or the
// three-table int8 embedding lookup in front, and behind it the abs-max of its output, which is
// the first half of the next FC layer's quantizer (Section 4.1).  One pass over HBM instead of
// three or four: per element 4 B (+ 4 B residual, or 3 B of int8 codes) read and 4 B written.
//
// A wave owns a row.  The row lives in registers (up to 2048 columns); its sum and its sum of
// squared deviations are accumulated in binary64 and reduced across the wave in a fixed order,
// and the normalisation itself runs in binary64 with one final rounding, so the result is within
// an ulp of the exact one and the same bytes come out on every run.  The kernel is bound by
// memory: the binary64 arithmetic (about ten operations per element) hides under the loads.
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

constexpr int kLnThreads = 256;            // four waves = four rows per workgroup per trip
constexpr int kLnMaxVec = 8;               // float4 vectors per lane: rows up to 64 * 4 * 8 = 2048 columns
constexpr int kLnRowsShort = 2;           // rows a wave carries side by side: plain LayerNorm of rows of at most 1024 columns (with a
                                          // residual or the embedding rows in front the extra registers cost more than they win)
constexpr int kLnSlots = 2048;             // abs-max slots (= Q8_AMAX_SLOTS): one per workgroup, the rest zero

// Sum of a double over the 64 lanes, the same value in every lane, in a fixed order (so the same bytes come out on
// every run): an inclusive scan inside each row of 16 lanes with DPP row shifts (1, 2, 4, 8; lanes shifted in from
// outside the row contribute zero), then the row totals carried across rows with the two row broadcasts, and lane
// 63's total read back as a scalar.  A 64-bit value moves as two 32-bit DPP moves; the cross-lane traffic stays in
// the vector ALU (a butterfly of ds_bpermute exchanges costs ten times the latency, and a wave does two of these
// reductions per row with nothing else to do meanwhile).
template <int kCtrl, int kRowMask>
__device__ __forceinline__ double dpp_move_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), kCtrl, kRowMask, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), kCtrl, kRowMask, 0xf, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum_f64(double v)
{
    v += dpp_move_f64<0x111, 0xf>(v);  // row_shr:1
    v += dpp_move_f64<0x112, 0xf>(v);  // row_shr:2
    v += dpp_move_f64<0x114, 0xf>(v);  // row_shr:4
    v += dpp_move_f64<0x118, 0xf>(v);  // row_shr:8   -> lane 15 of each row holds its row's sum
    v += dpp_move_f64<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v += dpp_move_f64<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3 -> lane 63 holds the total
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}

// 16-byte load with the non-temporal hint: the inputs of a LayerNorm are read exactly once, and streamed
// past the Infinity Cache they leave it to the tensors that are read again (layer step with the fused
// LayerNorms 5 % faster with dynamic scales, 9 % with stored ones).
typedef float f32x4_ln __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_f4_nt_ln(const float4* p)
{
    const f32x4_ln v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_ln*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

struct EmbedSrc {
    const unsigned *word, *pos, *typ;  // int8 tables viewed as packed dwords
    int64_t Vw, Vp, Vt;
    const float* scales;
    const int32_t *wid, *pid, *tid;
    int32_t* err_flag;
};

__device__ __forceinline__ float4 dequant4_ln(unsigned packed, float r)
{
    float4 o;
    o.x = (float)(int)(int8_t)(packed & 0xff) * r;
    o.y = (float)(int)(int8_t)((packed >> 8) & 0xff) * r;
    o.z = (float)(int)(int8_t)((packed >> 16) & 0xff) * r;
    o.w = (float)(int)(int8_t)(packed >> 24) * r;
    return o;
}

// kSrc: 0 = x is a; 1 = x is a + r (one binary32 addition); 2 = x is the sum of three
// dequantized embedding rows, (word + position) + type as in the plain lookup.
// H % 4 == 0, H <= 256 * kVec (kVec float4 vectors per lane: 4 for rows of up to 1024 columns -- fewer registers, more
// waves in flight -- 8 up to 2048), every pointer 16-byte aligned (tables 4-byte).
template <int kSrc, int kVec, int kRows>
__global__ __launch_bounds__(kLnThreads) void layernorm_rows_kernel(const float* a, const float* r, EmbedSrc es,
                                                                     const float* __restrict__ gamma,
                                                                     const float* __restrict__ beta, double eps,
                                                                     int64_t M, int H, float* y,
                                                                     unsigned* __restrict__ amax_slots,
                                                                     const float* __restrict__ q_scale,
                                                                     unsigned* __restrict__ q_out)
{
    __shared__ unsigned wave_amax[kLnThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nvec = H >> 2;
    const float qs = q_out ? q_scale[0] : 0.0f;
    float amax = 0.0f;
    float r0 = 0.f, r1 = 0.f, r2 = 0.f;
    if (kSrc == 2) {
        r0 = __fdiv_rn(1.0f, es.scales[0]);
        r1 = __fdiv_rn(1.0f, es.scales[1]);
        r2 = __fdiv_rn(1.0f, es.scales[2]);
    }
    // A wave takes kRows consecutive rows per trip and carries them side by side: all their loads are in flight
    // together and their reductions -- chains of dependent cross-lane exchanges -- interleave, so a wave spends its
    // time waiting for memory once per trip instead of once per row.  Each row's arithmetic is unchanged.
    constexpr int kWaves = kLnThreads / 64;
    const int64_t row_step = (int64_t)gridDim.x * kWaves * kRows;
    // kSrc 0 and 1: the rows of the NEXT trip are requested as soon as this trip's have arrived, so their flight
    // covers this trip's reductions, normalisation and stores (a wave otherwise has nothing in flight while it
    // computes, and with four or five waves per SIMD the pass ran at 5 TB/s where a copy gets 6.5).
    float4 na[kRows][kVec], nr[kRows][kVec];
    auto request_rows = [&](int64_t r0) {
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            const int64_t row = r0 + q;
            const float4* av = reinterpret_cast<const float4*>(a) + row * nvec;
            const float4* rv = kSrc == 1 ? reinterpret_cast<const float4*>(r) + row * nvec : nullptr;
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const int v = j * 64 + lane;
                const bool in = row < M && v < nvec;
                na[q][j] = in ? load_f4_nt_ln(&av[v]) : make_float4(0.f, 0.f, 0.f, 0.f);
                if (kSrc == 1) nr[q][j] = in ? load_f4_nt_ln(&rv[v]) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    const int64_t first_row0 = ((int64_t)blockIdx.x * kWaves + wave) * kRows;
    if (kSrc != 2 && first_row0 < M) request_rows(first_row0);
    for (int64_t row0 = first_row0; row0 < M; row0 += row_step) {
        float4 x[kRows][kVec];
        bool live[kRows];
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            const int64_t row = row0 + q;
            live[q] = row < M;
#pragma unroll
            for (int j = 0; j < kVec; ++j) x[q][j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (kSrc != 2) {   // this trip's rows were requested a trip ago
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    x[q][j] = kSrc == 1 ? make_float4(__fadd_rn(na[q][j].x, nr[q][j].x), __fadd_rn(na[q][j].y, nr[q][j].y),
                                                      __fadd_rn(na[q][j].z, nr[q][j].z), __fadd_rn(na[q][j].w, nr[q][j].w))
                                        : na[q][j];
                continue;
            }
            if (!live[q]) continue;
            if (kSrc == 2) {
                const int64_t ia = es.wid[row], ib = es.pid[row], ic = es.tid[row];
                const bool ok = ia >= 0 && ia < es.Vw && ib >= 0 && ib < es.Vp && ic >= 0 && ic < es.Vt;
                if (!ok && es.err_flag && lane == 0) es.err_flag[0] = 1;
                const unsigned* wr = es.word + (ok ? ia : 0) * nvec;
                const unsigned* pr = es.pos + (ok ? ib : 0) * nvec;
                const unsigned* tr = es.typ + (ok ? ic : 0) * nvec;
#pragma unroll
                for (int j = 0; j < kVec; ++j) {
                    const int v = j * 64 + lane;
                    if (v < nvec && ok) {
                        const float4 p = dequant4_ln(wr[v], r0), t1 = dequant4_ln(pr[v], r1), t2 = dequant4_ln(tr[v], r2);
                        x[q][j] = make_float4((p.x + t1.x) + t2.x, (p.y + t1.y) + t2.y, (p.z + t1.z) + t2.z, (p.w + t1.w) + t2.w);
                    }
                }
            }
        }
        if (kSrc != 2 && row0 + row_step < M) request_rows(row0 + row_step);
        double mean[kRows], rstd[kRows];
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            double s = 0.0;
#pragma unroll
            for (int j = 0; j < kVec; ++j)  // lanes past the row hold zeros
                s += ((double)x[q][j].x + (double)x[q][j].y) + ((double)x[q][j].z + (double)x[q][j].w);
            mean[q] = s;
        }
#pragma unroll
        for (int q = 0; q < kRows; ++q) mean[q] = wave_sum_f64(mean[q]) / (double)H;
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            double ss = 0.0;
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                if (j * 64 + lane < nvec) {
                    const double d0 = (double)x[q][j].x - mean[q], d1 = (double)x[q][j].y - mean[q];
                    const double d2 = (double)x[q][j].z - mean[q], d3 = (double)x[q][j].w - mean[q];
                    ss += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
                }
            }
            rstd[q] = ss;
        }
#pragma unroll
        for (int q = 0; q < kRows; ++q) rstd[q] = 1.0 / sqrt(wave_sum_f64(rstd[q]) / (double)H + eps);
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            if (!live[q]) continue;
            const int64_t row = row0 + q;
            float4* yv = reinterpret_cast<float4*>(y) + row * nvec;
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const int v = j * 64 + lane;
                if (v < nvec) {
                    const float4 g = reinterpret_cast<const float4*>(gamma)[v], b = reinterpret_cast<const float4*>(beta)[v];
                    float4 o;
                    o.x = (float)(((double)x[q][j].x - mean[q]) * rstd[q] * (double)g.x + (double)b.x);
                    o.y = (float)(((double)x[q][j].y - mean[q]) * rstd[q] * (double)g.y + (double)b.y);
                    o.z = (float)(((double)x[q][j].z - mean[q]) * rstd[q] * (double)g.z + (double)b.z);
                    o.w = (float)(((double)x[q][j].w - mean[q]) * rstd[q] * (double)g.w + (double)b.w);
                    yv[v] = o;
                    if (q_out)  // stored-scale quantizer of the next FC (Eq. 1 on the rounded fp32 value), 4 codes per lane
                        q_out[row * nvec + v] = ((unsigned)quantize_code(o.x, qs) & 0xffu) | (((unsigned)quantize_code(o.y, qs) & 0xffu) << 8) |
                                                (((unsigned)quantize_code(o.z, qs) & 0xffu) << 16) | ((unsigned)quantize_code(o.w, qs) << 24);
                    amax = __builtin_fmaxf(amax, __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(o.x), __builtin_fabsf(o.y)),
                                                                __builtin_fmaxf(__builtin_fabsf(o.z), __builtin_fabsf(o.w))));
                }
            }
        }
    }
    if (amax_slots) {
        unsigned m = wave_max_u32(__float_as_uint(amax));  // non-negative floats order like their bit patterns
        if (lane == 0) wave_amax[wave] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int w = 1; w < kLnThreads / 64; ++w) m = max(m, wave_amax[w]);
            amax_slots[blockIdx.x] = m;
        }
        if (blockIdx.x == 0)  // slots no workgroup owns
            for (int i = gridDim.x + threadIdx.x; i < kLnSlots; i += kLnThreads) amax_slots[i] = 0u;
    }
}

// Any H and alignment: a wave per row, three passes over the row (the second and third come
// from cache).  Same arithmetic; rows are read element by element.
template <int kSrc>
__global__ __launch_bounds__(kLnThreads) void layernorm_generic_kernel(const float* a, const float* r, EmbedSrc es,
                                                                        const int8_t* word8, const int8_t* pos8,
                                                                        const int8_t* typ8,
                                                                        const float* __restrict__ gamma,
                                                                        const float* __restrict__ beta, double eps,
                                                                        int64_t M, int64_t H, float* y,
                                                                        unsigned* __restrict__ amax_slots,
                                                                        const float* __restrict__ q_scale,
                                                                        int8_t* __restrict__ q_out)
{
    __shared__ unsigned wave_amax[kLnThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float amax = 0.0f;
    const float qs = q_out ? q_scale[0] : 0.0f;
    float r0 = 0.f, r1 = 0.f, r2 = 0.f;
    if (kSrc == 2) {
        r0 = __fdiv_rn(1.0f, es.scales[0]);
        r1 = __fdiv_rn(1.0f, es.scales[1]);
        r2 = __fdiv_rn(1.0f, es.scales[2]);
    }
    for (int64_t row = ((int64_t)blockIdx.x * (kLnThreads / 64)) + wave; row < M;
         row += (int64_t)gridDim.x * (kLnThreads / 64)) {
        int64_t ia = 0, ib = 0, ic = 0;
        bool ok = true;
        if (kSrc == 2) {
            ia = es.wid[row], ib = es.pid[row], ic = es.tid[row];
            ok = ia >= 0 && ia < es.Vw && ib >= 0 && ib < es.Vp && ic >= 0 && ic < es.Vt;
            if (!ok && es.err_flag && lane == 0) es.err_flag[0] = 1;
        }
        auto value = [&](int64_t h) -> float {
            if (kSrc == 2) {
                if (!ok) return 0.0f;
                const float p = (float)(int)word8[ia * H + h] * r0, q = (float)(int)pos8[ib * H + h] * r1;
                const float t = (float)(int)typ8[ic * H + h] * r2;
                return (p + q) + t;
            }
            const float v = a[row * H + h];
            return kSrc == 1 ? __fadd_rn(v, r[row * H + h]) : v;
        };
        double s = 0.0;
        for (int64_t h = lane; h < H; h += 64) s += (double)value(h);
        const double mean = wave_sum_f64(s) / (double)H;
        double ss = 0.0;
        for (int64_t h = lane; h < H; h += 64) {
            const double d = (double)value(h) - mean;
            ss += d * d;
        }
        const double rstd = 1.0 / sqrt(wave_sum_f64(ss) / (double)H + eps);
        for (int64_t h = lane; h < H; h += 64) {
            const float o = (float)(((double)value(h) - mean) * rstd * (double)gamma[h] + (double)beta[h]);
            y[row * H + h] = o;
            if (q_out) q_out[row * H + h] = (int8_t)quantize_code(o, qs);
            amax = __builtin_fmaxf(amax, __builtin_fabsf(o));
        }
    }
    if (amax_slots) {
        unsigned m = wave_max_u32(__float_as_uint(amax));
        if (lane == 0) wave_amax[wave] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int w = 1; w < kLnThreads / 64; ++w) m = max(m, wave_amax[w]);
            amax_slots[blockIdx.x] = m;
        }
        if (blockIdx.x == 0)
            for (int i = gridDim.x + threadIdx.x; i < kLnSlots; i += kLnThreads) amax_slots[i] = 0u;
    }
}

__global__ void amax_slots_clear_kernel(unsigned* slots)
{
    for (int i = threadIdx.x; i < kLnSlots; i += kLnThreads) slots[i] = 0u;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

static int ln_grid(int64_t M, int rows_per_wave = 1)
{
    // one slot per workgroup caps the grid; within the cap, spread the rows evenly over the trips
    const int64_t per_wg = (int64_t)(kLnThreads / 64) * rows_per_wave;
    const int64_t need = (M + per_wg - 1) / per_wg;
    if (need <= 1) return 1;
    // at most 1024 workgroups (four per compute unit, all resident at once; fewer than the slots): beyond that a
    // workgroup makes several trips and fetches the next trip's rows under the arithmetic of the current one
    const int64_t cap = kLnSlots < 1024 ? kLnSlots : 1024;
    const int64_t trips = (need + cap - 1) / cap;
    return (int)((need + trips - 1) / trips);
}

int launch_layernorm(const float* a, const float* r, const float* gamma, const float* beta, float eps, int64_t M,
                     int64_t H, float* y, float* amax_slots, const float* q_scale, int8_t* q_out, hipStream_t st)
{
    unsigned* slots = reinterpret_cast<unsigned*>(amax_slots);
    if (M == 0) {
        if (slots) hipLaunchKernelGGL(amax_slots_clear_kernel, dim3(1), dim3(kLnThreads), 0, st, slots);
        return hipGetLastError() == hipSuccess ? 0 : 1;
    }
    EmbedSrc es = {};
    const bool fast = H % 4 == 0 && H <= 64 * 4 * kLnMaxVec && aligned16(a) && aligned16(y) && aligned16(gamma) &&
                      aligned16(beta) && (!r || aligned16(r)) && (reinterpret_cast<uintptr_t>(q_out) & 3) == 0;
    const dim3 grid(ln_grid(M)), block(kLnThreads);
    if (fast) {
        if (r)
            if (H <= 1024)
                hipLaunchKernelGGL((layernorm_rows_kernel<1, 4, 1>), dim3(ln_grid(M, 1)), block, 0, st, a, r, es, gamma, beta, (double)eps, M,
                               (int)H, y, slots, q_scale, reinterpret_cast<unsigned*>(q_out));
            else
                hipLaunchKernelGGL((layernorm_rows_kernel<1, 8, 1>), grid, block, 0, st, a, r, es, gamma, beta, (double)eps, M,
                               (int)H, y, slots, q_scale, reinterpret_cast<unsigned*>(q_out));
        else
            if (H <= 1024)
                hipLaunchKernelGGL((layernorm_rows_kernel<0, 4, kLnRowsShort>), dim3(ln_grid(M, kLnRowsShort)), block, 0, st, a, r, es, gamma, beta, (double)eps, M,
                               (int)H, y, slots, q_scale, reinterpret_cast<unsigned*>(q_out));
            else
                hipLaunchKernelGGL((layernorm_rows_kernel<0, 8, 1>), grid, block, 0, st, a, r, es, gamma, beta, (double)eps, M,
                               (int)H, y, slots, q_scale, reinterpret_cast<unsigned*>(q_out));
    } else {
        if (r)
            hipLaunchKernelGGL(layernorm_generic_kernel<1>, grid, block, 0, st, a, r, es, nullptr, nullptr, nullptr,
                               gamma, beta, (double)eps, M, H, y, slots, q_scale, q_out);
        else
            hipLaunchKernelGGL(layernorm_generic_kernel<0>, grid, block, 0, st, a, r, es, nullptr, nullptr, nullptr,
                               gamma, beta, (double)eps, M, H, y, slots, q_scale, q_out);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_embedding_sum3_layernorm(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp, const int8_t* typ,
                                    int64_t Vt, const float* scales, int64_t H, const int32_t* wid,
                                    const int32_t* pid, const int32_t* tid, int64_t T, const float* gamma,
                                    const float* beta, float eps, float* y, float* amax_slots, const float* q_scale,
                                    int8_t* q_out, int32_t* err_flag, hipStream_t st)
{
    unsigned* slots = reinterpret_cast<unsigned*>(amax_slots);
    if (T == 0) {
        if (slots) hipLaunchKernelGGL(amax_slots_clear_kernel, dim3(1), dim3(kLnThreads), 0, st, slots);
        return hipGetLastError() == hipSuccess ? 0 : 1;
    }
    EmbedSrc es;
    es.word = reinterpret_cast<const unsigned*>(word);
    es.pos = reinterpret_cast<const unsigned*>(pos);
    es.typ = reinterpret_cast<const unsigned*>(typ);
    es.Vw = Vw, es.Vp = Vp, es.Vt = Vt;
    es.scales = scales;
    es.wid = wid, es.pid = pid, es.tid = tid;
    es.err_flag = err_flag;
    const auto a4 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; };
    const bool fast = H % 4 == 0 && H <= 64 * 4 * kLnMaxVec && a4(word) && a4(pos) && a4(typ) && aligned16(y) &&
                      aligned16(gamma) && aligned16(beta) && a4(q_out);
    const dim3 grid(ln_grid(T)), block(kLnThreads);
    if (fast)
        if (H <= 1024)
                hipLaunchKernelGGL((layernorm_rows_kernel<2, 4, 1>), dim3(ln_grid(T, 1)), block, 0, st, nullptr, nullptr, es, gamma, beta,
                           (double)eps, T, (int)H, y, slots, q_scale, reinterpret_cast<unsigned*>(q_out));
            else
                hipLaunchKernelGGL((layernorm_rows_kernel<2, 8, 1>), grid, block, 0, st, nullptr, nullptr, es, gamma, beta,
                           (double)eps, T, (int)H, y, slots, q_scale, reinterpret_cast<unsigned*>(q_out));
    else
        hipLaunchKernelGGL(layernorm_generic_kernel<2>, grid, block, 0, st, nullptr, nullptr, es, word, pos, typ, gamma,
                           beta, (double)eps, T, H, y, slots, q_scale, q_out);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace q8

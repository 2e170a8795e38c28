// C ABI of the q8 library: argument checks, then launches.  See include/q8.h for the
// contract of every entry point.
#include "q8.h"
#include "q8_launch.h"

#include <mutex>

namespace {

// Scratch of q8_linear_f32_static, the entry point for callers that cannot allocate: Q8_SCAL_WORK floats
// (abs-max, scale, per-workgroup partial maxima; padded to 16 KiB) followed by the int8 codes of the
// activation tensor.  Every GPU the library runs on holds its own copy of this array until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address is looked up
// once per device (static_scratch below) and everything else -- kernel arguments included -- uses that pointer.
constexpr size_t kStaticScalBytes = 16384;
static_assert(kStaticScalBytes >= Q8_SCAL_WORK * sizeof(float), "scalar part of the static scratch");
static __device__ __align__(256) unsigned char scratch[kStaticScalBytes + Q8_STATIC_MAX_CODES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, or null if the runtime refuses the lookup.
unsigned char* static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    return g_scratch_ptr[dev];
}

inline bool misaligned(const void* p, unsigned a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
const unsigned kKnownFlags = Q8_EPI_GELU | Q8_EPI_ABSMAX | Q8_EPI_REQUANT;

q8_status check_linear(const int8_t* xq, const int8_t* wq, const float* bias, const float* sx, const float* sw,
                       int n_groups, int64_t M, int64_t N, int64_t K, void* y, int32_t* acc_out, float* out_amax,
                       const float* next_scale, uint32_t flags)
{
    if (M < 0 || N < 0 || K < 0 || K > Q8_MAX_K || n_groups < 1) return Q8_ERR_SHAPE;
    if (N % n_groups != 0) return Q8_ERR_SHAPE;
    if (flags & ~kKnownFlags) return Q8_ERR_FLAGS;
    if ((flags & Q8_EPI_ABSMAX) && !out_amax) return Q8_ERR_FLAGS;
    if ((flags & Q8_EPI_REQUANT) && !next_scale) return Q8_ERR_FLAGS;
    if (M == 0 || N == 0) return Q8_OK;
    if (!sx || !sw || !y) return Q8_ERR_NULL;
    if (K > 0 && (!xq || !wq)) return Q8_ERR_NULL;
    if (misaligned(bias, 4) || misaligned(sx, 4) || misaligned(sw, 4) || misaligned(acc_out, 4) ||
        misaligned(out_amax, 4) || misaligned(next_scale, 4))
        return Q8_ERR_ALIGN;
    if (!(flags & Q8_EPI_REQUANT) && misaligned(y, 4)) return Q8_ERR_ALIGN;
    if ((M * N + 255) / 256 > 0x7fffffffLL) return Q8_ERR_SHAPE;
    return Q8_OK;
}

q8::Epilogue make_epilogue(const float* bias, const float* sx, const float* sw, int n_groups, int64_t N, void* y,
                           int32_t* acc_out, float* out_amax, const float* next_scale, const float* residual,
                           uint32_t flags)
{
    q8::Epilogue ep;
    ep.residual = residual;
    ep.bias = bias;
    ep.sx = sx;
    ep.sw = sw;
    ep.n_groups = n_groups;
    ep.cols_per_group = (int)(N / n_groups);
    ep.y = y;
    ep.acc_out = acc_out;
    ep.out_amax = out_amax;
    ep.next_scale = next_scale;
    ep.flags = flags;
    return ep;
}

// Checks, fills the epilogue and picks the MFMA kernel or the generic one.
q8_status linear_launch(const int8_t* xq, const int8_t* wq, const float* bias, const float* sx, const float* sw,
                        int n_groups, int64_t M, int64_t N, int64_t K, void* y, int32_t* acc_out, float* out_amax,
                        const float* next_scale, const float* residual, uint32_t flags, void* stream)
{
    q8_status s = check_linear(xq, wq, bias, sx, sw, n_groups, M, N, K, y, acc_out, out_amax, next_scale, flags);
    if (s != Q8_OK || M == 0 || N == 0) return s;
    const q8::Epilogue ep = make_epilogue(bias, sx, sw, n_groups, N, y, acc_out, out_amax, next_scale, residual, flags);
    int rc = q8::gemm_mfma_eligible(xq, wq, M, N, K)
                 ? q8::launch_gemm_mfma(xq, wq, M, N, K, ep, as_stream(stream))
                 : q8::launch_gemm_generic(xq, wq, M, N, K, ep, as_stream(stream));
    return rc ? Q8_ERR_LAUNCH : Q8_OK;
}

}  // namespace

extern "C" {

q8_status q8_absmax(const float* x, int64_t n, float* amax_out, float* scale_out, void* stream)
{
    if (n < 0) return Q8_ERR_SHAPE;
    if (!amax_out || (n > 0 && !x)) return Q8_ERR_NULL;
    if (amax_out == scale_out) return Q8_ERR_NULL;
    if (misaligned(x, 4) || misaligned(amax_out, 4) || misaligned(scale_out, 4)) return Q8_ERR_ALIGN;
    return q8::launch_absmax(x, n, amax_out, scale_out, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_scale_from_amax(const float* amax, float* scale_out, void* stream)
{
    if (!amax || !scale_out) return Q8_ERR_NULL;
    if (misaligned(amax, 4) || misaligned(scale_out, 4)) return Q8_ERR_ALIGN;
    return q8::launch_scale_from_amax(amax, scale_out, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_quantize(const float* x, int64_t n, const float* scale, int8_t* q, void* stream)
{
    if (n < 0) return Q8_ERR_SHAPE;
    if (n == 0) return Q8_OK;
    if (!x || !scale || !q) return Q8_ERR_NULL;
    if (misaligned(x, 4) || misaligned(scale, 4)) return Q8_ERR_ALIGN;
    return q8::launch_quantize(x, n, scale, q, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_quantize_amax(const float* x, int64_t n, const float* amax, int n_amax, float* amax_out,
                           float* scale_out, int8_t* q, void* stream)
{
    if (n < 0 || n_amax < 1) return Q8_ERR_SHAPE;
    if (!amax || !scale_out) return Q8_ERR_NULL;
    if (n > 0 && (!x || !q)) return Q8_ERR_NULL;
    if (misaligned(x, 4) || misaligned(amax, 4) || misaligned(amax_out, 4) || misaligned(scale_out, 4))
        return Q8_ERR_ALIGN;
    // n = 0 still folds the n_amax values and publishes their maximum and the scale (one workgroup, no element read)
    return q8::launch_quantize_amax(x, n, amax, n_amax, amax_out, scale_out, q, nullptr, as_stream(stream)) ? Q8_ERR_LAUNCH
                                                                                                    : Q8_OK;
}

q8_status q8_linear(const int8_t* xq, const int8_t* wq, const float* bias, const float* sx, const float* sw,
                    int n_groups, int64_t M, int64_t N, int64_t K, void* y, int32_t* acc_out, float* out_amax,
                    const float* next_scale, uint32_t flags, void* stream)
{
    return linear_launch(xq, wq, bias, sx, sw, n_groups, M, N, K, y, acc_out, out_amax, next_scale, nullptr, flags,
                         stream);
}

q8_status q8_linear_residual(const int8_t* xq, const int8_t* wq, const float* bias, const float* sx, const float* sw,
                             int n_groups, int64_t M, int64_t N, int64_t K, const float* residual, float* y,
                             int32_t* acc_out, float* out_amax, uint32_t flags, void* stream)
{
    if (flags & Q8_EPI_REQUANT) return Q8_ERR_FLAGS;  // the sum is what the FP32 LayerNorm behind it reads
    if (M > 0 && N > 0 && !residual) return Q8_ERR_NULL;
    if (misaligned(residual, 4)) return Q8_ERR_ALIGN;
    return linear_launch(xq, wq, bias, sx, sw, n_groups, M, N, K, y, acc_out, out_amax, nullptr, residual, flags,
                         stream);
}

q8_status q8_quantize_dynamic(const float* x, int64_t n, int8_t* q, float* scal_work, float* zero_slot, void* stream)
{
    if (n < 0) return Q8_ERR_SHAPE;
    if (!scal_work) return Q8_ERR_NULL;
    if (n > 0 && (!x || !q)) return Q8_ERR_NULL;
    if (misaligned(x, 4) || misaligned(scal_work, 4) || misaligned(zero_slot, 4)) return Q8_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    if (n <= q8::quantize_onepass_max()) {
        // a tensor one workgroup can hold in registers (an empty one included): abs-max, scale and quantize in a single launch
        return q8::launch_quantize_onepass(x, n, scal_work, scal_work + 1, q, zero_slot, st) ? Q8_ERR_LAUNCH : Q8_OK;
    }
    // a tensor the chip's registers can hold between the reduction and the rounding: one pass, x read once
    const int one_pass = q8::launch_quantize_resident(x, n, scal_work, scal_work + 1, q, zero_slot, st);
    if (one_pass != 2) return one_pass ? Q8_ERR_LAUNCH : Q8_OK;
    // abs-max slots in scal_work[2..], folded by the quantize kernel: no atomics, no extra launch
    int slots = 0;
    if (q8::launch_absmax_partial(x, n, scal_work + 2, &slots, st)) return Q8_ERR_LAUNCH;
    return q8::launch_quantize_amax(x, n, scal_work + 2, slots, scal_work, scal_work + 1, q, zero_slot, st) ? Q8_ERR_LAUNCH
                                                                                                        : Q8_OK;
}

q8_status q8_linear_f32(const float* x, const int8_t* wq, const float* bias, const float* sw, int n_groups, int64_t M,
                        int64_t N, int64_t K, int8_t* xq_work, float* scal_work, void* y, int32_t* acc_out,
                        float* out_amax, const float* next_scale, uint32_t flags, void* stream)
{
    if (!scal_work) return Q8_ERR_NULL;
    if (misaligned(scal_work, 4)) return Q8_ERR_ALIGN;
    q8_status s = check_linear(xq_work, wq, bias, scal_work + 1, sw, n_groups, M, N, K, y, acc_out, out_amax,
                               next_scale, flags);
    if (s != Q8_OK) return s;
    if (M > 0 && K > 0 && (!x || !xq_work)) return Q8_ERR_NULL;
    if (misaligned(x, 4)) return Q8_ERR_ALIGN;
    // a handful of tokens: quantizer and GEMM in one launch (the layer is bound by launch latency there)
    if (q8::fc_small_eligible(x, wq, M, N, K, flags) && !misaligned(xq_work, 4)) {
        const q8::Epilogue ep =
            make_epilogue(bias, scal_work + 1, sw, n_groups, N, y, acc_out, out_amax, next_scale, nullptr, flags);
        return q8::launch_fc_small(x, wq, M, N, K, xq_work, scal_work, ep, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
    }
    s = q8_quantize_dynamic(x, M * K, xq_work, scal_work, (flags & Q8_EPI_ABSMAX) ? out_amax : nullptr, stream);
    if (s != Q8_OK) return s;
    return q8_linear(xq_work, wq, bias, scal_work + 1, sw, n_groups, M, N, K, y, acc_out, out_amax, next_scale, flags,
                     stream);
}

q8_status q8_linear_f32_static(const float* x, const int8_t* wq, const float* bias, const float* sw, int n_groups,
                               int64_t M, int64_t N, int64_t K, void* y, float* stats_out, float* out_amax,
                               const float* next_scale, uint32_t flags, void* stream)
{
    if (M < 0 || K < 0) return Q8_ERR_SHAPE;
    if (K > 0 && M > (int64_t)Q8_STATIC_MAX_CODES / K) return Q8_ERR_TOO_LARGE;
    if (misaligned(stats_out, 4)) return Q8_ERR_ALIGN;
    unsigned char* base = static_scratch();
    if (!base) return Q8_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: the abs-max pass writes every partial-maximum slot the
    // quantize pass reads, and the codes are written before the GEMM reads them.
    float* scal = reinterpret_cast<float*>(base);
    int8_t* codes = reinterpret_cast<int8_t*>(base + kStaticScalBytes);
    const q8_status s = q8_linear_f32(x, wq, bias, sw, n_groups, M, N, K, codes, scal, y, nullptr, out_amax, next_scale,
                                      flags, stream);
    if (s != Q8_OK || !stats_out) return s;
    // (max|x|, S_x) for the caller: a device-to-device copy of two floats on the same stream
    return hipMemcpyAsync(stats_out, scal, 2 * sizeof(float), hipMemcpyDeviceToDevice, as_stream(stream)) == hipSuccess
               ? Q8_OK
               : Q8_ERR_LAUNCH;
}

q8_status q8_linear_f32_slots(const float* x, const float* amax_slots, int n_slots, const int8_t* wq, const float* bias,
                              const float* sw, int n_groups, int64_t M, int64_t N, int64_t K, int8_t* xq_work,
                              float* scal_work, void* y, int32_t* acc_out, float* out_amax, const float* next_scale,
                              uint32_t flags, void* stream)
{
    if (!scal_work || !amax_slots) return Q8_ERR_NULL;
    if (n_slots < 1) return Q8_ERR_SHAPE;
    if (misaligned(scal_work, 4) || misaligned(amax_slots, 4)) return Q8_ERR_ALIGN;
    q8_status s = check_linear(xq_work, wq, bias, scal_work + 1, sw, n_groups, M, N, K, y, acc_out, out_amax,
                               next_scale, flags);
    if (s != Q8_OK) return s;
    if (M > 0 && K > 0 && (!x || !xq_work)) return Q8_ERR_NULL;
    if (misaligned(x, 4)) return Q8_ERR_ALIGN;
    if (q8::launch_quantize_amax(x, M * K, amax_slots, n_slots, scal_work, scal_work + 1, xq_work,
                                 (flags & Q8_EPI_ABSMAX) ? out_amax : nullptr, as_stream(stream)))
        return Q8_ERR_LAUNCH;  // M * K = 0: the slots are still folded into scal_work, nothing is quantized
    return q8_linear(xq_work, wq, bias, scal_work + 1, sw, n_groups, M, N, K, y, acc_out, out_amax, next_scale, flags,
                     stream);
}

q8_status q8_embedding(const int8_t* table, const float* scale, int64_t V, int64_t H, const int32_t* ids, int64_t T,
                       void* out, int out_is_int8, int32_t* err_flag, void* stream)
{
    if (V < 0 || H < 0 || T < 0) return Q8_ERR_SHAPE;
    if (T == 0 || H == 0) return Q8_OK;
    if (!ids || !out || (V > 0 && !table) || (!out_is_int8 && !scale)) return Q8_ERR_NULL;
    if (misaligned(ids, 4) || misaligned(err_flag, 4) || misaligned(scale, 4)) return Q8_ERR_ALIGN;
    if (!out_is_int8 && misaligned(out, 4)) return Q8_ERR_ALIGN;
    if ((T * H + 255) / 256 > 0x7fffffffLL) return Q8_ERR_SHAPE;
    return q8::launch_embedding(table, scale, V, H, ids, T, out, out_is_int8, err_flag, as_stream(stream))
               ? Q8_ERR_LAUNCH
               : Q8_OK;
}

q8_status q8_embedding_sum3(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp, const int8_t* type,
                            int64_t Vt, const float* scales, int64_t H, const int32_t* wid, const int32_t* pid,
                            const int32_t* tid, int64_t T, float* out, int32_t* err_flag, void* stream)
{
    if (Vw < 0 || Vp < 0 || Vt < 0 || H < 0 || T < 0) return Q8_ERR_SHAPE;
    if (T == 0 || H == 0) return Q8_OK;
    if (!wid || !pid || !tid || !out || !scales) return Q8_ERR_NULL;
    if ((Vw > 0 && !word) || (Vp > 0 && !pos) || (Vt > 0 && !type)) return Q8_ERR_NULL;
    if (misaligned(wid, 4) || misaligned(pid, 4) || misaligned(tid, 4) || misaligned(out, 4) ||
        misaligned(scales, 4) || misaligned(err_flag, 4))
        return Q8_ERR_ALIGN;
    if ((T * H + 255) / 256 > 0x7fffffffLL) return Q8_ERR_SHAPE;
    return q8::launch_embedding_sum3(word, Vw, pos, Vp, type, Vt, scales, H, wid, pid, tid, T, out, err_flag,
                                     as_stream(stream))
               ? Q8_ERR_LAUNCH
               : Q8_OK;
}

q8_status q8_fake_quantize(const float* x, int64_t n, const float* scale, float* xq, void* stream)
{
    if (n < 0) return Q8_ERR_SHAPE;
    if (n == 0) return Q8_OK;
    if (!x || !scale || !xq) return Q8_ERR_NULL;
    if (misaligned(x, 4) || misaligned(scale, 4) || misaligned(xq, 4)) return Q8_ERR_ALIGN;
    return q8::launch_fake_quantize(x, n, scale, xq, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_ema_update(const float* amax, int n_amax, float decay, float* state, float* amax_out, float* scale_out,
                        void* stream)
{
    if (n_amax < 1 || !(decay >= 0.0f && decay <= 1.0f)) return Q8_ERR_SHAPE;
    if (!amax || !state) return Q8_ERR_NULL;
    if (misaligned(amax, 4) || misaligned(state, 4) || misaligned(amax_out, 4) || misaligned(scale_out, 4))
        return Q8_ERR_ALIGN;
    return q8::launch_ema_update(amax, n_amax, decay, state, amax_out, scale_out, as_stream(stream)) ? Q8_ERR_LAUNCH
                                                                                                      : Q8_OK;
}

q8_status q8_fake_quantize_ema(const float* x, int64_t n, float decay, float* state, float* scal_work, float* xq,
                               void* stream)
{
    if (n < 0 || !(decay >= 0.0f && decay <= 1.0f)) return Q8_ERR_SHAPE;
    if (!state || !scal_work) return Q8_ERR_NULL;
    if (n > 0 && (!x || !xq)) return Q8_ERR_NULL;
    if (misaligned(x, 4) || misaligned(xq, 4) || misaligned(state, 4) || misaligned(scal_work, 4)) return Q8_ERR_ALIGN;
    int slots = 1;
    if (n == 0) {
        if (q8::launch_absmax(x, 0, scal_work + 2, nullptr, as_stream(stream))) return Q8_ERR_LAUNCH;
    } else if (q8::launch_absmax_partial(x, n, scal_work + 2, &slots, as_stream(stream))) {
        return Q8_ERR_LAUNCH;
    }
    if (q8::launch_ema_update(scal_work + 2, slots, decay, state, scal_work, scal_work + 1, as_stream(stream)))
        return Q8_ERR_LAUNCH;
    return q8::launch_fake_quantize(x, n, scal_work + 1, xq, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_ste_backward(const float* grad_xq, int64_t n, float* grad_x, void* stream)
{
    if (n < 0) return Q8_ERR_SHAPE;
    if (n == 0) return Q8_OK;
    if (!grad_xq || !grad_x) return Q8_ERR_NULL;
    if (misaligned(grad_xq, 4) || misaligned(grad_x, 4)) return Q8_ERR_ALIGN;
    return q8::launch_ste_backward(grad_xq, n, grad_x, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_layernorm_absmax(const float* a, const float* residual, const float* gamma, const float* beta, float eps,
                              int64_t M, int64_t H, float* y, float* amax_slots, const float* q_scale, int8_t* q_out,
                              void* stream)
{
    if (M < 0 || H < 1 || !(eps >= 0.0f)) return Q8_ERR_SHAPE;
    if (!gamma || !beta || ((q_scale == nullptr) != (q_out == nullptr))) return Q8_ERR_NULL;
    if (misaligned(q_scale, 4)) return Q8_ERR_ALIGN;
    if (M > 0 && (!a || !y)) return Q8_ERR_NULL;
    if (misaligned(a, 4) || misaligned(residual, 4) || misaligned(gamma, 4) || misaligned(beta, 4) || misaligned(y, 4) ||
        misaligned(amax_slots, 4))
        return Q8_ERR_ALIGN;
    return q8::launch_layernorm(a, residual, gamma, beta, eps, M, H, y, amax_slots, q_scale, q_out, as_stream(stream))
               ? Q8_ERR_LAUNCH
               : Q8_OK;
}

q8_status q8_embedding_sum3_layernorm(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp, const int8_t* type,
                                      int64_t Vt, const float* scales, int64_t H, const int32_t* wid,
                                      const int32_t* pid, const int32_t* tid, int64_t T, const float* gamma,
                                      const float* beta, float eps, float* y, float* amax_slots, const float* q_scale,
                                      int8_t* q_out, int32_t* err_flag, void* stream)
{
    if (Vw < 0 || Vp < 0 || Vt < 0 || H < 1 || T < 0 || !(eps >= 0.0f)) return Q8_ERR_SHAPE;
    if (!gamma || !beta || !scales || ((q_scale == nullptr) != (q_out == nullptr))) return Q8_ERR_NULL;
    if (misaligned(q_scale, 4)) return Q8_ERR_ALIGN;
    if (T > 0 && (!wid || !pid || !tid || !y)) return Q8_ERR_NULL;
    if (T > 0 && ((Vw > 0 && !word) || (Vp > 0 && !pos) || (Vt > 0 && !type))) return Q8_ERR_NULL;
    if (misaligned(wid, 4) || misaligned(pid, 4) || misaligned(tid, 4) || misaligned(y, 4) || misaligned(scales, 4) ||
        misaligned(err_flag, 4) || misaligned(gamma, 4) || misaligned(beta, 4) || misaligned(amax_slots, 4))
        return Q8_ERR_ALIGN;
    return q8::launch_embedding_sum3_layernorm(word, Vw, pos, Vp, type, Vt, scales, H, wid, pid, tid, T, gamma, beta, eps,
                                               y, amax_slots, q_scale, q_out, err_flag, as_stream(stream))
               ? Q8_ERR_LAUNCH
               : Q8_OK;
}

q8_status q8_attention(const float* qkv, int64_t B, int64_t S, int heads, int d, const float* mask, float scale, float* ctx,
                       float* amax_slots, const float* q_scale, int8_t* q_out, void* stream)
{
    if (B < 0 || S < 1 || heads < 1 || d < 1 || !(scale > 0.0f) || !(scale < 3.0e38f)) return Q8_ERR_SHAPE;
    if ((int64_t)heads * d > ((int64_t)1 << 24) || B > ((int64_t)1 << 40) / S) return Q8_ERR_SHAPE;
    if ((q_scale == nullptr) != (q_out == nullptr)) return Q8_ERR_NULL;
    if (B > 0 && (!qkv || (!ctx && !q_out))) return Q8_ERR_NULL;
    if (misaligned(qkv, 4) || misaligned(mask, 4) || misaligned(ctx, 4) || misaligned(amax_slots, 4) || misaligned(q_scale, 4))
        return Q8_ERR_ALIGN;
    if (B > 0 && !q8::attention_mfma_eligible(qkv, B, S, heads, d, ctx, q_out)) {
        if (S > q8::attention_generic_max_s() || B * heads * S >= ((int64_t)1 << 31)) return Q8_ERR_SHAPE;
    }
    return q8::launch_attention(qkv, B, S, heads, d, mask, scale, ctx, amax_slots, q_scale, q_out, as_stream(stream))
               ? Q8_ERR_LAUNCH
               : Q8_OK;
}

const char* q8_version(void) { return "q8 0.1.0 (gfx950)"; }

const char* q8_status_str(q8_status s)
{
    switch (s) {
        case Q8_OK: return "ok";
        case Q8_ERR_NULL: return "null pointer";
        case Q8_ERR_SHAPE: return "bad shape";
        case Q8_ERR_ALIGN: return "misaligned pointer";
        case Q8_ERR_FLAGS: return "bad epilogue flags";
        case Q8_ERR_LAUNCH: return "launch failed";
        case Q8_ERR_TOO_LARGE: return "input exceeds the static scratch of the no-allocation entry point";
    }
    return "unknown status";
}

q8_status q8_debug_mfma_rate(const int8_t* operands, int iters, int workgroups, int32_t* sink, void* stream)
{
    if (!operands || !sink) return Q8_ERR_NULL;
    if (iters < 0 || workgroups < 1 || workgroups > 65536) return Q8_ERR_SHAPE;
    if (misaligned(operands, 16) || misaligned(sink, 4)) return Q8_ERR_ALIGN;
    return q8::launch_mfma_rate(operands, iters, workgroups, sink, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_debug_loop_probe(int what, const void* operand_window, float* store_window, int stages, int32_t* sink, void* stream)
{
    if (!operand_window || !store_window || !sink) return Q8_ERR_NULL;
    if (stages < 0 || stages > (1 << 24)) return Q8_ERR_SHAPE;
    if (misaligned(operand_window, 16) || misaligned(store_window, 16) || misaligned(sink, 4)) return Q8_ERR_ALIGN;
    if (what != 0 && what != 7 && what != 15 && what != 64 && what != 71 && what != 79) return Q8_ERR_FLAGS;
    return q8::launch_loop_probe(what, operand_window, store_window, stages, sink, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

q8_status q8_debug_stream_copy(const void* src, void* dst, int64_t nbytes, void* stream)
{
    if (nbytes < 0 || nbytes % 16 || nbytes / 1024 > 0x7fffffffLL) return Q8_ERR_SHAPE;  // one wave per KiB: the grid is an int
    if (nbytes == 0) return Q8_OK;
    if (!dst) return Q8_ERR_NULL;
    if (misaligned(src, 16) || misaligned(dst, 16)) return Q8_ERR_ALIGN;
    return q8::launch_stream_copy(src, dst, nbytes, as_stream(stream)) ? Q8_ERR_LAUNCH : Q8_OK;
}

/* Tuning hook for the benchmark (not part of the method): pick the MFMA tile variant, 0 = automatic. */
void q8_debug_set_gemm_variant(int v) { q8::set_gemm_variant(v); }

void q8_debug_set_quantize_one_pass(int enabled, uint32_t barrier_polls)
{
    q8::set_quantize_resident(enabled != 0, barrier_polls);
}

}  // extern "C"

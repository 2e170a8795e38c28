// Host-side launchers behind the C ABI.  Each returns 0 on success, 1 if the HIP
// runtime refused a launch.  Arguments are already validated by the callers in
// q8_api.hip; all pointers are device pointers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace q8 {

// Everything the GEMM epilogue needs (Section 3: Int32 bias, dequantize; optional
// fp32 GELU, the encoder's residual addition, abs-max of the outputs, requantize with a stored scale).
struct Epilogue {
    const float* bias;        // fp32[N] or null
    const float* sx;          // fp32[1]
    const float* sw;          // fp32[n_groups]
    int n_groups;
    int cols_per_group;       // N / n_groups
    void* y;                  // fp32[M,N] or int8[M,N] (requant)
    int32_t* acc_out;         // int32[M,N] or null
    float* out_amax;          // fp32[1] or null
    const float* next_scale;  // fp32[1] or null
    const float* residual;    // fp32[M,N] added to the fp32 output (may be y itself), or null
    unsigned flags;
};

int launch_absmax(const float* x, int64_t n, float* amax_out, float* scale_out, hipStream_t st);
// Fused dynamic-quantization path: per-workgroup abs-max slots (at most 2048), folded by the quantize kernel.
int launch_absmax_partial(const float* x, int64_t n, float* partials, int* n_partials, hipStream_t st);
// zero_slot (or null): a float the kernel sets to 0, for the abs-max epilogue of the GEMM that follows.
int launch_quantize_amax(const float* x, int64_t n, const float* amax, int n_amax, float* amax_out, float* scale_out,
                         int8_t* q, float* zero_slot, hipStream_t st);
// Tensors of at most quantize_onepass_max() elements: abs-max, scale and quantize in one single-workgroup launch.
int quantize_onepass_max();
int launch_quantize_onepass(const float* x, int64_t n, float* amax_out, float* scale_out, int8_t* q, float* zero_slot,
                            hipStream_t st);
// Tensors that fit the chip's register files: abs-max, scale and quantize in one pass over x with a grid-wide barrier
// in between (q8_elementwise.hip).  Returns 2 when the case is not one for this kernel: take the two-pass path then.
int launch_quantize_resident(const float* x, int64_t n, float* amax_out, float* scale_out, int8_t* q, float* zero_slot,
                             hipStream_t st);
// Tuning hook: switch that kernel off, or set how often a workgroup polls the barrier before it stops waiting and scans
// x itself (0: never wait -- the tests run the give-up path that way).
void set_quantize_resident(bool enabled, unsigned polls);
int launch_scale_from_amax(const float* amax, float* scale_out, hipStream_t st);
int launch_quantize(const float* x, int64_t n, const float* scale, int8_t* q, hipStream_t st);

// Training side: fake quantization (Section 2.2), moving average of max|x| (Eq. 4), gradient copy (Eq. 5).
int launch_fake_quantize(const float* x, int64_t n, const float* scale, float* xq, hipStream_t st);
int launch_ema_update(const float* amax, int n_amax, float decay, float* state, float* amax_out, float* scale_out,
                      hipStream_t st);
int launch_ste_backward(const float* g, int64_t n, float* gx, hipStream_t st);

// True when the MFMA kernel can take the problem (K % 128 == 0, K >= 128, 16-byte
// aligned operands; operands and output may be of any size, they are addressed per tile).
bool gemm_mfma_eligible(const int8_t* xq, const int8_t* wq, int64_t M, int64_t N, int64_t K);
int launch_gemm_mfma(const int8_t* xq, const int8_t* wq, int64_t M, int64_t N, int64_t K, const Epilogue& ep,
                     hipStream_t st);
int launch_gemm_generic(const int8_t* xq, const int8_t* wq, int64_t M, int64_t N, int64_t K, const Epilogue& ep,
                        hipStream_t st);

// The dynamic-quantization FC layer of at most 32 tokens in one launch (q8_fc_small.hip): every workgroup runs the
// quantizer itself and keeps the codes in LDS.  Eligible: M <= 32, M * K <= 16384, K a multiple of 128 up to 1024,
// 16-byte aligned x and wq, no abs-max epilogue.  scal_out[0] = max|x|, scal_out[1] = S_x, xq_out = the codes.
bool fc_small_eligible(const float* x, const int8_t* wq, int64_t M, int64_t N, int64_t K, unsigned flags);
int launch_fc_small(const float* x, const int8_t* wq, int64_t M, int64_t N, int64_t K, int8_t* xq_out, float* scal_out,
                    const Epilogue& ep, hipStream_t st);

int launch_embedding(const int8_t* table, const float* scale, int64_t V, int64_t H, const int32_t* ids, int64_t T,
                     void* out, int out_is_int8, int32_t* err_flag, hipStream_t st);
int launch_embedding_sum3(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp, const int8_t* type,
                          int64_t Vt, const float* scales, int64_t H, const int32_t* wid, const int32_t* pid,
                          const int32_t* tid, int64_t T, float* out, int32_t* err_flag, hipStream_t st);

// FP32 glue fused with the abs-max of the next quantizer: LayerNorm of a (+ r), or of the summed embedding rows.
int launch_layernorm(const float* a, const float* r, const float* gamma, const float* beta, float eps, int64_t M,
                     int64_t H, float* y, float* amax_slots, const float* q_scale, int8_t* q_out, hipStream_t st);
int launch_embedding_sum3_layernorm(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp, const int8_t* typ,
                                    int64_t Vt, const float* scales, int64_t H, const int32_t* wid,
                                    const int32_t* pid, const int32_t* tid, int64_t T, const float* gamma,
                                    const float* beta, float eps, float* y, float* amax_slots, const float* q_scale,
                                    int8_t* q_out, int32_t* err_flag, hipStream_t st);

// FP32 softmax attention on the fused Q|K|V projection output (Section 3 keeps Softmax in FP32), with the
// abs-max slots or the stored-scale int8 codes of its result for the attention-output FC layer behind it.
// attention_mfma_eligible: head width 64 and 16-byte aligned tensors take the MFMA kernel, anything else a
// generic one that keeps one query's scores in LDS (S <= attention_generic_max_s()).
bool attention_mfma_eligible(const float* qkv, int64_t B, int64_t S, int heads, int d, const float* ctx, const int8_t* q_out);
int attention_generic_max_s();
int launch_attention(const float* qkv, int64_t B, int64_t S, int heads, int d, const float* mask, float scale, float* ctx,
                     float* amax_slots, const float* q_scale, int8_t* q_out, hipStream_t st);

// Measurement kernels of the benchmark (q8_ceiling.hip): a register-resident i8 MFMA loop on caller-given operands
// (iters x 8 MFMAs per wave, 8 waves per workgroup) and a streaming copy (src null: fill) with 16-byte accesses.
int launch_mfma_rate(const int8_t* ops, int iters, int workgroups, int* sink, hipStream_t st);
int launch_stream_copy(const void* src, void* dst, int64_t nbytes, hipStream_t st);
// One stage of a GEMM main loop piece by piece (what: 0, 7, 15, 64, 71 or 79; see q8_ceiling.hip): 256 workgroups x `stages` stages.
int launch_loop_probe(int what, const void* opbuf, float* ybuf, int stages, int* sink, hipStream_t st);

// Tuning hook used by the benchmark and tests: selects the MFMA tile variant
// (0 = automatic choice from the shape).
void set_gemm_variant(int v);
int get_gemm_variant();

}  // namespace q8

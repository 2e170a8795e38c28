/*
 * q8 -- symmetric linear int8 quantized fully-connected layer and int8 embedding
 * lookup for AMD MI355X (gfx950), after "Q8BERT: Quantized 8Bit BERT"
 * (arxiv 1910.06188).  C ABI; every kernel behind it is hand-written HIP.
 *
 * Conventions shared by all entry points
 *   - Every pointer is a DEVICE pointer owned by the caller unless a comment says
 *     "host".  The library never allocates, frees or keeps a pointer.  (Its own state on a GPU is two
 *     static device arrays that come with the code object: the scratch of q8_linear_f32_static and
 *     128 KiB of barrier slots for the one-pass dynamic quantizer.)
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it: no host synchronisation, no host read of device data.
 *     Data-dependent scalars (abs-max, scales) therefore live in device memory so
 *     calls chain on a stream without a round trip.
 *   - The return value reports what the host can see before launching (null
 *     pointers, shapes, alignment, launch failure).  Data-dependent problems are
 *     reported through device flags where stated.
 *   - Results are deterministic: same bytes in, same bytes out.
 *   - Inputs must be finite; NaN/Inf give unspecified codes (the method has no
 *     meaning for them).
 *   - Tensors are dense row-major.  Activations x[M,K], weights w[N,K]
 *     (the layer computes x w^T + b), outputs y[M,N].
 *   - M is the highest quantized value of Eq. 2: 127 for int8 codes, 2^31-1 for
 *     the int32 bias.
 */
#ifndef Q8_H
#define Q8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    Q8_OK = 0,
    Q8_ERR_NULL = 1,   /* a required pointer is NULL */
    Q8_ERR_SHAPE = 2,  /* negative size, K above Q8_MAX_K, n_groups not dividing N, more than 2^39 output elements */
    Q8_ERR_ALIGN = 3,  /* a pointer breaks the alignment its type needs (4 bytes for float/int32) */
    Q8_ERR_FLAGS = 4,  /* unknown epilogue bit, or a flag without the pointer it needs */
    Q8_ERR_LAUNCH = 5,    /* the HIP runtime refused a launch */
    Q8_ERR_TOO_LARGE = 6  /* q8_linear_f32_static: M*K exceeds Q8_STATIC_MAX_CODES */
} q8_status;

/* Largest reduction length: 128*128*K must stay below 2^31 so that no int8 input,
 * -128 included, can overflow the int32 accumulator before the bias is added. */
#define Q8_MAX_K 131071

/* Floats of scalar scratch q8_linear_f32 needs: abs-max, scale and up to 2048 partial maxima. */
#define Q8_SCAL_WORK 2050

/* Largest activation tensor, in elements (M*K), that q8_linear_f32_static takes: its int8 codes live in a
 * static device array of this many bytes (64 MiB; every FC input of a BERT-Large layer at 12288 tokens fits). */
#define Q8_STATIC_MAX_CODES (64u << 20)

/* Abs-max slots written by the fused LayerNorm entry points (fp32 each; unused slots are set to 0). */
#define Q8_AMAX_SLOTS 2048

/* q8_linear epilogue bits. */
#define Q8_EPI_GELU 1u     /* y <- gelu(y) = y Phi(y), the erf form (not the tanh form), in fp32 (GELU stays
                              FP32: Section 3).  Evaluated as max(y,0) - |y| Q(|y|) with log2 of the normal upper
                              tail Q fitted on [0, 6] by a degree-6 polynomial: absolute error <= 5.2e-7, i.e. the
                              result agrees with the exact function within 1e-6 absolute + 1e-5 relative, not
                              within the 1e-6 relative of the FC output itself. */
#define Q8_EPI_ABSMAX 2u   /* out_amax[0] <- max(out_amax[0], max|y|) over the fp32 outputs of this call */
#define Q8_EPI_REQUANT 4u  /* y is written as int8 codes Quantize(y | next_scale[0], 127) instead of fp32 */

/*
 * Abs-max and scale of a whole tensor: Eq. 3, S = M / max|x| with M = 127, which
 * Section 4.1 (dynamic quantization) also applies to each incoming activation tensor.
 *   x          fp32[n], any shape flattened; n >= 0 (n = 0 behaves as all zeros).
 *   amax_out   fp32[1], required: receives max_i |x_i|.
 *   scale_out  fp32[1] or NULL: receives 127 / amax as one binary32 division, or 1.0
 *              when amax is 0 (every code is then 0).
 * The previous contents of both outputs are ignored.
 */
q8_status q8_absmax(const float* x, int64_t n, float* amax_out, float* scale_out, void* stream);

/*
 * Scale from an abs-max that is already on the device (for instance the one the
 * Q8_EPI_ABSMAX epilogue of the previous layer produced): scale_out[0] = 127 / amax[0],
 * 1.0 when amax[0] is 0.  Eq. 3.
 */
q8_status q8_scale_from_amax(const float* amax, float* scale_out, void* stream);

/*
 * Eq. 1: q[i] = Clamp(round(x[i] * scale[0]), -127, 127).  The product is one
 * binary32 multiply; round is to nearest with ties away from zero; -128 is never
 * produced.
 *   x fp32[n]; scale fp32[1] on the device (dynamic from q8_absmax, or a stored
 *   constant as in Eq. 4); q int8[n]; n >= 0.
 */
q8_status q8_quantize(const float* x, int64_t n, const float* scale, int8_t* q, void* stream);

/*
 * Eq. 3 then Eq. 1 in one launch: amax[0..n_amax) hold abs-max values whose maximum is the
 * abs-max of the tensor being quantized (one value from q8_absmax or from the
 * Q8_EPI_ABSMAX epilogue, or several partial maxima).  Computes a = max_i amax[i],
 * S = 127 / a (1.0 if a is 0), writes scale_out[0] = S and, if amax_out is not NULL,
 * amax_out[0] = a, and q[i] = Clamp(round(x[i] * S), -127, 127).
 *   n >= 0; n_amax >= 1; amax_out and scale_out must not overlap amax[0..n_amax).
 */
q8_status q8_quantize_amax(const float* x, int64_t n, const float* amax, int n_amax, float* amax_out,
                           float* scale_out, int8_t* q, void* stream);

/*
 * The quantized FC layer at inference (Section 3): Int8 x Int8 GEMM accumulated in
 * Int32 onto the Int32 bias, then dequantized for the FP32 consumers.
 *     bq[n]    = Clamp(round(bias[n] * (sx * sw[g(n)])), -(2^31-1), 2^31-1)   (0 if bias is NULL)
 *     acc[m,n] = bq[n] + sum_k xq[m,k] * wq[n,k]                              (exact int32)
 *     y[m,n]   = acc[m,n] / (sx * sw[g(n)])                                   (fp32, within 1e-6 relative)
 *   xq int8[M,K], wq int8[N,K]; bias fp32[N] or NULL.
 *   sx fp32[1]: activation scale.  sw fp32[n_groups]: weight scale per column group;
 *   the N columns are split evenly, g(n) = n / (N / n_groups).  n_groups = 1 is the
 *   paper's layer; 3 packs the Q, K and V projections, each keeping its own S_W.
 *   y: fp32[M,N], or int8[M,N] with Q8_EPI_REQUANT (then next_scale fp32[1] is required).
 *   acc_out: int32[M,N] or NULL -- dump of the post-bias accumulator, for parity checks.
 *   out_amax: fp32[1], required with Q8_EPI_ABSMAX; the caller sets it to 0 beforehand
 *   (one atomic max per workgroup lands in it).
 *   Epilogue order: dequantize, GELU, abs-max, requantize.
 * M, N >= 0 (either 0: nothing is written); 0 <= K <= Q8_MAX_K; sizes are otherwise
 * free -- shapes with K % 128 == 0 and 16-byte aligned xq/wq take the MFMA kernel,
 * anything else a slower generic kernel with identical results.
 * bq + sum must fit int32 (it wraps otherwise; unreachable for BERT-sized biases).
 */
q8_status q8_linear(const int8_t* xq, const int8_t* wq, const float* bias,
                    const float* sx, const float* sw, int n_groups,
                    int64_t M, int64_t N, int64_t K,
                    void* y, int32_t* acc_out, float* out_amax, const float* next_scale,
                    uint32_t epilogue_flags, void* stream);

/*
 * q8_linear with the encoder's residual addition fused into the epilogue: the two FC layers that are followed
 * by "add the block's input, then Layer Normalization" (attention output and the second feed-forward layer;
 * both the addition and the normalization stay in FP32, Section 3) write the sum, so that the normalization
 * reads one tensor instead of two.
 *     y[m,n] = act(acc[m,n] / (sx * sw[g(n)])) + residual[m,n]        one fp32 addition, round to nearest
 *   residual fp32[M,N], same layout as y; y may be the residual tensor itself (updated in place).
 *   flags: Q8_EPI_GELU and Q8_EPI_ABSMAX (of the sum) are accepted, Q8_EPI_REQUANT is not (Q8_ERR_FLAGS).
 *   Everything else as q8_linear.  Same result as q8_linear followed by an elementwise fp32 addition.
 */
q8_status q8_linear_residual(const int8_t* xq, const int8_t* wq, const float* bias,
                             const float* sx, const float* sw, int n_groups,
                             int64_t M, int64_t N, int64_t K,
                             const float* residual, float* y, int32_t* acc_out, float* out_amax,
                             uint32_t epilogue_flags, void* stream);

/*
 * The dynamic quantizer of Section 4.1 on its own: a = max|x| over the whole tensor, S = 127 / a (Eq. 3; 1.0 when
 * a is 0), q = Quantize(x | S, 127) (Eq. 1) -- two launches (per-workgroup partial maxima, then a quantize pass
 * that folds them); one launch for tensors of at most 16384 elements, and one launch that reads x only once for
 * tensors the chip can hold in registers between the two steps (up to 12.5 M elements on 256 compute units; see
 * q8_debug_set_quantize_one_pass).  Same results as q8_absmax followed by q8_quantize in every case.
 *   x fp32[n]; q int8[n]; n >= 0 (n = 0: a = 0, S = 1).
 *   scal_work fp32[Q8_SCAL_WORK], caller-provided scratch: on return scal_work[0] = a, scal_work[1] = S (a device
 *   scalar to hand to q8_linear as sx); the rest holds the partial maxima.
 *   zero_slot fp32[1] or NULL: set to 0 by the same launch (the out_amax of a q8_linear call that follows).
 */
q8_status q8_quantize_dynamic(const float* x, int64_t n, int8_t* q, float* scal_work, float* zero_slot, void* stream);

/*
 * Dynamic-quantization FC layer in one call (Section 4.1): abs-max of x, S_x = 127/max,
 * quantize, then q8_linear.  Same results as calling the three entry points in turn.
 *   x fp32[M,K]; xq_work int8[M*K] and scal_work fp32[Q8_SCAL_WORK] are caller-provided
 *   scratch (on return scal_work[0] = max|x|, scal_work[1] = S_x, xq_work = the int8 codes;
 *   the rest of scal_work holds per-workgroup partial maxima).
 *   Other arguments as q8_linear, with one convenience: with Q8_EPI_ABSMAX this call sets
 *   out_amax[0] to 0 itself before the GEMM accumulates into it (q8_linear leaves that to the
 *   caller), so on return out_amax[0] = max|y| of this call alone.
 *   Launches: two (quantizer, GEMM) -- the quantizer is one launch whenever x has at most 16384 elements or
 *   fits the chip's registers (q8_quantize_dynamic) -- and a single one for a handful of tokens (M <= 32,
 *   M * K <= 16384, K a multiple of 128 up to 1024, 16-byte aligned x and wq, 4-byte aligned xq_work, no
 *   Q8_EPI_ABSMAX): there the layer is bound by launch latency, so every workgroup quantizes x itself and keeps
 *   the codes on chip.  Results do not depend on the path taken.
 */
q8_status q8_linear_f32(const float* x, const int8_t* wq, const float* bias,
                        const float* sw, int n_groups,
                        int64_t M, int64_t N, int64_t K,
                        int8_t* xq_work, float* scal_work,
                        void* y, int32_t* acc_out, float* out_amax, const float* next_scale,
                        uint32_t epilogue_flags, void* stream);

/*
 * q8_linear_f32 for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation and same results as
 * q8_linear_f32, bit for bit, but the scratch (the partial maxima, max|x|, S_x and the int8 codes of x) lives
 * in a static device array inside the library, 64 MiB + 16 KiB per GPU, held until the process ends.  The call
 * allocates and frees nothing (no hipMalloc, no hipFree, no allocating library routine); its first call on a
 * device looks the array's address up once.
 *   x, wq, bias, sw, n_groups, M, N, K, y, out_amax, next_scale, epilogue_flags: as q8_linear_f32.
 *   stats_out fp32[2] or NULL: receives (max|x|, S_x) of this call.
 *   M*K > Q8_STATIC_MAX_CODES returns Q8_ERR_TOO_LARGE before anything is launched.
 * Every call on a GPU shares that GPU's array and leaves its contents behind (nothing in it needs clearing
 * between calls): two calls that overlap in time on one GPU -- different streams, or different host threads --
 * race on it and must be serialised by the caller.  Calls on one stream are ordered and safe.
 */
q8_status q8_linear_f32_static(const float* x, const int8_t* wq, const float* bias,
                               const float* sw, int n_groups,
                               int64_t M, int64_t N, int64_t K,
                               void* y, float* stats_out, float* out_amax, const float* next_scale,
                               uint32_t epilogue_flags, void* stream);

/*
 * The same layer when the producer of x has already left the abs-max of x behind
 * (q8_layernorm_absmax, q8_embedding_sum3_layernorm, q8_attention, or the Q8_EPI_ABSMAX
 * epilogue of the previous layer): S_x = 127 / max(amax_slots[0 .. n_slots)) (Eq. 3 on
 * the maximum of Section 4.1), quantize, q8_linear -- two launches and no pass over x for
 * its maximum.  Same results as q8_quantize_amax followed by q8_linear.
 *   amax_slots fp32[n_slots], n_slots >= 1, non-negative values whose maximum is max|x|.
 *   scal_work fp32[2]: on return scal_work[0] = max|x|, scal_work[1] = S_x.
 *   Other arguments, and the handling of out_amax, as q8_linear_f32.
 */
q8_status q8_linear_f32_slots(const float* x, const float* amax_slots, int n_slots,
                              const int8_t* wq, const float* bias,
                              const float* sw, int n_groups,
                              int64_t M, int64_t N, int64_t K,
                              int8_t* xq_work, float* scal_work,
                              void* y, int32_t* acc_out, float* out_amax, const float* next_scale,
                              uint32_t epilogue_flags, void* stream);

/*
 * The quantized Embedding layer at inference (Section 3): returns the Int8 rows,
 * or the rows divided by the table's scale for the FP32 sum + LayerNorm that follow.
 *   table int8[V,H]; scale fp32[1] (ignored when out_is_int8); ids int32[T].
 *   out: int8[T,H] if out_is_int8, else fp32[T,H] with out[t,h] = table[ids[t],h] / scale[0].
 *   err_flag: int32[1] or NULL, zeroed by the caller.  An id outside [0,V) writes a
 *   zero row and sets err_flag[0] = 1; nothing is ever read out of bounds.
 */
q8_status q8_embedding(const int8_t* table, const float* scale, int64_t V, int64_t H,
                       const int32_t* ids, int64_t T, void* out, int out_is_int8,
                       int32_t* err_flag, void* stream);

/*
 * BERT's input embedding from three int8 tables, each with its own scale
 * (Section 3: all Embedding layers are quantized): out[t,:] =
 * (word[wid[t]]/s[0] + pos[pid[t]]/s[1]) + type[tid[t]]/s[2], fp32[T,H].
 *   scales fp32[3]; tables int8[Vw,H], int8[Vp,H], int8[Vt,H]; ids int32[T] each.
 *   Bad ids as in q8_embedding (the whole output row is zero).
 */
q8_status q8_embedding_sum3(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp,
                            const int8_t* type, int64_t Vt, const float* scales, int64_t H,
                            const int32_t* wid, const int32_t* pid, const int32_t* tid, int64_t T,
                            float* out, int32_t* err_flag, void* stream);

/*
 * ---- training side (quantization-aware training, Section 2.2) ----
 *
 * Fake quantization: xq[i] = Quantize(x[i] | scale[0], 127) / scale[0], the int8 code of
 * Eq. 1 taken straight back to fp32 (one binary32 division), so that the tensor carries the
 * rounding error of the code.  The quantized Embedding layer in training is q8_embedding with
 * fp32 output: its rows are already fake quantized values.
 *   x fp32[n]; scale fp32[1] on the device; xq fp32[n], may be x itself (in place); n >= 0.
 */
q8_status q8_fake_quantize(const float* x, int64_t n, const float* scale, float* xq, void* stream);

/*
 * One step of the exponential moving average of max|x| that Eq. 4 divides M by.
 *   amax[0..n_amax): abs-max values whose maximum a is this batch's max|x| (n_amax >= 1).
 *   decay: host float in [0, 1].  The paper prints neither the decay nor the start value:
 *   the first update (state[1] == 0) starts the average at a.
 *   state fp32[2], kept by the caller between steps and zeroed before the first:
 *     state[0] <- a                                   on the first update,
 *                 decay*state[0] + (1 - decay)*a      afterwards (each operation rounded to
 *                 binary32: the two products, the difference and the sum, in that order);
 *     state[1] <- 1.
 *   scale_out fp32[1] or NULL: 127 / state[0] (1.0 if the average is 0), Eq. 4.
 *   amax_out fp32[1] or NULL: a.  Neither may overlap amax[0..n_amax) or state.
 */
q8_status q8_ema_update(const float* amax, int n_amax, float decay, float* state, float* amax_out,
                        float* scale_out, void* stream);

/*
 * The activation quantizer of a training step in one call: abs-max of x, the moving-average
 * step above, then fake quantization with the updated scale (Eq. 4 with the average that
 * already includes this batch).  With decay = 0 the average is this tensor's own max|x|, which
 * is the weights' quantizer in training (Eq. 3).
 *   x fp32[n]; xq fp32[n], may be x; state as in q8_ema_update;
 *   scal_work fp32[Q8_SCAL_WORK]: caller-provided scratch; on return scal_work[0] = max|x|,
 *   scal_work[1] = the scale used.  n >= 0 (n = 0 counts as a batch whose max is 0).
 */
q8_status q8_fake_quantize_ema(const float* x, int64_t n, float decay, float* state, float* scal_work,
                               float* xq, void* stream);

/*
 * Eq. 5, the straight-through estimator: d xq / d x is a vector of ones, so
 * grad_x[i] = grad_xq[i].  grad_x may be grad_xq itself (then nothing is launched);
 * otherwise the two must not overlap.  n >= 0.
 */
q8_status q8_ste_backward(const float* grad_xq, int64_t n, float* grad_x, void* stream);

/*
 * ---- FP32 glue fused with the next layer's quantizer ----
 *
 * Layer Normalization over the last dimension (Section 3: Softmax, Layer Normalization and
 * GELU are kept in FP32), with the residual addition in front of it and, behind it, the first
 * half of the dynamic quantizer of the FC layer that consumes its output (Section 4.1: the
 * abs-max of each incoming activation tensor):
 *     x[m,:] = a[m,:] (+ residual[m,:], one binary32 addition)
 *     y[m,h] = (x[m,h] - mean_m) / sqrt(var_m + eps) * gamma[h] + beta[h]      (biased variance)
 *     amax_slots[0..Q8_AMAX_SLOTS) = partial maxima of |y| whose maximum is max|y|; pass them to
 *     q8_quantize_amax(y, ..., amax_slots, Q8_AMAX_SLOTS, ...) and no abs-max pass is needed.
 *   a fp32[M,H]; residual fp32[M,H] or NULL; gamma, beta fp32[H]; eps host float (BERT: 1e-12).
 *   y fp32[M,H], may be a itself (in place); amax_slots fp32[Q8_AMAX_SLOTS] or NULL.
 *   q_scale fp32[1] and q_out int8[M,H], both or neither: with a stored activation scale (Eq. 4)
 *   the same pass also writes q_out = Quantize(y | q_scale[0], 127) (Eq. 1 on the fp32 y it
 *   stores), i.e. the next FC layer's whole quantizer; y is still written for the FP32 consumers
 *   (the residual path).
 *   Statistics and normalisation are evaluated in binary64 and rounded once: y is within one
 *   ulp of the exact value.  M >= 0 (M = 0: every slot 0); H >= 1.  Rows with H % 4 == 0,
 *   H <= 2048 and 16-byte aligned pointers stay in registers; others take a slower kernel with
 *   the same results.
 */
q8_status q8_layernorm_absmax(const float* a, const float* residual, const float* gamma, const float* beta,
                              float eps, int64_t M, int64_t H, float* y, float* amax_slots,
                              const float* q_scale, int8_t* q_out, void* stream);

/*
 * BERT's input block in one pass: the three-table int8 embedding lookup of q8_embedding_sum3
 * (Section 3), Layer Normalization of the summed rows, and the abs-max slots of the result as
 * above.  Arguments as q8_embedding_sum3 and q8_layernorm_absmax.  A token with an id outside
 * its table counts as an all-zero row (its output row is beta) and sets err_flag[0] = 1.
 */
q8_status q8_embedding_sum3_layernorm(const int8_t* word, int64_t Vw, const int8_t* pos, int64_t Vp,
                                      const int8_t* type, int64_t Vt, const float* scales, int64_t H,
                                      const int32_t* wid, const int32_t* pid, const int32_t* tid, int64_t T,
                                      const float* gamma, const float* beta, float eps,
                                      float* y, float* amax_slots, const float* q_scale, int8_t* q_out,
                                      int32_t* err_flag, void* stream);

/*
 * Multi-head softmax attention in FP32 (Section 3: Softmax is kept in FP32, and only Embedding
 * and FC layers are quantized, so the two matrix products around it stay FP32 too) -- the
 * operation between the fused Q|K|V FC layer and the attention-output FC layer -- with the
 * first half of that next layer's quantizer behind it, as in q8_layernorm_absmax:
 *     s[i,j]   = scale * sum_c Q[i,c] K[j,c]  (+ mask[b,j])        i, j tokens of sequence b
 *     p[i,:]   = softmax over j of s[i,:]
 *     ctx[i,c] = sum_j p[i,j] V[j,c]
 *   qkv fp32[B*S, 3*heads*d]: the output of q8_linear(_f32) with n_groups = 3 -- columns
 *   [0, heads*d) hold Q, the next heads*d hold K, the last heads*d hold V; head h owns columns
 *   h*d .. h*d+d-1 of each.  B sequences of S tokens, rows in sequence order.
 *   mask fp32[B,S] or NULL: added to the scores of key j (BERT: 0, or -10000 for padding).
 *   scale host float > 0 (BERT: 1/sqrt(d)).
 *   ctx fp32[B*S, heads*d], or NULL when only the codes are wanted.
 *   amax_slots fp32[Q8_AMAX_SLOTS] or NULL: partial maxima of |ctx| for q8_quantize_amax.
 *   q_scale fp32[1] and q_out int8[B*S, heads*d], both or neither: q_out = Quantize(ctx | q_scale[0], 127)
 *   (Eq. 1 on the fp32 value), the whole quantizer of the next FC layer under a stored scale (Eq. 4).
 * Arithmetic is binary32 throughout (fp32 matrix pipes, running-maximum softmax, exp2): ctx agrees
 * with the exact result to about 1e-6 of the largest |V| of its head as long as the scores stay
 * within a few tens; a sequence whose every key carries a large negative mask loses the low bits of
 * its scores to that offset.  Inputs must be finite.
 * B >= 0 (B = 0: nothing written, slots cleared); S >= 1; heads, d >= 1.  d = 64 with 16-byte
 * aligned qkv and ctx (4-byte q_out) and one sequence of qkv below 2^31 floats takes the MFMA
 * kernel; other widths or alignments take a slower kernel that needs S <= 16384 (Q8_ERR_SHAPE
 * beyond).  The softmax runs on a running reference maximum (any S; scores never stored).
 */
q8_status q8_attention(const float* qkv, int64_t B, int64_t S, int heads, int d,
                       const float* mask, float scale, float* ctx, float* amax_slots,
                       const float* q_scale, int8_t* q_out, void* stream);

/*
 * ---- tuning / debugging (not part of the method) ----
 *
 * Forces the tile shape of the MFMA GEMM behind q8_linear for every later call of this process:
 * 0 = automatic choice from the shape (the default), 1..6 = one fixed tile variant (tests and
 * tile sweeps use it to run every variant on every shape).  Process-global and unsynchronised: set it
 * while no other thread is inside q8_linear.  An unknown variant makes q8_linear return Q8_ERR_LAUNCH.
 */
void q8_debug_set_gemm_variant(int variant);

/*
 * The dynamic quantizer (q8_quantize_dynamic, q8_linear_f32, q8_linear_f32_static) takes a one-pass kernel for
 * tensors that fit the register files of the chip: 4-element multiples of n between 4096 and 49152 floats per
 * compute unit, x 16-byte aligned, stream not under graph capture.  Its workgroups meet at a barrier; one that has
 * polled `barrier_polls` times (default 64, about 80 us) stops waiting and reads the shares of the absent
 * workgroups itself, so the result never depends on the wait.  enabled = 0 turns the kernel off (two passes over
 * x, same results); barrier_polls = 0 makes a workgroup scan for every other one that is not there at its first
 * look (tests).  Process-global, unsynchronised.
 */
void q8_debug_set_quantize_one_pass(int enabled, uint32_t barrier_polls);

/*
 * Measurement kernels for the benchmark: what the chip sustains next to the library's own kernels.
 * q8_debug_mfma_rate: `workgroups` workgroups of 8 waves, every wave running iters x 8 independent
 *   v_mfma_i32_32x32x32_i8 on operand fragments read once from `operands` (int8[65536], 16-byte aligned; their bit
 *   pattern decides the clock the chip holds): 2 * 32*32*32 * 8 * iters * 8 * workgroups int8 operations, no
 *   memory traffic.  sink int32[1] is never written in practice.
 * q8_debug_stream_copy: dst[0..nbytes) = src[0..nbytes) (src NULL: dst is filled instead), one 16-byte vector per
 *   thread and many small workgroups in address order -- the shape that moves the most bytes on this part;
 *   nbytes a multiple of 16 (at most 2^41), pointers 16-byte aligned.
 */
q8_status q8_debug_mfma_rate(const int8_t* operands, int iters, int workgroups, int32_t* sink, void* stream);
q8_status q8_debug_stream_copy(const void* src, void* dst, int64_t nbytes, void* stream);
/*
 * q8_debug_loop_probe: one stage of a GEMM main loop, piece by piece -- 256 workgroups of 8 waves run `stages` stages of 16
 * MFMAs per wave (a 256 x 128 tile in 128-byte K stages) on zero operands, plus what `what` adds (a sum of: 1 the
 * fragment reads from LDS, 2 the stage barrier, 4 the stage's 48 KiB of global -> LDS loads, 8 eight dword stores per
 * wave -- 16 KiB per workgroup, the fp32 output of a K = 1024 tile spread over its stages --, 64 eight GELU evaluations
 * per wave; accepted: 0, 7, 15, 64, 71, 79).  Shows which part of a kernel's structure costs what, with the clock
 * unaffected by operand toggling.  operand_window: 4 MiB to load from; store_window: 32 MiB to store into (both
 * device, 16-byte aligned, contents irrelevant).
 */
q8_status q8_debug_loop_probe(int what, const void* operand_window, float* store_window, int stages, int32_t* sink, void* stream);

/* Library version string and a short text for a status code (host pointers, static storage). */
const char* q8_version(void);
const char* q8_status_str(q8_status s);

#ifdef __cplusplus
}
#endif
#endif /* Q8_H */

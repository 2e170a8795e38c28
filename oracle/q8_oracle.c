/*
 * q8 CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar implementation of the symmetric linear int8 quantized
 * fully-connected layer and int8 embedding lookup of Q8BERT (arxiv 1910.06188),
 * written from the paper's equations.  It exists to check the HIP kernels and is
 * never part of the product path: only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may build or call it.  It shares no source,
 * header, table or helper with the GPU library.
 *
 * Arithmetic conventions (the paper's evaluation ran in FP32, Section 3):
 *   - scales, products x*S and the rounding decision are IEEE-754 binary32,
 *     each operation rounded separately (build with -ffp-contract=off, never
 *     -ffast-math);
 *   - the rounding bracket of Eq. 1 is round-to-nearest with ties away from zero;
 *   - integer accumulation is exact (checked against the int32 range);
 *   - dequantisation and GELU are evaluated in binary64 and rounded once to
 *     binary32.
 *
 * Pins (see tests/test_oracle_*.py): hand-worked rounding/clamp/bias cases,
 * an independent float64 NumPy formulation of Eq. 1, exact int64 NumPy matmul,
 * Python-integer brute force on tiny shapes, int32-exactness stress values,
 * a closed form for constant tensors, and the deterministic half-step error
 * bound against the dense fp64 product; for the training-side operations hand
 * values, the grid/half-step properties of fake quantization and closed forms of
 * the moving average; for Layer Normalization a hand case, the library routine in
 * binary64 and its invariants.  Parity unpinned: the decay and start value of the moving
 * average under Eq. 4 (the paper prints neither; they are arguments).
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#define Q8O_OK 0
#define Q8O_ERR_NONFINITE 1 /* NaN/Inf input or non-finite scale: outside the method's domain */
#define Q8O_ERR_OVERFLOW 2  /* an accumulator left the int32 range */
#define Q8O_ERR_INDEX 3     /* embedding id outside [0, V) */
#define Q8O_ERR_SHAPE 4

/* Eq. 2: M = 2^(b-1) - 1. */
static double top_value(int bits) { return ldexp(1.0, bits - 1) - 1.0; }

/* max |x_i| over the whole tensor: the denominator of Eq. 3, which Section 4.1
 * (dynamic quantization) also applies to every incoming activation tensor. */
int q8o_absmax(const float *x, int64_t n, float *amax_out)
{
    float a = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        if (!isfinite(x[i])) return Q8O_ERR_NONFINITE;
        float v = fabsf(x[i]);
        if (v > a) a = v;
    }
    *amax_out = a;
    return Q8O_OK;
}

/* Eq. 3 with M = 127 (Eq. 2, b = 8): S = M / max|.|, one binary32 division.
 * An all-zero tensor has no defined scale in the paper; S = 1 is used so that
 * every code is 0. */
int q8o_scale(float amax, float *scale_out)
{
    float m = (float)top_value(8);
    float s = (amax == 0.0f) ? 1.0f : m / amax;
    if (!isfinite(s)) return Q8O_ERR_NONFINITE;
    *scale_out = s;
    return Q8O_OK;
}

/* The bracket of Eq. 1 on a binary32 value: nearest integer, ties away from zero.
 * t is p with its fraction dropped; p - t is exact in binary32. */
static float round_half_away(float p)
{
    float t = truncf(p);
    float frac = p - t;
    if (fabsf(frac) >= 0.5f) t += (p < 0.0f) ? -1.0f : 1.0f;
    return t;
}

/* Eq. 1: Quantize(x | S, M) = Clamp(round(x * S), -M, M), M = 127. */
int q8o_quantize(const float *x, int64_t n, float scale, int8_t *q)
{
    const float m = (float)top_value(8);
    if (!isfinite(scale)) return Q8O_ERR_NONFINITE;
    for (int64_t i = 0; i < n; ++i) {
        if (!isfinite(x[i])) return Q8O_ERR_NONFINITE;
        float p = x[i] * scale;
        float r = round_half_away(p);
        r = fminf(fmaxf(r, -m), m); /* Clamp(x,a,b) = min(max(x,a),b) */
        q[i] = (int8_t)r;
    }
    return Q8O_OK;
}

/* Section 3: the bias is quantized to Int32 with the product of the activation
 * and weight scaling-factors; Eq. 1 with Eq. 2 at b = 32 gives the clamp.
 * sw holds n_groups weight scales; output columns are split evenly over groups. */
int q8o_quantize_bias(const float *b, int64_t n, float sx, const float *sw, int n_groups, int32_t *bq)
{
    if (n_groups < 1 || n % n_groups != 0) return Q8O_ERR_SHAPE;
    const double m32 = top_value(32); /* 2147483647 */
    const int64_t per = n / n_groups;
    for (int64_t j = 0; j < n; ++j) {
        if (b == NULL) { bq[j] = 0; continue; }
        float sb = sx * sw[j / per];
        if (!isfinite(b[j]) || !isfinite(sb)) return Q8O_ERR_NONFINITE;
        float p = b[j] * sb;
        double r = (double)round_half_away(p);
        if (r > m32) r = m32;
        if (r < -m32) r = -m32;
        bq[j] = (int32_t)r;
    }
    return Q8O_OK;
}

/* Section 3, inference: GEMM between Int8 inputs and Int8 weights accumulated
 * onto the Int32 bias.  x is [M,K], w is [N,K] (y = x w^T), both row-major.
 * The sum is formed in int64 and must fit int32. */
int q8o_gemm_i8(const int8_t *xq, const int8_t *wq, const int32_t *bq,
                int64_t M, int64_t N, int64_t K, int32_t *acc, int threads)
{
    int status = Q8O_OK;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = bq ? (int64_t)bq[n] : 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)xq[m * K + k] * (int64_t)wq[n * K + k];
            if (s > INT32_MAX || s < INT32_MIN) {
#pragma omp atomic write
                status = Q8O_ERR_OVERFLOW;
                s = 0;
            }
            acc[m * N + n] = (int32_t)s;
        }
    }
    return status;
}

/* The FP32 consumers of Section 3 (Softmax, LayerNorm, GELU) need real values
 * back: acc represents y * S_x * S_W, so y = acc / (S_x * S_W). */
int q8o_dequant(const int32_t *acc, int64_t M, int64_t N, float sx, const float *sw, int n_groups, float *y)
{
    if (n_groups < 1 || N % n_groups != 0) return Q8O_ERR_SHAPE;
    const int64_t per = N / n_groups;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = (double)sx * (double)sw[n / per];
            y[m * N + n] = (float)((double)acc[m * N + n] / s);
        }
    return Q8O_OK;
}

/* GELU stays in floating point (Section 3).  Exact-erf form, written with erfc
 * so the negative tail does not cancel: gelu(v) = v * Phi(v) = 0.5 v erfc(-v/sqrt 2). */
void q8o_gelu(const float *v, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        double d = (double)v[i];
        out[i] = (float)(0.5 * d * erfc(-d / sqrt(2.0)));
    }
}

/* Section 3, inference: the quantized Embedding layer returns Int8 embedding
 * vectors; dividing by the table's scale gives the FP32 rows LayerNorm consumes.
 * Either output may be NULL. */
int q8o_embedding(const int8_t *table, int64_t V, int64_t H, float scale,
                  const int32_t *ids, int64_t T, int8_t *out_i8, float *out_f32)
{
    for (int64_t t = 0; t < T; ++t) {
        int64_t id = ids[t];
        if (id < 0 || id >= V) return Q8O_ERR_INDEX;
        for (int64_t h = 0; h < H; ++h) {
            int8_t q = table[id * H + h];
            if (out_i8) out_i8[t * H + h] = q;
            if (out_f32) out_f32[t * H + h] = (float)((double)q / (double)scale);
        }
    }
    return Q8O_OK;
}

/* BERT's input embedding: word + position + token-type rows, each table with
 * its own scale, summed in the order (word + position) + type. */
int q8o_embedding_sum3(const int8_t *word, int64_t Vw, float sw_,
                       const int8_t *pos, int64_t Vp, float sp,
                       const int8_t *typ, int64_t Vt, float st,
                       int64_t H, const int32_t *wid, const int32_t *pid, const int32_t *tid,
                       int64_t T, float *out)
{
    for (int64_t t = 0; t < T; ++t) {
        int64_t a = wid[t], b = pid[t], c = tid[t];
        if (a < 0 || a >= Vw || b < 0 || b >= Vp || c < 0 || c >= Vt) return Q8O_ERR_INDEX;
        for (int64_t h = 0; h < H; ++h) {
            double s = ((double)word[a * H + h] / (double)sw_ + (double)pos[b * H + h] / (double)sp)
                       + (double)typ[c * H + h] / (double)st;
            out[t * H + h] = (float)s;
        }
    }
    return Q8O_OK;
}

/* ---- training-side operations (Section 2.2; Eq. 4; Eq. 5) ------------------------------ */

/* Fake quantization (Section 2.2): the value is quantized with Eq. 1 and taken straight back
 * to floating point, x^q = Quantize(x | S, 127) / S, so that the fp32 tensor carries the
 * rounding error of the int8 code.  One binary32 division per element. */
int q8o_fake_quantize(const float *x, int64_t n, float scale, float *xq)
{
    const float m = (float)top_value(8);
    if (!isfinite(scale) || scale == 0.0f) return Q8O_ERR_NONFINITE;
    for (int64_t i = 0; i < n; ++i) {
        if (!isfinite(x[i])) return Q8O_ERR_NONFINITE;
        float p = x[i] * scale;
        float r = round_half_away(p);
        r = fminf(fmaxf(r, -m), m);
        xq[i] = r / scale;
    }
    return Q8O_OK;
}

/* The running statistic under Eq. 4: an exponential moving average of max|x| over the
 * batches seen in training.  The paper prints neither the decay nor the start value; both are
 * arguments here (the first batch starts the average at its own max|x|):
 *     ema <- decay * ema + (1 - decay) * amax,
 * four binary32 operations, each rounded, in exactly this order. */
int q8o_ema_update(float ema_prev, int initialized, float amax, float decay, float *ema_out)
{
    if (!isfinite(amax) || !isfinite(ema_prev) || !(decay >= 0.0f && decay <= 1.0f)) return Q8O_ERR_NONFINITE;
    if (!initialized) {
        *ema_out = amax;
        return Q8O_OK;
    }
    float keep = decay * ema_prev;
    float w = 1.0f - decay;
    float take = w * amax;
    *ema_out = keep + take;
    return Q8O_OK;
}

/* Eq. 5, the straight-through estimator: the derivative of the fake-quantized value with
 * respect to its input is a vector of ones, so the gradient passes unchanged. */
void q8o_ste_backward(const float *grad_xq, int64_t n, float *grad_x)
{
    for (int64_t i = 0; i < n; ++i) grad_x[i] = grad_xq[i] * 1.0f;
}

/* ---- FP32 glue around the FC layers (Section 3: Layer Normalization is kept in FP32) ------- */

/* Layer Normalization over the last dimension of x[M,H], x = a (+ r when a residual is given,
 * one binary32 addition): y = (x - mean) / sqrt(var + eps) * gamma + beta with the biased
 * variance (1/H), as in BERT.  Statistics and the normalisation are evaluated in binary64 and
 * the result is rounded once to binary32.  The paper only says that the operation stays in
 * FP32; the formula is the standard one (Ba et al. 2016). */
int q8o_layernorm(const float *a, const float *r, const float *gamma, const float *beta, double eps,
                  int64_t M, int64_t H, float *y)
{
    if (M < 0 || H <= 0) return Q8O_ERR_SHAPE;
    for (int64_t m = 0; m < M; ++m) {
        const float *pa = a + m * H, *pr = r ? r + m * H : NULL;
        double sum = 0.0;
        for (int64_t h = 0; h < H; ++h) {
            float x = pr ? pa[h] + pr[h] : pa[h];
            if (!isfinite(x)) return Q8O_ERR_NONFINITE;
            sum += (double)x;
        }
        double mean = sum / (double)H, ss = 0.0;
        for (int64_t h = 0; h < H; ++h) {
            float x = pr ? pa[h] + pr[h] : pa[h];
            double d = (double)x - mean;
            ss += d * d;
        }
        double rstd = 1.0 / sqrt(ss / (double)H + eps);
        for (int64_t h = 0; h < H; ++h) {
            float x = pr ? pa[h] + pr[h] : pa[h];
            y[m * H + h] = (float)(((double)x - mean) * rstd * (double)gamma[h] + (double)beta[h]);
        }
    }
    return Q8O_OK;
}

/* Multi-head scaled dot-product attention of one encoder layer, the FP32 operation that sits
 * between the fused Q|K|V projection and the attention-output FC layer (Section 3: Softmax is
 * kept in FP32; the two matrix products around it are not FC layers, so they are not quantized
 * either).  The paper takes the operation from BERT without printing it; this is the standard
 * definition (Vaswani et al. 2017), written out:
 *     s[i,j]   = scale * sum_c Q[i,c] K[j,c]  (+ mask[b,j])
 *     p[i,:]   = softmax over j of s[i,:]
 *     ctx[i,c] = sum_j p[i,j] V[j,c]
 * qkv is the projection's output, fp32 [B*S, 3*heads*d]: columns [0, heads*d) hold Q,
 * the next heads*d hold K, the last heads*d hold V; head h owns columns h*d .. h*d+d-1 of each.
 * mask (or NULL) is additive, fp32 [B,S], one value per key position (BERT: 0 or -10000).
 * ctx is fp32 [B*S, heads*d].  Everything is evaluated in binary64 and rounded once. */
int q8o_attention(const float *qkv, int64_t B, int64_t S, int64_t heads, int64_t d, const float *mask,
                  double scale, float *ctx, int threads)
{
    if (B < 0 || S < 1 || heads < 1 || d < 1) return Q8O_ERR_SHAPE;
    const int64_t HD = heads * d, ld = 3 * HD;
    for (int64_t i = 0; i < B * S * ld; ++i)
        if (!isfinite(qkv[i])) return Q8O_ERR_NONFINITE;
    if (mask)
        for (int64_t i = 0; i < B * S; ++i)
            if (!isfinite(mask[i])) return Q8O_ERR_NONFINITE;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t bh = 0; bh < B * heads; ++bh) {
        const int64_t b = bh / heads, h = bh % heads;
        double *s = (double *)malloc((size_t)S * sizeof(double));
        for (int64_t i = 0; i < S; ++i) {
            const float *q = qkv + (b * S + i) * ld + h * d;
            double top = -INFINITY;
            for (int64_t j = 0; j < S; ++j) {
                const float *k = qkv + (b * S + j) * ld + HD + h * d;
                double dot = 0.0;
                for (int64_t c = 0; c < d; ++c) dot += (double)q[c] * (double)k[c];
                s[j] = scale * dot + (mask ? (double)mask[b * S + j] : 0.0);
                if (s[j] > top) top = s[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j < S; ++j) {
                s[j] = exp(s[j] - top);
                den += s[j];
            }
            for (int64_t c = 0; c < d; ++c) {
                double o = 0.0;
                for (int64_t j = 0; j < S; ++j) o += s[j] * (double)qkv[(b * S + j) * ld + 2 * HD + h * d + c];
                ctx[(b * S + i) * HD + h * d + c] = (float)(o / den);
            }
        }
        free(s);
    }
    return Q8O_OK;
}

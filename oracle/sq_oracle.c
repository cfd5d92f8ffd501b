/*
 * SmoothQuant W8A8 hot path -- CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.
 *
 * Every function follows the paper's equations step by step, in IEEE fp32
 * with round-to-nearest-even and no fused multiply-add (build with
 * -ffp-contract=off, never -ffast-math), because the bit-exact gate on int8
 * codes requires both sides to take the rounding decision in one precision.
 * Integer contractions are exact triple loops in int32.
 *
 * Paper passages followed:
 *   Eq. 1  (Sec. 2)  symmetric absmax quantizer, Delta = max|X| / (2^(N-1)-1)
 *   Eq. 2  (Sec. 3)  Y = diag(Delta_X) (Xq Wq) diag(Delta_W), outer-dim scaling
 *   Eq. 3  (Sec. 4)  Y = (X diag(s)^-1)(diag(s) W)
 *   Eq. 4  (Sec. 4)  s_j = max|X_j|^alpha / max|W_j|^(1-alpha)
 *   Table 2          O1 per-token dynamic / O2 per-tensor dynamic / O3 static
 *   Sec. 4 "Applying ... to Transformer blocks": INT8 BMMs, FP16 softmax / LN
 *
 * Readings taken where the paper is silent (also listed in the design notes):
 *   - rounding function of Eq. 1 = round-half-to-even;
 *   - X/Delta is evaluated as X * r with r = fl32(127 / absmax) computed once
 *     per token (or tensor); static mode uses r = fl32(1 / Delta);
 *   - codes live in [-127, 127]; static mode saturates;
 *   - an all-zero row/tensor gives Delta = 0, r = 0, codes 0;
 *   - Eq. 4 clamps both maxima to 1e-5 from below;
 *   - max|W_j| runs over row j of W[C_i, C_o] (the j-th input channel);
 *   - all scales are kept in fp32, only the final output is 16-bit.
 *
 * dtype codes: 0 = IEEE fp16, 1 = bfloat16 (both passed as raw uint16 bits).
 * Return value: 0 on success, non-zero on invalid arguments.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_F16 0
#define ORC_BF16 1
#define ORC_PER_TOKEN_DYNAMIC 0
#define ORC_PER_TENSOR_DYNAMIC 1
#define ORC_PER_TENSOR_STATIC 2

/* ---------------------------------------------------------------- 16-bit formats */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* IEEE binary16 -> binary32, exact. */
float orc_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t m = h & 0x3ffu;
    if (e == 0) {
        if (m == 0) return bits_to_f32(sign);
        /* subnormal: value = m * 2^-24, exactly representable in fp32 */
        float v = (float)m * 5.9604644775390625e-08f;
        return sign ? -v : v;
    }
    if (e == 31) return bits_to_f32(sign | 0x7f800000u | (m << 13));
    return bits_to_f32(sign | ((e + 112u) << 23) | (m << 13));
}

/* binary32 -> binary16, round-to-nearest-even, overflow to infinity. */
uint16_t orc_f2h(float f)
{
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u) /* inf / nan */
        return (uint16_t)(sign | 0x7c00u | ((a > 0x7f800000u) ? 0x200u : 0u));
    if (a >= 0x477ff000u) /* >= 65520 rounds to infinity */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x33000001u) /* <= 2^-25: rounds to zero (tie at 2^-25 goes to even = 0) */
        return sign;
    int32_t e = (int32_t)(a >> 23) - 127;
    uint32_t m = (a & 0x7fffffu) | 0x800000u; /* 24-bit significand */
    int shift;                                /* bits to drop */
    uint32_t base;
    if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; }
    else          { shift = 13 + (-14 - e); base = 0; }
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept++;
    /* for normals "kept" carries the implicit bit (0x400): adding base-0x400 merges it,
       and a carry out of the mantissa correctly bumps the exponent. */
    uint32_t out = (e >= -14) ? (base - 0x400u + kept) : kept;
    return (uint16_t)(sign | out);
}

float orc_bf2f(uint16_t b) { return bits_to_f32((uint32_t)b << 16); }

/* binary32 -> bfloat16, round-to-nearest-even. */
uint16_t orc_f2bf(float f)
{
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u); /* quiet nan */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static float load16(const uint16_t* p, int dtype) { return dtype == ORC_BF16 ? orc_bf2f(*p) : orc_h2f(*p); }
static uint16_t store16(float v, int dtype) { return dtype == ORC_BF16 ? orc_f2bf(v) : orc_f2h(v); }

/* Eq. 1 rounding + range: round-half-even, then saturate to [-127, 127]. */
static int8_t round_code(float v)
{
    float r = rintf(v); /* default rounding mode = nearest-even */
    if (r > 127.0f) r = 127.0f;
    if (r < -127.0f) r = -127.0f;
    return (int8_t)(int)r;
}

/* ---------------------------------------------------------------- Eq. 4 */

/* s_j = max|X_j|^alpha / max|W_j|^(1-alpha), powers in fp64, result rounded to fp32;
   inv_s_j = fl32(1 / s_j).  inv_s may be NULL. */
int orc_smooth_scales(const float* x_absmax, const float* w_absmax, float alpha, int64_t c_i,
                      float* s, float* inv_s)
{
    if (!x_absmax || !w_absmax || !s || c_i <= 0) return 1;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return 4;
    for (int64_t j = 0; j < c_i; ++j) {
        double ax = x_absmax[j] > 1e-5f ? (double)x_absmax[j] : (double)1e-5f;
        double aw = w_absmax[j] > 1e-5f ? (double)w_absmax[j] : (double)1e-5f;
        double sj = pow(ax, (double)alpha) / pow(aw, 1.0 - (double)alpha);
        s[j] = (float)sj;
        if (inv_s) inv_s[j] = 1.0f / s[j];
    }
    return 0;
}

/* max over calibration tokens of |X_tj|: fp32 [c_i]. */
int orc_act_absmax_per_channel(const uint16_t* x, int dtype, int64_t t, int64_t c_i, float* out)
{
    if (!x || !out || t <= 0 || c_i <= 0) return 1;
    for (int64_t j = 0; j < c_i; ++j) out[j] = 0.0f;
    for (int64_t i = 0; i < t; ++i)
        for (int64_t j = 0; j < c_i; ++j) {
            float v = fabsf(load16(x + i * c_i + j, dtype));
            if (v > out[j]) out[j] = v;
        }
    return 0;
}

/* max|W_j| over the output channels of input channel j; W is [c_i, c_o] row-major. */
int orc_weight_absmax_per_in_channel(const uint16_t* w, int dtype, int64_t c_i, int64_t c_o, float* out)
{
    if (!w || !out || c_i <= 0 || c_o <= 0) return 1;
    for (int64_t j = 0; j < c_i; ++j) {
        float m = 0.0f;
        for (int64_t n = 0; n < c_o; ++n) {
            float v = fabsf(load16(w + j * c_o + n, dtype));
            if (v > m) m = v;
        }
        out[j] = m;
    }
    return 0;
}

/* ---------------------------------------------------------------- Eq. 3 + Eq. 1 on W */

/* W_hat = diag(s) W (s == NULL means s = 1); Delta_W = max|W_hat| / 127 (per tensor);
   Wq = round(W_hat * (127 / max|W_hat|)), written transposed as [c_o, c_i]. */
int orc_prepare_weight(const uint16_t* w, int dtype, const float* s, int64_t c_i, int64_t c_o,
                       int8_t* wq, float* w_scale)
{
    if (!w || !wq || !w_scale || c_i <= 0 || c_o <= 0) return 1;
    float a = 0.0f;
    for (int64_t j = 0; j < c_i; ++j)
        for (int64_t n = 0; n < c_o; ++n) {
            float v = load16(w + j * c_o + n, dtype);
            if (s) v = v * s[j];
            v = fabsf(v);
            if (v > a) a = v;
        }
    float delta = a / 127.0f;
    float r = a > 0.0f ? 127.0f / a : 0.0f;
    *w_scale = delta;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < c_o; ++n)
        for (int64_t j = 0; j < c_i; ++j) {
            float v = load16(w + j * c_o + n, dtype);
            if (s) v = v * s[j];
            wq[n * c_i + j] = round_code(v * r);
        }
    return 0;
}

/* Per-output-channel weight quantization (the weight granularity of Table 7): one step per column n of
   W_hat [c_i, c_o], Delta_W[n] = max_j |W_hat[j, n]| / 127, Wq[n, j] = round(W_hat[j, n] * (127 / max_j|W_hat[j, n]|)).
   A column of zeros gets step 0 and codes 0. */
int orc_prepare_weight_per_channel(const uint16_t* w, int dtype, const float* s, int64_t c_i, int64_t c_o,
                                   int8_t* wq, float* w_scale)
{
    if (!w || !wq || !w_scale || c_i <= 0 || c_o <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < c_o; ++n) {
        float a = 0.0f;
        for (int64_t j = 0; j < c_i; ++j) {
            float v = load16(w + j * c_o + n, dtype);
            if (s) v = v * s[j];
            v = fabsf(v);
            if (v > a) a = v;
        }
        w_scale[n] = a / 127.0f;
        float r = a > 0.0f ? 127.0f / a : 0.0f;
        for (int64_t j = 0; j < c_i; ++j) {
            float v = load16(w + j * c_o + n, dtype);
            if (s) v = v * s[j];
            wq[n * c_i + j] = round_code(v * r);
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- Eq. 1 on activations */

static float smoothed(const uint16_t* x, int dtype, const float* inv_s, int64_t j)
{
    float v = load16(x, dtype);
    if (inv_s) v = v * inv_s[j];
    return v;
}

/* x: [t, c_i] with row stride ldx (elements).  inv_s: fp32 [c_i] or NULL.
   mode 0: scale[t] written, one Delta per token.
   mode 1: scale[1] written, one Delta for the tensor.
   mode 2: scale[1] read (calibrated Delta), codes saturate. */
int orc_quantize_act(const uint16_t* x, int dtype, int64_t t, int64_t c_i, int64_t ldx,
                     const float* inv_s, int mode, float* scale, int8_t* xq)
{
    if (!x || !scale || !xq) return 1;
    if (t <= 0 || c_i <= 0 || ldx < c_i) return 2;
    if (mode == ORC_PER_TOKEN_DYNAMIC) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < t; ++i) {
            const uint16_t* row = x + i * ldx;
            float a = 0.0f;
            for (int64_t j = 0; j < c_i; ++j) {
                float v = fabsf(smoothed(row + j, dtype, inv_s, j));
                if (v > a) a = v;
            }
            float delta = a / 127.0f;
            float r = a > 0.0f ? 127.0f / a : 0.0f;
            scale[i] = delta;
            for (int64_t j = 0; j < c_i; ++j)
                xq[i * c_i + j] = round_code(smoothed(row + j, dtype, inv_s, j) * r);
        }
        return 0;
    }
    float r;
    if (mode == ORC_PER_TENSOR_DYNAMIC) {
        float a = 0.0f;
        for (int64_t i = 0; i < t; ++i)
            for (int64_t j = 0; j < c_i; ++j) {
                float v = fabsf(smoothed(x + i * ldx + j, dtype, inv_s, j));
                if (v > a) a = v;
            }
        scale[0] = a / 127.0f;
        r = a > 0.0f ? 127.0f / a : 0.0f;
    } else if (mode == ORC_PER_TENSOR_STATIC) {
        float delta = scale[0];
        r = delta > 0.0f ? 1.0f / delta : 0.0f;
    } else {
        return 4;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i)
        for (int64_t j = 0; j < c_i; ++j)
            xq[i * c_i + j] = round_code(smoothed(x + i * ldx + j, dtype, inv_s, j) * r);
    return 0;
}

/* ---------------------------------------------------------------- Eq. 2 */

/* acc_tn = sum_j xq[t, j] * wq[n, j]; xq [t, c_i], wq [c_o, c_i] (both K-contiguous). */
int orc_i8_gemm_i32(const int8_t* xq, const int8_t* wq, int32_t* acc, int64_t t, int64_t c_i, int64_t c_o)
{
    if (!xq || !wq || !acc) return 1;
    if (t <= 0 || c_i <= 0 || c_o <= 0) return 2;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t i = 0; i < t; ++i)
        for (int64_t n = 0; n < c_o; ++n) {
            int32_t sum = 0;
            for (int64_t j = 0; j < c_i; ++j) sum += (int32_t)xq[i * c_i + j] * (int32_t)wq[n * c_i + j];
            acc[i * c_o + n] = sum;
        }
    return 0;
}

/* The dequantizing epilogue for one accumulator.
   c = fl32(Delta_x * Delta_w); v = fl32(float(acc) * c); + bias; ReLU; + residual; round to 16 bit. */
static uint16_t epilogue(int32_t acc, float c, const float* bias, int64_t n, int relu,
                         const uint16_t* residual, int64_t idx, int out_dtype)
{
    float v = (float)acc * c;
    if (bias) v = v + bias[n];
    if (relu) v = v > 0.0f ? v : 0.0f;
    if (residual) v = v + load16(residual + idx, out_dtype);
    return store16(v, out_dtype);
}

/* Rows [row0, row0 + nrows) of Y = diag(Delta_x) (Xq Wq^T) Delta_w (+bias)(ReLU)(+residual).
   xq / x_scale / residual / y are indexed by absolute row; a row subset lets the tests sample
   rows of a full-size problem.  x_scale has t entries if per_token else 1.  w_scale has c_o
   entries if w_per_channel else 1. */
int orc_w8a8_linear_rows(const int8_t* xq, const float* x_scale, int per_token, const int8_t* wq,
                         const float* w_scale, int w_per_channel, const float* bias,
                         const uint16_t* residual, int relu, uint16_t* y, int out_dtype,
                         int64_t t, int64_t c_i, int64_t c_o, const int64_t* rows, int64_t nrows)
{
    if (!xq || !x_scale || !wq || !w_scale || !y) return 1;
    if (t <= 0 || c_i <= 0 || c_o <= 0) return 2;
    int64_t count = rows ? nrows : t;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t ri = 0; ri < count; ++ri)
        for (int64_t n = 0; n < c_o; ++n) {
            int64_t i = rows ? rows[ri] : ri;
            int32_t sum = 0;
            for (int64_t j = 0; j < c_i; ++j) sum += (int32_t)xq[i * c_i + j] * (int32_t)wq[n * c_i + j];
            float c = x_scale[per_token ? i : 0] * w_scale[w_per_channel ? n : 0];
            y[i * c_o + n] = epilogue(sum, c, bias, n, relu, residual, i * c_o + n, out_dtype);
        }
    return 0;
}

int orc_w8a8_linear(const int8_t* xq, const float* x_scale, int per_token, const int8_t* wq,
                    const float* w_scale, const float* bias, const uint16_t* residual, int relu,
                    uint16_t* y, int out_dtype, int64_t t, int64_t c_i, int64_t c_o)
{
    return orc_w8a8_linear_rows(xq, x_scale, per_token, wq, w_scale, 0, bias, residual, relu, y, out_dtype,
                                t, c_i, c_o, NULL, 0);
}

/* ---------------------------------------------------------------- INT8 attention BMMs */

/* c[b, m, n] = round16( fl32( float(sum_k a[b,m,k] * B[b,k,n]) * alpha ) ).
   trans_b = 1: bm is [b, n, k] (Q K^T);  trans_b = 0: bm is [b, k, n] (P V).
   Batch strides in elements.  Only batches listed in `batches` (or all if NULL). */
int orc_w8a8_bmm(const int8_t* a, const int8_t* bm, int trans_b, float alpha, uint16_t* c, int out_dtype,
                 int64_t b, int64_t m, int64_t n, int64_t k, int64_t stride_a, int64_t stride_b,
                 int64_t stride_c, const int64_t* batches, int64_t nbatches)
{
    if (!a || !bm || !c) return 1;
    if (b <= 0 || m <= 0 || n <= 0 || k <= 0) return 2;
    int64_t count = batches ? nbatches : b;
    for (int64_t bi = 0; bi < count; ++bi) {
        int64_t ib = batches ? batches[bi] : bi;
        const int8_t* pa = a + ib * stride_a;
        const int8_t* pb = bm + ib * stride_b;
        uint16_t* pc = c + ib * stride_c;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                int32_t sum = 0;
                if (trans_b)
                    for (int64_t kk = 0; kk < k; ++kk) sum += (int32_t)pa[i * k + kk] * (int32_t)pb[j * k + kk];
                else
                    for (int64_t kk = 0; kk < k; ++kk) sum += (int32_t)pa[i * k + kk] * (int32_t)pb[kk * n + j];
                pc[i * n + j] = store16((float)sum * alpha, out_dtype);
            }
    }
    return 0;
}

/* Row softmax in fp64 on 16-bit scores, probabilities rounded to the 16-bit type (the paper keeps
   Softmax in FP16), then quantized with the fixed step 1/127: code = round(p * 127) in [0, 127]. */
int orc_softmax_quant_p(const uint16_t* s, int dtype, int64_t rows, int64_t cols, int8_t* pq)
{
    if (!s || !pq) return 1;
    if (rows <= 0 || cols <= 0) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const uint16_t* row = s + i * cols;
        double mx = -INFINITY;
        for (int64_t j = 0; j < cols; ++j) {
            double z = (double)load16(row + j, dtype);
            if (z > mx) mx = z;
        }
        double den = 0.0;
        for (int64_t j = 0; j < cols; ++j) den += exp((double)load16(row + j, dtype) - mx);
        for (int64_t j = 0; j < cols; ++j) {
            double p = exp((double)load16(row + j, dtype) - mx) / den;
            float p16 = load16(&(uint16_t){store16((float)p, dtype)}, dtype);
            pq[i * cols + j] = round_code(p16 * 127.0f);
        }
    }
    return 0;
}

/* The same with a causal mask, as the decoder-only models of the paper apply it (the paper does not spell the
   mask out; reading: query i of a head sees the keys j <= i + (s_k - s_q), i.e. the last query sees every key,
   which is the usual rule when s_k - s_q earlier keys sit in a cache).  s, pq: [b, s_q, s_k].  Only the visible
   scores enter the maximum and the sum; hidden positions get code 0.  Needs s_k >= s_q (every row sees a key). */
int orc_softmax_quant_p_causal(const uint16_t* s, int dtype, int64_t b, int64_t s_q, int64_t s_k, int8_t* pq)
{
    if (!s || !pq) return 1;
    if (b <= 0 || s_q <= 0 || s_k < s_q) return 2;
    const int64_t off = s_k - s_q;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < b * s_q; ++r) {
        const int64_t i = r % s_q;
        const int64_t vis = i + off + 1; /* number of visible keys */
        const uint16_t* row = s + r * s_k;
        double mx = -INFINITY;
        for (int64_t j = 0; j < vis; ++j) {
            double z = (double)load16(row + j, dtype);
            if (z > mx) mx = z;
        }
        double den = 0.0;
        for (int64_t j = 0; j < vis; ++j) den += exp((double)load16(row + j, dtype) - mx);
        for (int64_t j = 0; j < vis; ++j) {
            double p = exp((double)load16(row + j, dtype) - mx) / den;
            float p16 = load16(&(uint16_t){store16((float)p, dtype)}, dtype);
            pq[r * s_k + j] = round_code(p16 * 127.0f);
        }
        for (int64_t j = vis; j < s_k; ++j) pq[r * s_k + j] = 0;
    }
    return 0;
}

/* LayerNorm whose affine parameters already carry 1/s (gamma' = gamma * inv_s, beta' = beta * inv_s,
   folded offline), followed by per-token dynamic quantization.  Statistics in fp64 over the row;
   x_hat = fl32( (x - mu) / sqrt(var + eps) * gamma'_j + beta'_j ). */
int orc_ln_quantize(const uint16_t* x, int dtype, int64_t t, int64_t c_i, const float* gamma_f,
                    const float* beta_f, float eps, float* scale, int8_t* xq)
{
    if (!x || !gamma_f || !beta_f || !scale || !xq) return 1;
    if (t <= 0 || c_i <= 0) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i) {
        const uint16_t* row = x + i * c_i;
        double mu = 0.0;
        for (int64_t j = 0; j < c_i; ++j) mu += (double)load16(row + j, dtype);
        mu /= (double)c_i;
        double var = 0.0;
        for (int64_t j = 0; j < c_i; ++j) {
            double d = (double)load16(row + j, dtype) - mu;
            var += d * d;
        }
        var /= (double)c_i;
        double rstd = 1.0 / sqrt(var + (double)eps);
        float* xh = (float*)malloc((size_t)c_i * sizeof(float));
        float a = 0.0f;
        for (int64_t j = 0; j < c_i; ++j) {
            double v = ((double)load16(row + j, dtype) - mu) * rstd * (double)gamma_f[j] + (double)beta_f[j];
            xh[j] = (float)v;
            float av = fabsf(xh[j]);
            if (av > a) a = av;
        }
        scale[i] = a / 127.0f;
        float r = a > 0.0f ? 127.0f / a : 0.0f;
        for (int64_t j = 0; j < c_i; ++j) xq[i * c_i + j] = round_code(xh[j] * r);
        free(xh);
    }
    return 0;
}

/* Number of OpenMP threads the loops above will use (reported by the CPU-baseline timing). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif

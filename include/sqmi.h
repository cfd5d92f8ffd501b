/*
 * sqmi -- SmoothQuant W8A8 hot path for AMD MI355X (gfx950).  C ABI.
 *
 * The library computes a linear layer Y = X W (X [T, C_i], W [C_i, C_o]; Sec. 2) as
 *     Y = diag(Delta_X) (Xq Wq) diag(Delta_W)                       (Eq. 2)
 * after the offline smoothing transform X_hat = X diag(s)^-1, W_hat = diag(s) W (Eq. 3) with
 * s_j = max|X_j|^alpha / max|W_j|^(1-alpha) (Eq. 4), quantizing with the symmetric absmax
 * quantizer Xq = round(X / Delta), Delta = max|X| / 127 (Eq. 1) at one of the granularities of
 * Table 2 (O1 per-token dynamic, O2 per-tensor dynamic, O3 per-tensor static), plus the two INT8
 * batched matmuls of attention (Sec. 4, "Applying ... to Transformer blocks").
 *
 * Conventions for every entry point
 *  - "device" pointers are HIP device memory of the current device, "host" pointers ordinary memory.
 *  - The caller owns every buffer, workspace included; the library never allocates, frees or keeps
 *    a pointer.  Calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL = default
 *    stream) and never synchronize; buffers must stay alive until the stream has run the work.
 *  - Errors are returned as sq_status; argument errors are detected on the host before any launch.
 *  - Device tensors must be 16-byte aligned; C_i (the contraction length) must be a multiple of 16.
 *    Further limits are stated with the entry point they belong to; all of them are checked on the host.
 *  - Fixed arithmetic (so that int8 codes are reproducible bit for bit): round-half-to-even;
 *    X / Delta is evaluated as X * r with r = fl32(127 / absmax) (r = fl32(1 / Delta) in static
 *    mode); codes lie in [-127, 127] (static mode saturates); absmax = 0 gives Delta = 0 and codes
 *    0; all scales are fp32; no fused multiply-add in scale arithmetic.  Non-finite inputs:
 *    unspecified.
 */
#ifndef SQMI_H
#define SQMI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SQ_OK = 0,
    SQ_ERR_NULL = 1,        /* a required pointer is NULL */
    SQ_ERR_SHAPE = 2,       /* non-positive / overflowing / inconsistent dimension */
    SQ_ERR_ALIGN = 3,       /* pointer not 16-byte aligned, or a dimension / stride not a multiple of what the entry
                               point asks for (C_i % 16 everywhere; see each declaration) */
    SQ_ERR_UNSUPPORTED = 4, /* enum value or parameter outside the supported set */
    SQ_ERR_WORKSPACE = 5,   /* workspace missing or smaller than sq_workspace_bytes() */
    SQ_ERR_HIP = 6          /* the HIP runtime reported an error at launch */
} sq_status;

typedef enum { SQ_F16 = 0, SQ_BF16 = 1 } sq_dtype;

/* Table 2: activation quantization granularity. */
typedef enum {
    SQ_PER_TOKEN_DYNAMIC = 0,  /* O1 */
    SQ_PER_TENSOR_DYNAMIC = 1, /* O2 */
    SQ_PER_TENSOR_STATIC = 2   /* O3 */
} sq_act_mode;

/* Memory layout of an int8 GEMM operand with `rows` rows and k contraction elements.
 *  SQ_ROW_MAJOR: [rows, k], k contiguous.
 *  SQ_TILED:     the layout the GEMM streams fastest (every wave-wide load reads 1 KB of contiguous
 *                memory).  Requires k % 64 == 0.  The buffer holds ceil(rows/16)*16 rows
 *                (sq_tiled_bytes()); element (r, c) lives at byte
 *                  ((r/16) * (k/64) + c/64) * 1024 + (r%16) * 64 + ((((c%64)/16) ^ sw) * 16) + c%16,
 *                  sw = (((r%16) >> 1) & 3) ^ (((r%16) >> 3) & 1).
 *                Rows beyond `rows` in the last block row are padding: never read as results, their
 *                content is unspecified. */
typedef enum { SQ_ROW_MAJOR = 0, SQ_TILED = 1 } sq_layout;

/* Bytes of an int8 [rows, k] operand in SQ_TILED layout (k % 64 == 0), 0 on invalid arguments. */
size_t sq_tiled_bytes(int64_t rows, int64_t k);

typedef enum {
    SQ_OP_QUANTIZE_ACT = 0,
    SQ_OP_PREPARE_WEIGHT = 1,
    SQ_OP_W8A8_LINEAR = 2,
    SQ_OP_I8_GEMM_I32 = 3,
    SQ_OP_W8A8_BMM = 4
} sq_op;

const char* sq_status_string(sq_status st);

/* Eq. 4 (Sec. 4): s_j = max(x_absmax_j, 1e-5)^alpha / max(w_absmax_j, 1e-5)^(1-alpha), powers in
 * fp64 rounded to fp32; inv_s_j = fl32(1 / s_j).  Offline, tiny: HOST pointers, computed on the
 * host.  x_absmax, w_absmax, s: fp32 [c_i]; inv_s: fp32 [c_i] or NULL.  alpha outside [0, 1] ->
 * SQ_ERR_UNSUPPORTED. */
sq_status sq_smooth_scales(const float* x_absmax, const float* w_absmax, float alpha, int64_t c_i,
                           float* s, float* inv_s);

/* Calibration statistic of Eq. 4: out_j = max_t |X_tj|.  x: device [t, c_i] row-major 16-bit;
 * out: device fp32 [c_i], overwritten. */
sq_status sq_act_absmax_per_channel(const void* x, sq_dtype dtype, int64_t t, int64_t c_i,
                                    float* out, void* stream);

/* Weight statistic of Eq. 4: out_j = max_n |W_jn| (row j of W = input channel j).  w: device
 * [c_i, c_o] row-major 16-bit (the paper's W orientation); out: device fp32 [c_i].
 * Limits: c_o % 8 == 0 (SQ_ERR_ALIGN). */
sq_status sq_weight_absmax_per_in_channel(const void* w, sq_dtype dtype, int64_t c_i, int64_t c_o,
                                          float* out, void* stream);

/* Offline weight preparation (Eq. 3 then Eq. 1, per-tensor as in Table 2):
 *   W_hat = diag(s) W;  Delta_W = max|W_hat| / 127;  Wq = round(W_hat * fl32(127 / max|W_hat|)).
 * With w_scale_per_channel != 0 the maximum, the step and the rounding are taken per output channel n
 * (column n of W_hat), the weight granularity of Table 7: Delta_W[n] = max_j |W_hat[j, n]| / 127.
 * w: device [c_i, c_o] row-major 16-bit; s: device fp32 [c_i] or NULL (s = 1);
 * wq: device int8 [c_o, c_i] (transposed: contraction index contiguous) in layout `wq_layout`;
 * w_scale: device fp32 [1], or [c_o] with w_scale_per_channel.
 * workspace: device, >= sq_workspace_bytes(SQ_OP_PREPARE_WEIGHT, 0, c_i, c_o) bytes.
 * Limits: c_i % 16 == 0 and c_o % 8 == 0 (SQ_ERR_ALIGN); c_i <= 64 * 65535 (SQ_ERR_SHAPE); SQ_TILED needs
 * c_i % 64 == 0. */
sq_status sq_prepare_weight(const void* w, sq_dtype dtype, const float* s, int64_t c_i, int64_t c_o,
                            int8_t* wq, sq_layout wq_layout, float* w_scale, int w_scale_per_channel,
                            void* workspace, size_t ws_bytes, void* stream);

/* Activation quantization (Eq. 1; granularities of Table 2).
 * x: device [t, c_i] 16-bit, row stride ldx elements (ldx >= c_i, multiple of 8);
 * inv_s: device fp32 [c_i] or NULL -- when given, x_hat = fl32(x * inv_s_j) is quantized (the
 *   "extra scaling" for inputs whose producer cannot absorb 1/s, Sec. 4);
 * scale: device fp32; written in the dynamic modes ([t] per token, [1] per tensor), read in
 *   SQ_PER_TENSOR_STATIC ([1], the calibrated Delta);
 * xq: device int8 [t, c_i] in layout `xq_layout`;  workspace: device, needed for
 *   SQ_PER_TENSOR_DYNAMIC only: with sq_workspace_bytes(SQ_OP_QUANTIZE_ACT, ...) bytes, tensors of up to
 *   512 x 16384 elements run as one launch and cross HBM once (the maximum and the rounding are separated inside
 *   the kernel by a bounded wait on an arrival count; should the wait ever expire, scale[0] = NaN and no code is
 *   written).  Larger tensors, a smaller workspace (at least 4 bytes) or a stream under graph capture run as
 *   three launches with identical results.  The workspace needs no initialisation; concurrent calls must not
 *   share it. */
sq_status sq_quantize_act(const void* x, sq_dtype dtype, int64_t t, int64_t c_i, int64_t ldx,
                          const float* inv_s, sq_act_mode mode, float* scale, int8_t* xq,
                          sq_layout xq_layout, void* workspace, size_t ws_bytes, void* stream);

/* W8A8 linear layer (Eq. 2) with the dequantizing epilogue fused into the INT8 GEMM:
 *   acc_tn = sum_j xq[t, j] * wq[n, j]                                   (exact int32)
 *   v = fl32(float(acc_tn) * fl32(x_scale_t * w_scale_n)); v += bias_n; v = max(v, 0) if relu;
 *   v += residual_tn;  y_tn = round_to_16bit(v).
 * xq: device int8 [t, c_i]; x_scale: device fp32 [t] if x_scale_per_token else [1];
 * wq: device int8 [c_o, c_i]; w_scale: device fp32 [c_o] if w_scale_per_channel else [1] (Eq. 2's diag(Delta_W));
 * bias: device fp32 [c_o] or NULL; residual: device [t, c_o] of the output dtype or NULL;
 * y: device [t, c_o] of dtype `out`, row-major.
 * layout: layout of BOTH xq and wq (as produced by sq_quantize_act / sq_prepare_weight).
 * workspace: device, >= sq_workspace_bytes(SQ_OP_W8A8_LINEAR, t, c_i, c_o) bytes (may be 0). */
sq_status sq_w8a8_linear(const int8_t* xq, const float* x_scale, int x_scale_per_token,
                         const int8_t* wq, const float* w_scale, int w_scale_per_channel, const float* bias,
                         const void* residual, int relu, void* y, sq_dtype out, int64_t t,
                         int64_t c_i, int64_t c_o, sq_layout layout, void* workspace, size_t ws_bytes,
                         void* stream);

/* sq_w8a8_linear for callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same
 * kernels, same results.  The K-split scratch is a 64 MiB device array inside the library
 * (sq_static_scratch_bytes()); every GPU the library is used on holds its own copy until the process ends.  The
 * call allocates nothing; the first call on a device resolves the array's address (make that call outside a
 * graph capture).  Shapes whose sq_workspace_bytes(SQ_OP_W8A8_LINEAR, ...) exceeds the array are rejected with
 * SQ_ERR_WORKSPACE before any launch.  All calls on one GPU share the array: calls that overlap in time on the
 * same GPU (different streams or threads) race; calls on one stream are ordered and safe. */
sq_status sq_w8a8_linear_noalloc(const int8_t* xq, const float* x_scale, int x_scale_per_token,
                                 const int8_t* wq, const float* w_scale, int w_scale_per_channel,
                                 const float* bias, const void* residual, int relu, void* y, sq_dtype out,
                                 int64_t t, int64_t c_i, int64_t c_o, sq_layout layout, void* stream);
size_t sq_static_scratch_bytes(void);

/* The same layer with the static activation quantizer of the NEXT int8 kernel fused into the epilogue (the
 * "fuse into the previous layer" idea of Sec. 4 applied to the quantize step; Table 2's O3 pipeline):
 *   v16 = the 16-bit value sq_w8a8_linear would store, in dtype `mid`;
 *   yq_tn = clamp(round_half_even(fl32(v16 * fl32(1 / y_step))), -127, 127)   -- sq_quantize_act, static mode.
 * So the codes equal sq_quantize_act(SQ_PER_TENSOR_STATIC) applied to sq_w8a8_linear's output, without the
 * 16-bit tensor ever reaching HBM.  y_step: device fp32 [1], the calibrated Delta of the output tensor;
 * yq: device int8 [t, c_o] in `yq_layout` (SQ_TILED: c_o % 64 == 0, sq_tiled_bytes(t, c_o) bytes); c_o % 8 == 0;
 * residual: of dtype `mid`.  Other arguments as sq_w8a8_linear. */
sq_status sq_w8a8_linear_q8(const int8_t* xq, const float* x_scale, int x_scale_per_token,
                            const int8_t* wq, const float* w_scale, int w_scale_per_channel,
                            const float* bias, const void* residual, int relu, sq_dtype mid,
                            const float* y_step, int8_t* yq, sq_layout yq_layout, int64_t t, int64_t c_i,
                            int64_t c_o, sq_layout layout, void* workspace, size_t ws_bytes, void* stream);

/* The raw integer contraction of Eq. 2 (test export: makes the bit-exact int32 gate observable).
 * acc: device int32 [t, c_o] row-major; layout: layout of both xq and wq. */
sq_status sq_i8_gemm_i32(const int8_t* xq, const int8_t* wq, int32_t* acc, int64_t t, int64_t c_i,
                         int64_t c_o, sq_layout layout, void* workspace, size_t ws_bytes, void* stream);

/* INT8 batched matmul of attention (Sec. 4): c[b] = round_to_16bit( fl32( float(a[b] B[b]) * alpha ) ).
 * a: device int8 [b, m, k]; bm: device int8, [b, n, k] if trans_b (Q K^T) else [b, k, n] (P V);
 * alpha: HOST scalar (e.g. Delta_Q Delta_K / sqrt(d), or Delta_V / 127);
 * c: device [b, m, n] of dtype `out`.  Batch strides in elements (multiples of 16 for a and bm, of 8 for c);
 * k % 16 == 0; for trans_b == 0 also n % 16 == 0; b <= 65535.  Needs no workspace at any shape. */
sq_status sq_w8a8_bmm(const int8_t* a, const int8_t* bm, int trans_b, float alpha, void* c,
                      sq_dtype out, int64_t b, int64_t m, int64_t n, int64_t k, int64_t stride_a,
                      int64_t stride_b, int64_t stride_c, void* stream);

/* The INT8 attention block of Sec. 4 in one kernel -- both batched matmuls in INT8, the softmax in the 16-bit
 * floating type -- without the [s_q, s_k] score and probability tensors ever reaching memory:
 *   s_ij = round_to_16bit( fl32( float(sum_c q[i, c] k[j, c]) * alpha1 ) )            (sq_w8a8_bmm, trans_b = 1)
 *   p_ij = round_to_16bit( e^(s_ij - max_j s_ij) / sum_j e^(s_ij - max_j s_ij) ),  pq_ij = round(127 p_ij)   (sq_softmax_quant_p)
 *   o_ic = round_to_16bit( fl32( float(sum_j pq_ij v[j, c]) * alpha2 ) )              (sq_w8a8_bmm, trans_b = 0)
 * i.e. the quantization points of the chain of those three calls with `out` as the dtype of s, p and o.  The
 * integer sums are exact; the exponential and the division are fp32 on the device (as in sq_softmax_quant_p), so
 * a code pq may differ by one from an fp64 evaluation, rarely.
 * q: device int8 [b, s_q, d]; k, v: device int8 [b, s_k, d] (row-major, d contiguous); alpha1 (> 0, e.g.
 * Delta_Q Delta_K / sqrt(d)) and alpha2 (e.g. Delta_V / 127): HOST scalars; o: device [b, s_q, d] of dtype `out`.
 * Batch strides in elements (multiples of 16 for q, k, v, of 8 for o).
 * p_codes: NULL, or device int8 [b, s_q, s_k] (4-byte aligned) that receives the codes pq the kernel formed
 * (inspection and tests; costs their write).
 * Limits: d = 64 or 128 (else SQ_ERR_UNSUPPORTED: use the three calls above); s_k % 16 == 0 (SQ_ERR_ALIGN); any s_q.
 * Needs no workspace. */
sq_status sq_w8a8_attention(const int8_t* q, const int8_t* k, const int8_t* v, float alpha1, float alpha2,
                            void* o, sq_dtype out, int64_t b, int64_t s_q, int64_t s_k, int64_t d,
                            int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                            int8_t* p_codes, void* stream);

/* The same block with the causal mask of a decoder (the models of Sec. 5 are decoder-only; the paper does not spell
 * the mask out): query i sees the keys j <= i + (s_k - s_q), so with s_k = s_q every query sees the keys up to its
 * own position, and with s_k > s_q the first s_k - s_q keys (a cache of earlier tokens) are seen by all.  Hidden keys
 * take no part in the maximum or the sum of the softmax and get probability code 0; key tiles no row of a workgroup
 * sees are skipped, which is where the time goes down.  Arguments, layouts and limits as sq_w8a8_attention, plus
 * s_k >= s_q (SQ_ERR_SHAPE otherwise: the first queries would see nothing).  Equals sq_w8a8_bmm, then
 * sq_softmax_quant_p on scores that hold -inf at the hidden positions, then sq_w8a8_bmm. */
sq_status sq_w8a8_attention_causal(const int8_t* q, const int8_t* k, const int8_t* v, float alpha1, float alpha2,
                                   void* o, sq_dtype out, int64_t b, int64_t s_q, int64_t s_k, int64_t d,
                                   int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                                   int8_t* p_codes, void* stream);

/* Row softmax kept in 16-bit floating point (Sec. 4 keeps Softmax in FP16) followed by quantization
 * of the probabilities with the fixed step 1/127: pq = round(p * 127) in [0, 127].
 * s: device [rows, cols] 16-bit scores, packed; pq: device int8 [rows, cols].
 * Limits: cols % 8 == 0 (SQ_ERR_ALIGN), cols <= 16384 (SQ_ERR_UNSUPPORTED).  Scores of -inf (masked positions)
 * get probability 0; a row that holds nothing but -inf gets codes 0 throughout.  NaN or +inf: unspecified. */
sq_status sq_softmax_quant_p(const void* s, sq_dtype dtype, int64_t rows, int64_t cols, int8_t* pq,
                             void* stream);

/* LayerNorm whose affine parameters already carry the smoothing factors (gamma_f = gamma / s,
 * beta_f = beta / s, folded offline as Sec. 4 describes) fused with per-token dynamic quantization:
 *   x_hat_tj = (x_tj - mean_t) * rstd_t * gamma_f_j + beta_f_j;  then Eq. 1 per token.
 * x: device [t, c_i] 16-bit packed; gamma_f, beta_f: device fp32 [c_i]; scale: device fp32 [t];
 * xq: device int8 [t, c_i] in layout `xq_layout`.
 * Limits: c_i % 16 == 0 (SQ_ERR_ALIGN), c_i <= 16384 (SQ_ERR_UNSUPPORTED); gamma_f, beta_f 16-byte aligned. */
sq_status sq_ln_quantize(const void* x, sq_dtype dtype, int64_t t, int64_t c_i, const float* gamma_f,
                         const float* beta_f, float eps, float* scale, int8_t* xq, sq_layout xq_layout,
                         void* stream);

/* Workspace size in bytes for `op` at the given problem size (0 if none is needed).  For
 * SQ_OP_W8A8_BMM pass (m, k, n) as (t, c_i, c_o). */
size_t sq_workspace_bytes(sq_op op, int64_t t, int64_t c_i, int64_t c_o);

#ifdef __cplusplus
}
#endif
#endif /* SQMI_H */

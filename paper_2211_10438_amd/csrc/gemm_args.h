// Argument block and epilogue arithmetic shared by the INT8 GEMM kernels (gfx950).
#pragma once
#include "common.h"

#define GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define LPTR(p) ((__attribute__((address_space(3))) void*)(p))

struct GemmArgs {
    const int8_t* A;  // [batch][M, K], row stride lda bytes
    const int8_t* B;  // [batch][N, K], row stride ldb bytes
    int M, N, K;
    int64_t lda, ldb;
    int64_t strideA, strideB, strideC;  // batch strides in elements
    int tiles_m, tiles_n, splits, iters_per_split;
    // dequant epilogue
    void* C;  // [batch][M, N] 16-bit, row stride N
    const float* x_scale;  // [M] or [1] or NULL (then `alpha` is the whole scale)
    int per_token;
    const float* w_scale;  // [1], or [N] with w_per_channel
    int w_per_channel;
    float alpha;
    const float* bias;     // [N] or NULL
    const void* residual;  // [M, N] out dtype or NULL
    int relu;
    // int32 output (raw accumulators or split-K partials): [splits][M, N]
    int32_t* acc_out;
    // int8 output (producer-side fusion): when q8_step is set, the 16-bit value the epilogue would have stored is
    // quantized with the calibrated step q8_step[0] (Eq. 1, static) and written to q8_out [M, N] instead of C.
    const float* q8_step;
    int8_t* q8_out;
    int q8_tiled;
};

// Static per-tensor quantization of a value that has already been rounded to the 16-bit type `BF16` selects:
// the same arithmetic as the static mode of the activation quantizer (x * fl32(1 / Delta), nearest-even, +-127).
template <bool BF16> SQ_DEVICE int requant_code(uint32_t bits16, float r)
{
    return round_code(load16_bits<BF16>(bits16) * r);
}

template <int N> SQ_DEVICE void wait_vmcnt_imm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// Outer-dimension scaling of Eq. 2 on one accumulator: (float)acc * c, then the optional terms in the
// order bias, ReLU, residual, then one rounding to the 16-bit output type.
template <bool BF16>
SQ_DEVICE uint32_t dequant_one(int acc, float c, float bias, bool has_bias, bool relu, uint32_t res_bits, bool has_res)
{
    float v = (float)acc * c;
    if (has_bias) v = v + bias;
    if (relu) v = v > 0.0f ? v : 0.0f;
    if (has_res) v = v + load16_bits<BF16>(res_bits);
    return store16_bits<BF16>(v);
}

// The same for two neighbouring outputs, narrowed together (lo = first): one conversion instruction for the pair.
// (the accumulators arrive already converted to fp32: exact up to 2^24, round-to-nearest-even beyond, like the cast)
template <bool BF16>
SQ_DEVICE uint32_t dequant_pair_f(float acc0, float acc1, float c0, float c1, float bias0, float bias1, bool has_bias, bool relu,
                                  uint32_t res_pair, bool has_res)
{
    float v0 = acc0 * c0, v1 = acc1 * c1;
    if (has_bias) { v0 = v0 + bias0; v1 = v1 + bias1; }
    if (relu) { v0 = v0 > 0.0f ? v0 : 0.0f; v1 = v1 > 0.0f ? v1 : 0.0f; }
    if (has_res) { v0 = v0 + load16_bits<BF16>(res_pair); v1 = v1 + load16_bits<BF16>(res_pair >> 16); }
    return store16x2_bits<BF16>(v0, v1);
}
template <bool BF16>
SQ_DEVICE uint32_t dequant_pair(int acc0, int acc1, float c0, float c1, float bias0, float bias1, bool has_bias, bool relu,
                                uint32_t res_pair, bool has_res)
{
    return dequant_pair_f<BF16>((float)acc0, (float)acc1, c0, c1, bias0, bias1, has_bias, relu, res_pair, has_res);
}

// Weight-streaming GEMM for few-token shapes (gemm_i8_stream.hip).  sq_stream_gemm_splits returns 0
// when the shape is left to the tile kernels, else the number of K splits of its plan: 1 = the kernel
// writes the final output itself; > 1 = it writes int32 partial sums to a.acc_out[splits][M][N] (which
// the caller points at a workspace) and the split-K reduction kernel finishes the job.
int sq_stream_gemm_splits(int64_t M, int64_t N, int64_t K, int64_t batch, bool tiled);
void sq_stream_gemm_launch(const GemmArgs& a, bool to_i32, bool bf16, bool tiled, hipStream_t st);

// Strip kernel for attention scores (bmm_strip.hip): B = [N, K] with K <= 128, alpha-only epilogue.
bool sq_strip_bmm_eligible(int64_t M, int64_t N, int64_t K, int64_t batch);
void sq_strip_bmm_launch(const GemmArgs& a, int batch, bool bf16, hipStream_t st);

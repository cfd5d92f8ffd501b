// Row-wise 16-bit floating point operators that sit between the INT8 kernels (Sec. 4 keeps Softmax
// and LayerNorm in FP16) fused with the quantization that feeds the next INT8 kernel, gfx950:
//   * softmax over attention scores + quantization of P with the fixed step 1/127,
//   * LayerNorm with the smoothing factors folded into gamma/beta + per-token dynamic quantization.
// One row per 256-thread workgroup, the row held in registers: one HBM pass, 2 B in + 1 B out.
#include "common.h"

namespace {

template <bool BF16> SQ_DEVICE void unpack8r(const v4u raw, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = load16_bits<BF16>(raw[e]);
        f[2 * e + 1] = load16_bits<BF16>(raw[e] >> 16);
    }
}

// e^x for x <= 0 through the hardware 2^x instruction (v_exp_f32): about 3 ulp of fp32 where the result
// matters (x > -6), far below the half-ulp of the 16-bit rounding that follows; results below 2^-126 come
// out as 0, which is what their codes are anyway.  The library routine costs ~20 instructions per call and
// made this pass ALU-bound.
// e^(z - m) with the subtraction folded into one fused multiply-add: 2^(z * log2(e) + nm), nm = -m * log2(e)
// rounded once per row.  Against (z - m) * log2(e) the argument differs by at most ~2 of its ulps (|argument| < 64),
// i.e. a relative 1e-5 in the result, far below the half-ulp of the 16-bit rounding that follows.
SQ_DEVICE float fast_exp_shifted(float z, float nm) { return __builtin_amdgcn_exp2f(__builtin_fmaf(z, 1.44269504088896340736f, nm)); }
// Code of a probability p16 in [0, 1] (already rounded to the 16-bit type): round(p16 * 127) needs no clamp, and
// p16 * 127 is exact in fp32 (11 x 7 significant bits), so the fused multiply-add with 1.5 * 2^23 rounds exactly
// once, to nearest-even, like the separate multiply and add of code_bits.
SQ_DEVICE uint32_t prob_code_bits(float p16) { return __builtin_bit_cast(uint32_t, __builtin_fmaf(p16, 127.0f, 12582912.0f)); }

template <int NT = 256> SQ_DEVICE float block_max_r(float v, float* red)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float m = __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
#pragma unroll
    for (int w = 4; w < NT / 64; w += 4)
        m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fmaxf(red[w], red[w + 1]), __builtin_fmaxf(red[w + 2], red[w + 3])));
    return m;
}
template <int NT = 256> SQ_DEVICE float block_sum_r(float v, float* red)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = (red[0] + red[1]) + (red[2] + red[3]);
#pragma unroll
    for (int w = 4; w < NT / 64; w += 4) t += (red[w] + red[w + 1]) + (red[w + 2] + red[w + 3]);
    return t;
}

SQ_DEVICE v2u pack8(const uint32_t (&q)[8])  // code_bits words -> 8 bytes
{
    return v2u{pack4_low_bytes(q[0], q[1], q[2], q[3]), pack4_low_bytes(q[4], q[5], q[6], q[7])};
}

template <bool BF16, int NV>
__global__ __launch_bounds__(256) void softmax_quant_kernel(const uint16_t* __restrict__ s, int cols, int8_t* __restrict__ pq)
{
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const v4u* sr = (const v4u*)(s + row * (int64_t)cols);
    const int nvec = cols >> 3;
    float z[NV][8];
    float mx = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * 256;
        if (idx < nvec) {
            unpack8r<BF16>(__builtin_nontemporal_load(sr + idx), z[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) mx = __builtin_fmaxf(mx, z[i][e]);
        }
    }
    mx = block_max_r(mx, red);
    // a row of -inf only (fully masked) has no maximum to shift by: its exponentials are 0 and so are its codes
    const float nmx = mx == -__builtin_inff() ? 0.0f : -mx * 1.44269504088896340736f;
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * 256;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                z[i][e] = fast_exp_shifted(z[i][e], nmx);
                sum += z[i][e];
            }
        }
    }
    sum = block_sum_r(sum, red);
    const float inv = sum > 0.0f ? 1.0f / sum : 0.0f;
    v2u* out = (v2u*)(pq + row * (int64_t)cols);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * 256;
        if (idx < nvec) {
            uint32_t q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // probability rounded to the 16-bit type first (the softmax output is a 16-bit tensor)
                const float p16 = load16_bits<BF16>(store16_bits<BF16>(z[i][e] * inv));
                q[e] = prob_code_bits(p16);
            }
            __builtin_nontemporal_store(pack8(q), out + idx);
        }
    }
}

// One row per wave (rows up to 4096 scores): four rows per 256-thread workgroup, the reductions are
// cross-lane shuffles only (no barriers), and every lane keeps NV 16-byte loads in flight, which is what a
// pass bound by HBM latency x bandwidth needs (a 256-thread workgroup per 4 KB row had 16 bytes per lane).
template <bool BF16, int NV>
__global__ __launch_bounds__(256) void softmax_quant_wave_kernel(const uint16_t* __restrict__ s, int64_t rows, int cols,
                                                                int8_t* __restrict__ pq)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const v4u* sr = (const v4u*)(s + row * (int64_t)cols);
    const int nvec = cols >> 3;
    float z[NV][8];
    float mx = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            unpack8r<BF16>(__builtin_nontemporal_load(sr + idx), z[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) mx = __builtin_fmaxf(mx, z[i][e]);
        }
    }
    mx = wave_max(mx);
    // a row of -inf only (fully masked) has no maximum to shift by: its exponentials are 0 and so are its codes
    const float nmx = mx == -__builtin_inff() ? 0.0f : -mx * 1.44269504088896340736f;
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                z[i][e] = fast_exp_shifted(z[i][e], nmx);
                sum += z[i][e];
            }
        }
    }
    sum = wave_sum(sum);
    const float inv = sum > 0.0f ? 1.0f / sum : 0.0f;
    v2u* out = (v2u*)(pq + row * (int64_t)cols);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            uint32_t q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float p16 = load16_bits<BF16>(store16_bits<BF16>(z[i][e] * inv));
                q[e] = prob_code_bits(p16);
            }
            __builtin_nontemporal_store(pack8(q), out + idx);
        }
    }
}

template <bool BF16, int NV, int NT>
__global__ __launch_bounds__(NT) void ln_quant_kernel(const uint16_t* __restrict__ x, int c_i, const float* __restrict__ gamma_f,
                                                      const float* __restrict__ beta_f, float eps, float* __restrict__ scale,
                                                      int8_t* __restrict__ xq, bool tiled)
{
    __shared__ float red[NT / 64];
    const int64_t row = blockIdx.x;
    const v4u* xr = (const v4u*)(x + row * (int64_t)c_i);
    const int nvec = c_i >> 3;
    float f[NV][8];
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        if (idx < nvec) {
            unpack8r<BF16>(__builtin_nontemporal_load(xr + idx), f[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += f[i][e];
        }
    }
    const float mean = block_sum_r<NT>(sum, red) / (float)c_i;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = f[i][e] - mean;
                sq += d * d;
            }
        }
    }
    const float var = block_sum_r<NT>(sq, red) / (float)c_i;
    const float rstd = 1.0f / sqrtf(var + eps);
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        if (idx < nvec) {
            const float4 g0 = *(const float4*)(gamma_f + idx * 8), g1 = *(const float4*)(gamma_f + idx * 8 + 4);
            const float4 b0 = *(const float4*)(beta_f + idx * 8), b1 = *(const float4*)(beta_f + idx * 8 + 4);
            const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
            const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                f[i][e] = (f[i][e] - mean) * rstd * g[e] + b[e];
                m = __builtin_fmaxf(m, __builtin_fabsf(f[i][e]));
            }
        }
    }
    const float a = block_max_r<NT>(m, red);
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    if (threadIdx.x == 0) scale[row] = a / 127.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        if (idx < nvec) {
            uint32_t q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = code_bits(f[i][e] * r);
            __builtin_nontemporal_store(pack8(q), (v2u*)code_dst(xq, row, idx * 8, c_i, tiled));
        }
    }
}

// One row per wave (hidden sizes up to 2048, where it measures faster than a workgroup per row): the three
// reductions are cross-lane shuffles, no barriers, and a lane keeps NV 16-byte loads in flight.
template <bool BF16, int NV>
__global__ __launch_bounds__(256) void ln_quant_wave_kernel(const uint16_t* __restrict__ x, int64_t t, int c_i,
                                                           const float* __restrict__ gamma_f, const float* __restrict__ beta_f,
                                                           float eps, float* __restrict__ scale, int8_t* __restrict__ xq, bool tiled)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= t) return;
    const v4u* xr = (const v4u*)(x + row * (int64_t)c_i);
    const int nvec = c_i >> 3;
    float f[NV][8];
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            unpack8r<BF16>(__builtin_nontemporal_load(xr + idx), f[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += f[i][e];
        }
    }
    const float mean = wave_sum(sum) / (float)c_i;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = f[i][e] - mean;
                sq += d * d;
            }
        }
    }
    const float var = wave_sum(sq) / (float)c_i;
    const float rstd = 1.0f / sqrtf(var + eps);
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            const float4 g0 = *(const float4*)(gamma_f + idx * 8), g1 = *(const float4*)(gamma_f + idx * 8 + 4);
            const float4 b0 = *(const float4*)(beta_f + idx * 8), b1 = *(const float4*)(beta_f + idx * 8 + 4);
            const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
            const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                f[i][e] = (f[i][e] - mean) * rstd * g[e] + b[e];
                m = __builtin_fmaxf(m, __builtin_fabsf(f[i][e]));
            }
        }
    }
    const float a = wave_max(m);
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    if (lane == 0) scale[row] = a / 127.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            uint32_t q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = code_bits(f[i][e] * r);
            __builtin_nontemporal_store(pack8(q), (v2u*)code_dst(xq, row, idx * 8, c_i, tiled));
        }
    }
}

}  // namespace

extern "C" {

sq_status sq_softmax_quant_p(const void* s, sq_dtype dtype, int64_t rows, int64_t cols, int8_t* pq, void* stream)
{
    if (!s || !pq) return SQ_ERR_NULL;
    if (rows <= 0 || cols <= 0 || rows >= ((int64_t)1 << 31)) return SQ_ERR_SHAPE;
    if (dtype != SQ_F16 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (cols > 8 * 256 * 8) return SQ_ERR_UNSUPPORTED;  // rows up to 16384 scores
    if ((cols & 7) || !sq_aligned16(s) || !sq_aligned16(pq)) return SQ_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int nvec = (int)(cols >> 3);
    const uint16_t* sp = (const uint16_t*)s;
#define SQ_SM(BF, NV) sq_launch((softmax_quant_kernel<BF, NV>), dim3((unsigned)rows), dim3(256), 0, st, sp, (int)cols, pq)
#define SQ_SMW(BF, NV) sq_launch((softmax_quant_wave_kernel<BF, NV>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, sp, rows, (int)cols, pq)
    if (dtype == SQ_BF16) {
        if (nvec <= 64) SQ_SMW(true, 1); else if (nvec <= 128) SQ_SMW(true, 2); else if (nvec <= 256) SQ_SMW(true, 4);
        else if (nvec <= 512) SQ_SMW(true, 8); else if (nvec <= 1024) SQ_SM(true, 4); else SQ_SM(true, 8);
    } else {
        if (nvec <= 64) SQ_SMW(false, 1); else if (nvec <= 128) SQ_SMW(false, 2); else if (nvec <= 256) SQ_SMW(false, 4);
        else if (nvec <= 512) SQ_SMW(false, 8); else if (nvec <= 1024) SQ_SM(false, 4); else SQ_SM(false, 8);
    }
#undef SQ_SM
#undef SQ_SMW
    return sq_launch_status();
}

sq_status sq_ln_quantize(const void* x, sq_dtype dtype, int64_t t, int64_t c_i, const float* gamma_f, const float* beta_f,
                         float eps, float* scale, int8_t* xq, sq_layout xq_layout, void* stream)
{
    if (!x || !gamma_f || !beta_f || !scale || !xq) return SQ_ERR_NULL;
    if (t <= 0 || c_i <= 0 || t >= ((int64_t)1 << 31)) return SQ_ERR_SHAPE;
    if (dtype != SQ_F16 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (c_i > 8 * 256 * 8) return SQ_ERR_UNSUPPORTED;  // hidden sizes up to 16384
    if (xq_layout != SQ_ROW_MAJOR && xq_layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if (xq_layout == SQ_TILED && (c_i & 63)) return SQ_ERR_ALIGN;
    const bool tiled = xq_layout == SQ_TILED;
    if ((c_i & 15) || !sq_aligned16(x) || !sq_aligned16(xq) || !sq_aligned16(gamma_f) || !sq_aligned16(beta_f))
        return SQ_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int nvec = (int)(c_i >> 3);
    const uint16_t* xp = (const uint16_t*)x;
    // Measured choice: up to 2048 channels one row per wave; up to 8192 one row per 256-thread workgroup; wider rows
    // one row per 512-thread workgroup (more loads in flight per row, fewer registers per thread).
#define SQ_LN(BF, NV, NT) sq_launch((ln_quant_kernel<BF, NV, NT>), dim3((unsigned)t), dim3(NT), 0, st, xp, (int)c_i, gamma_f, beta_f, eps, scale, xq, tiled)
#define SQ_LNW(BF, NV) sq_launch((ln_quant_wave_kernel<BF, NV>), dim3((unsigned)((t + 3) / 4)), dim3(256), 0, st, xp, t, (int)c_i, gamma_f, beta_f, eps, scale, xq, tiled)
    if (dtype == SQ_BF16) {
        if (nvec <= 128) SQ_LNW(true, 2); else if (nvec <= 256) SQ_LNW(true, 4); else if (nvec <= 512) SQ_LN(true, 2, 256);
        else if (nvec <= 1024) SQ_LN(true, 4, 256); else if (nvec <= 1536) SQ_LN(true, 3, 512); else SQ_LN(true, 4, 512);
    } else {
        if (nvec <= 128) SQ_LNW(false, 2); else if (nvec <= 256) SQ_LNW(false, 4); else if (nvec <= 512) SQ_LN(false, 2, 256);
        else if (nvec <= 1024) SQ_LN(false, 4, 256); else if (nvec <= 1536) SQ_LN(false, 3, 512); else SQ_LN(false, 4, 512);
    }
#undef SQ_LN
#undef SQ_LNW
    return sq_launch_status();
}

}  // extern "C"

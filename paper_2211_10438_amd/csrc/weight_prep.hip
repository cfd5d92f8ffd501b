// Offline weight preparation, gfx950: the statistics of Eq. 4, the smoothed weight of Eq. 3 and its
// per-tensor quantization by Eq. 1, written transposed ([C_o, C_i], contraction index contiguous)
// for the GEMM.  One-off work per layer: kept simple, coalesced on both sides of the transpose.
#include "common.h"

namespace {

template <bool BF16> SQ_DEVICE void unpack8w(const v4u raw, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = load16_bits<BF16>(raw[e]);
        f[2 * e + 1] = load16_bits<BF16>(raw[e] >> 16);
    }
}

SQ_DEVICE float block_max_256w(float v, float* red)
{
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    const float r = __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
    __syncthreads();
    return r;
}

// out_j = max_n |W_jn| * (s ? s_j : 1); one workgroup per input channel j (row of W).
// If tensor_bits is given, also folds the row maxima into the tensor-wide maximum.
template <bool BF16>
__global__ __launch_bounds__(256) void weight_row_absmax_kernel(const uint16_t* __restrict__ w, int c_i, int c_o,
                                                               const float* __restrict__ s, float* row_out,
                                                               uint32_t* tensor_bits)
{
    __shared__ float red[4];
    const int nvec = c_o >> 3;
    for (int j = blockIdx.x; j < c_i; j += gridDim.x) {
        const v4u* wr = (const v4u*)(w + (int64_t)j * c_o);
        const float sj = s ? s[j] : 1.0f;
        float m = 0.0f;
        for (int idx = threadIdx.x; idx < nvec; idx += 256) {
            float f[8];
            unpack8w<BF16>(wr[idx], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(s ? f[e] * sj : f[e]));
        }
        m = block_max_256w(m, red);
        if (threadIdx.x == 0) {
            if (row_out) row_out[j] = m;
            if (tensor_bits) atomicMax(tensor_bits, __builtin_bit_cast(uint32_t, m));
        }
    }
}

__global__ void zero_u32_kernel(uint32_t* p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// Per-output-channel maxima: col_bits[n] = max_j |W_jn * s_j| as the bit pattern of a non-negative float
// (its integer order is the float order, so atomicMax is exact).  A thread owns 8 neighbouring columns and
// walks a slab of 64 rows; slabs are spread over blockIdx.y.
template <bool BF16>
__global__ __launch_bounds__(256) void weight_col_absmax_kernel(const uint16_t* __restrict__ w, int c_i, int c_o,
                                                               const float* __restrict__ s, uint32_t* col_bits)
{
    const int n = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (n >= c_o) return;  // c_o % 8 == 0
    const int j0 = blockIdx.y * 64, j1 = j0 + 64 < c_i ? j0 + 64 : c_i;
    float m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = j0; j < j1; ++j) {
        float f[8];
        unpack8w<BF16>(*(const v4u*)(w + (int64_t)j * c_o + n), f);
        const float sj = s ? s[j] : 1.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] = __builtin_fmaxf(m[e], __builtin_fabsf(s ? f[e] * sj : f[e]));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) atomicMax(col_bits + n + e, __builtin_bit_cast(uint32_t, m[e]));
}

// 64 (input channels) x 64 (output channels) tile: read along C_o, quantize, transpose through LDS,
// write along C_i.
template <bool BF16>
__global__ __launch_bounds__(256) void weight_quant_transpose_kernel(const uint16_t* __restrict__ w, int c_i, int c_o,
                                                                    const float* __restrict__ s,
                                                                    const uint32_t* amax_bits, float* w_scale,
                                                                    int8_t* __restrict__ wq, bool tiled, bool per_channel)
{
    __shared__ __attribute__((aligned(16))) int8_t tileT[64][80];  // [n][j], padded pitch
    const float a = __builtin_bit_cast(float, *amax_bits);  // per-tensor maximum (per_channel: unused)
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    const int j0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    if (per_channel) {  // amax_bits[n]: maximum of column n
        if (blockIdx.y == 0 && threadIdx.x < 64 && n0 + threadIdx.x < c_o)
            w_scale[n0 + threadIdx.x] = __builtin_bit_cast(float, amax_bits[n0 + threadIdx.x]) / 127.0f;
    } else if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        w_scale[0] = a / 127.0f;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int v = threadIdx.x + h * 256;  // 512 vectors: 64 rows x 8 vectors of 8 channels
        const int jl = v >> 3, nl = (v & 7) * 8;
        const int j = j0 + jl, n = n0 + nl;
        if (j < c_i && n < c_o) {  // c_o % 8 == 0: a vector is inside or outside as a whole
            float f[8];
            unpack8w<BF16>(*(const v4u*)(w + (int64_t)j * c_o + n), f);
            const float sj = s ? s[j] : 1.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float re = r;
                if (per_channel) {
                    const float an = __builtin_bit_cast(float, amax_bits[n + e]);
                    re = an > 0.0f ? 127.0f / an : 0.0f;
                }
                tileT[nl + e][jl] = (int8_t)round_code((s ? f[e] * sj : f[e]) * re);
            }
        }
    }
    __syncthreads();
    {
        const int nl = threadIdx.x >> 2, jc = (threadIdx.x & 3) * 16;
        const int n = n0 + nl, j = j0 + jc;
        if (n < c_o && j < c_i)  // c_i % 16 == 0
            *(v4u*)code_dst(wq, n, j, c_i, tiled) = *(const v4u*)&tileT[nl][jc];  // 16 codes = one chunk
    }
}

}  // namespace

extern "C" {

sq_status sq_weight_absmax_per_in_channel(const void* w, sq_dtype dtype, int64_t c_i, int64_t c_o, float* out,
                                          void* stream)
{
    if (!w || !out) return SQ_ERR_NULL;
    if (c_i <= 0 || c_o <= 0 || c_i >= ((int64_t)1 << 31) || c_o >= ((int64_t)1 << 31)) return SQ_ERR_SHAPE;
    if (dtype != SQ_F16 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if ((c_o & 7) || !sq_aligned16(w)) return SQ_ERR_ALIGN;
    const unsigned grid = (unsigned)(c_i < 65535 ? c_i : 65535);
    if (dtype == SQ_BF16)
        sq_launch(weight_row_absmax_kernel<true>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint16_t*)w, (int)c_i, (int)c_o, (const float*)nullptr, out, (uint32_t*)nullptr);
    else
        sq_launch(weight_row_absmax_kernel<false>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint16_t*)w, (int)c_i, (int)c_o, (const float*)nullptr, out, (uint32_t*)nullptr);
    return sq_launch_status();
}

sq_status sq_prepare_weight(const void* w, sq_dtype dtype, const float* s, int64_t c_i, int64_t c_o, int8_t* wq,
                            sq_layout wq_layout, float* w_scale, int w_scale_per_channel, void* workspace, size_t ws_bytes,
                            void* stream)
{
    if (!w || !wq || !w_scale) return SQ_ERR_NULL;
    if (c_i <= 0 || c_o <= 0 || c_i >= ((int64_t)1 << 31) || c_o >= ((int64_t)1 << 31)) return SQ_ERR_SHAPE;
    if (dtype != SQ_F16 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (wq_layout != SQ_ROW_MAJOR && wq_layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if ((c_i & 15) || (c_o & 7) || !sq_aligned16(w) || !sq_aligned16(wq)) return SQ_ERR_ALIGN;
    if (wq_layout == SQ_TILED && (c_i & 63)) return SQ_ERR_ALIGN;
    const bool tiled = wq_layout == SQ_TILED;
    const bool pc = w_scale_per_channel != 0;
    if (!workspace || ws_bytes < sizeof(uint32_t) * (pc ? (size_t)c_o : 1)) return SQ_ERR_WORKSPACE;
    if (((int64_t)((c_i + 63) / 64)) > 65535) return SQ_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    uint32_t* amax = (uint32_t*)workspace;
    const int64_t ncell = pc ? c_o : 1;
    sq_launch(zero_u32_kernel, dim3((unsigned)((ncell + 255) / 256 < 1024 ? (ncell + 255) / 256 : 1024)), dim3(256), 0, st, amax, ncell);
    const unsigned grid1 = (unsigned)(c_i < 4096 ? c_i : 4096);
    dim3 gridc((unsigned)((c_o / 8 + 255) / 256), (unsigned)((c_i + 63) / 64));
    dim3 grid2((unsigned)((c_o + 63) / 64), (unsigned)((c_i + 63) / 64));
    if (dtype == SQ_BF16) {
        if (pc) sq_launch(weight_col_absmax_kernel<true>, gridc, dim3(256), 0, st, (const uint16_t*)w, (int)c_i, (int)c_o, s, amax);
        else sq_launch(weight_row_absmax_kernel<true>, dim3(grid1), dim3(256), 0, st, (const uint16_t*)w, (int)c_i, (int)c_o, s, (float*)nullptr, amax);
        sq_launch(weight_quant_transpose_kernel<true>, grid2, dim3(256), 0, st, (const uint16_t*)w, (int)c_i, (int)c_o, s, amax, w_scale, wq, tiled, pc);
    } else {
        if (pc) sq_launch(weight_col_absmax_kernel<false>, gridc, dim3(256), 0, st, (const uint16_t*)w, (int)c_i, (int)c_o, s, amax);
        else sq_launch(weight_row_absmax_kernel<false>, dim3(grid1), dim3(256), 0, st, (const uint16_t*)w, (int)c_i, (int)c_o, s, (float*)nullptr, amax);
        sq_launch(weight_quant_transpose_kernel<false>, grid2, dim3(256), 0, st, (const uint16_t*)w, (int)c_i, (int)c_o, s, amax, w_scale, wq, tiled, pc);
    }
    return sq_launch_status();
}

}  // extern "C"

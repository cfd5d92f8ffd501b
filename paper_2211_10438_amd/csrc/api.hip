// Host-only entry points of the sqmi C ABI: status strings, the smoothing factors of Eq. 4
// (offline, O(C_i)), workspace sizing and the attention BMM dispatcher.
#include <math.h>

#include <atomic>
#include <chrono>

#include "common.h"

extern "C" size_t sq_quantize_workspace_bytes(void);
extern "C" size_t sq_gemm_workspace_bytes(int64_t t, int64_t c_i, int64_t c_o);
extern "C" sq_status sq_internal_bmm(const int8_t* a, const int8_t* b, int trans_b, float alpha, void* c, sq_dtype out,
                                     int64_t batch, int64_t m, int64_t n, int64_t k, int64_t stride_a, int64_t stride_b,
                                     int64_t stride_c, void* stream);

uint32_t sq_next_ticket()
{
    static std::atomic<uint32_t> counter{(uint32_t)std::chrono::steady_clock::now().time_since_epoch().count() * 2654435761u};
    uint32_t v = counter.fetch_add(1u, std::memory_order_relaxed) + 1u;
    return v ? v : counter.fetch_add(1u, std::memory_order_relaxed) + 1u;
}

extern "C" {

const char* sq_status_string(sq_status st)
{
    switch (st) {
        case SQ_OK: return "ok";
        case SQ_ERR_NULL: return "required pointer is NULL";
        case SQ_ERR_SHAPE: return "invalid dimension";
        case SQ_ERR_ALIGN: return "pointer or dimension not aligned to 16";
        case SQ_ERR_UNSUPPORTED: return "unsupported parameter";
        case SQ_ERR_WORKSPACE: return "workspace missing or too small";
        case SQ_ERR_HIP: return "HIP runtime error at launch";
    }
    return "unknown status";
}

sq_status sq_smooth_scales(const float* x_absmax, const float* w_absmax, float alpha, int64_t c_i, float* s,
                           float* inv_s)
{
    if (!x_absmax || !w_absmax || !s) return SQ_ERR_NULL;
    if (c_i <= 0) return SQ_ERR_SHAPE;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return SQ_ERR_UNSUPPORTED;
    const float floor_v = 1e-5f;
    for (int64_t j = 0; j < c_i; ++j) {
        const double ax = (double)(x_absmax[j] > floor_v ? x_absmax[j] : floor_v);
        const double aw = (double)(w_absmax[j] > floor_v ? w_absmax[j] : floor_v);
        const float sj = (float)(pow(ax, (double)alpha) / pow(aw, 1.0 - (double)alpha));
        s[j] = sj;
        if (inv_s) inv_s[j] = 1.0f / sj;
    }
    return SQ_OK;
}

size_t sq_tiled_bytes(int64_t rows, int64_t k)
{
    if (rows <= 0 || k <= 0 || (k & 63)) return 0;
    return (size_t)((rows + 15) / 16 * 16) * (size_t)k;
}

size_t sq_workspace_bytes(sq_op op, int64_t t, int64_t c_i, int64_t c_o)
{
    switch (op) {
        case SQ_OP_QUANTIZE_ACT: return sq_quantize_workspace_bytes();  // partial maxima of the O2 mode
        case SQ_OP_PREPARE_WEIGHT: return 16 + (c_o > 0 ? (size_t)c_o * sizeof(uint32_t) : 0);  // column maxima (per-channel steps)
        case SQ_OP_W8A8_LINEAR:
        case SQ_OP_I8_GEMM_I32: return sq_gemm_workspace_bytes(t, c_i, c_o);
        case SQ_OP_W8A8_BMM: return 0;
    }
    return 0;
}

sq_status sq_w8a8_bmm(const int8_t* a, const int8_t* bm, int trans_b, float alpha, void* c, sq_dtype out, int64_t b,
                      int64_t m, int64_t n, int64_t k, int64_t stride_a, int64_t stride_b, int64_t stride_c,
                      void* stream)
{
    if (!a || !bm || !c) return SQ_ERR_NULL;
    const int64_t lim = (int64_t)1 << 31;
    if (b <= 0 || m <= 0 || n <= 0 || k <= 0 || b > 65535 || m >= lim || n >= lim || k >= lim || 256 * k >= lim ||
        256 * n >= lim)
        return SQ_ERR_SHAPE;
    if (stride_a < m * k || stride_b < n * k || stride_c < m * n) return SQ_ERR_SHAPE;
    if (out != SQ_F16 && out != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if ((k & 15) || (stride_a & 15) || (stride_b & 15) || (stride_c & 7) || !sq_aligned16(a) || !sq_aligned16(bm) ||
        !sq_aligned16(c))
        return SQ_ERR_ALIGN;
    if (!trans_b && (n & 15)) return SQ_ERR_ALIGN;
    return sq_internal_bmm(a, bm, trans_b ? 1 : 0, alpha, c, out, b, m, n, k, stride_a, stride_b, stride_c, stream);
}

}  // extern "C"

// Measurement aid (not part of the method): an MFMA-only loop that shows what the INT8 matrix pipes of this
// chip sustain when they are fed from registers, with no memory traffic at all.  bench.py reports the GEMM
// against this figure next to the nominal peak, because under a sustained MFMA load the shader clock drops
// well below the 2.4 GHz the nominal 5.0 POP/s assumes.
#include "common.h"
#include "sqmi_probe.h"

namespace {

// 8 waves per workgroup (two per SIMD, like the prefill GEMM tiles), each with 16 independent 16x16 accumulator
// blocks (the MFMA shape of the compute-bound GEMM tiles) fed by six operand fragments taken once from `data` (so the
// operand bits are the caller's: random int8 codes toggle far more wires than zeros do, and the sustained clock depends
// on it): fragments 0..3 as one operand, 2..5 as the other.
__global__ __launch_bounds__(512, 1) void mfma_probe_kernel(const v4i* __restrict__ data, int iters, int* __restrict__ sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v4i f[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) f[i] = data[((blockIdx.x * 8 + wave) * 6 + i) * 64 + lane];
    v4i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f[2 + j], f[i], acc[i][j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) s += acc[i][j][v];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

extern "C" {

sq_status sq_probe_mfma_i8(const int8_t* data, size_t data_bytes, int workgroups, int iters, int32_t* sink, void* stream)
{
    if (!data || !sink) return SQ_ERR_NULL;
    if (workgroups <= 0 || workgroups > 65535 || iters <= 0) return SQ_ERR_SHAPE;
    if (data_bytes < (size_t)workgroups * 8 * 6 * 64 * 16) return SQ_ERR_WORKSPACE;
    if (!sq_aligned16(data) || !sq_aligned16(sink)) return SQ_ERR_ALIGN;
    sq_launch(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(512), 0, (hipStream_t)stream, (const v4i*)data, iters, sink);
    return sq_launch_status();
}

}  // extern "C"

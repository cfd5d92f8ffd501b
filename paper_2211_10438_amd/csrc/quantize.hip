// Activation quantization (Eq. 1) at the granularities of Table 2, gfx950.
//
// Per-token dynamic (O1): one pass over HBM.  A row lives in registers between the absmax
// reduction and the rounding, so the traffic is 2 B read + 1 B written per element.  Rows are
// handled by a 256-thread workgroup (wide rows) or by one 64-lane wave (narrow rows, reduction
// with cross-lane shuffles only).
// Per-tensor static (O3): pure elementwise pass, saturating.
// Per-tensor dynamic (O2): tensors of up to 512 x 16384 elements run as ONE ordinary launch and cross HBM once.
// Workgroup b loads its 16384 elements into registers, stores its absmax to partial[b] (plain store: nothing to
// clear), adds 1 to an arrival count and waits until the count reaches the grid size; then every workgroup reduces
// the partial maxima and quantizes its registers.  The grid is at most 512 workgroups (a quarter of what the
// device keeps resident; the occupancy query sizes it), so every workgroup gets a slot while the others wait; the
// wait is bounded all the same (spin limit; on expiry scale[0] = NaN and nothing is quantized), so every wave
// leaves the kernel whatever happens.  The arrival count carries a per-call ticket in its upper half, so a stale
// workspace counts as zero.  Same-address atomics cost about 30 ns each on this part and serialize, which is why
// larger tensors (more workgroups, and the second read served by the memory-side cache anyway), streams under HIP
// graph capture (a replay would reuse the ticket) and callers with a small workspace get the three-launch version
// (clear, absmax with atomic max on the float's bit pattern, quantize); results are identical.
#include "common.h"

namespace {

template <bool BF16> SQ_DEVICE void unpack8(const v4u raw, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = load16_bits<BF16>(raw[e]);
        f[2 * e + 1] = load16_bits<BF16>(raw[e] >> 16);
    }
}

// x_hat = fl32(x * inv_s_j) for the 8 channels starting at `col` (Eq. 3 applied to the activation).
SQ_DEVICE void smooth8(float (&f)[8], const float* inv_s, int col)
{
    const float4 a = *(const float4*)(inv_s + col);
    const float4 b = *(const float4*)(inv_s + col + 4);
    f[0] = f[0] * a.x; f[1] = f[1] * a.y; f[2] = f[2] * a.z; f[3] = f[3] * a.w;
    f[4] = f[4] * b.x; f[5] = f[5] * b.y; f[6] = f[6] * b.z; f[7] = f[7] * b.w;
}

SQ_DEVICE float absmax8(const float (&f)[8])
{
    float m = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(f[e]));
    return m;
}

SQ_DEVICE v2u quant8(const float (&f)[8], float r)
{
    v2u out;
#pragma unroll
    for (int h = 0; h < 2; ++h)
        out[h] = pack4_low_bytes(code_bits(f[4 * h] * r), code_bits(f[4 * h + 1] * r), code_bits(f[4 * h + 2] * r),
                                 code_bits(f[4 * h + 3] * r));
    return out;
}

// Block-wide max for a workgroup of NT threads (NT / 64 waves).
template <int NT> SQ_DEVICE float block_max(float v, float* red)
{
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) m = __builtin_fmaxf(m, red[w]);
    return m;
}
SQ_DEVICE float block_max_256(float v, float* red) { return block_max<256>(v, red); }

// One row per workgroup of NT threads; NV 16-byte vectors (8 elements) per thread kept in registers.
// KEEP: the smoothed fp32 values stay in registers between the two phases (worth it while NV is small);
// otherwise x * inv_s is evaluated again in the second phase -- the same fp32 product, hence the same code.
template <bool BF16, int NV, int NT, bool KEEP>
__global__ __launch_bounds__(NT) void quant_per_token_block(const uint16_t* __restrict__ x, int64_t ldx, int c_i,
                                                           const float* __restrict__ inv_s, float* __restrict__ scale,
                                                           int8_t* __restrict__ xq, bool tiled)
{
    __shared__ float red[NT / 64];
    const int64_t row = blockIdx.x;
    const v4u* xr = (const v4u*)(x + row * ldx);
    const int nvec = c_i >> 3;
    v4u raw[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        raw[i] = idx < nvec ? __builtin_nontemporal_load(xr + idx) : v4u{0, 0, 0, 0};
    }
    float kept[KEEP ? NV : 1][8];
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        float f[8];
        unpack8<BF16>(raw[i], f);
        if (inv_s && idx < nvec) smooth8(f, inv_s, idx * 8);
        m = __builtin_fmaxf(m, absmax8(f));
        if constexpr (KEEP) {
#pragma unroll
            for (int e = 0; e < 8; ++e) kept[i][e] = f[e];
        }
    }
    const float a = block_max<NT>(m, red);
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    if (threadIdx.x == 0) scale[row] = a / 127.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        if (idx < nvec) {
            float f[8];
            if constexpr (KEEP) {
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] = kept[i][e];
            } else {
                unpack8<BF16>(raw[i], f);
                if (inv_s) smooth8(f, inv_s, idx * 8);
            }
            __builtin_nontemporal_store(quant8(f, r), (v2u*)code_dst(xq, row, idx * 8, c_i, tiled));
        }
    }
}

// Two rows per workgroup for inputs that take smoothing factors: the 4 * c_i bytes of fp32 factors a row needs are
// twice the row's own 2 * c_i bytes, so reading them once for two rows takes a third off what a workgroup pulls
// through its compute unit.  Both rows are in flight together (not one after the other), the products x * inv_s stay
// in registers between the reduction and the rounding.
template <bool BF16, int NV, int NT>
__global__ __launch_bounds__(NT) void quant_per_token_block2(const uint16_t* __restrict__ x, int64_t ldx, int c_i, int64_t t,
                                                            const float* __restrict__ inv_s, float* __restrict__ scale,
                                                            int8_t* __restrict__ xq, bool tiled)
{
    __shared__ float red[2][NT / 64];
    const int64_t row0 = (int64_t)blockIdx.x * 2;
    const bool two = row0 + 1 < t;
    const v4u* xr0 = (const v4u*)(x + row0 * ldx);
    const v4u* xr1 = (const v4u*)(x + (two ? row0 + 1 : row0) * ldx);
    const int nvec = c_i >> 3;
    v4u raw0[NV], raw1[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        raw0[i] = idx < nvec ? __builtin_nontemporal_load(xr0 + idx) : v4u{0, 0, 0, 0};
        raw1[i] = idx < nvec ? __builtin_nontemporal_load(xr1 + idx) : v4u{0, 0, 0, 0};
    }
    float k0[NV][8], k1[NV][8];
    float m0 = 0.0f, m1 = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        unpack8<BF16>(raw0[i], k0[i]);
        unpack8<BF16>(raw1[i], k1[i]);
        if (idx < nvec) {
            const float4 a = *(const float4*)(inv_s + idx * 8);
            const float4 b = *(const float4*)(inv_s + idx * 8 + 4);
            const float s8[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                k0[i][e] = k0[i][e] * s8[e];
                k1[i][e] = k1[i][e] * s8[e];
            }
        }
        m0 = __builtin_fmaxf(m0, absmax8(k0[i]));
        m1 = __builtin_fmaxf(m1, absmax8(k1[i]));
    }
    m0 = wave_max(m0);
    m1 = wave_max(m1);
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = m0;
        red[1][threadIdx.x >> 6] = m1;
    }
    __syncthreads();
    float a0 = red[0][0], a1 = red[1][0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) {
        a0 = __builtin_fmaxf(a0, red[0][w]);
        a1 = __builtin_fmaxf(a1, red[1][w]);
    }
    const float r0 = a0 > 0.0f ? 127.0f / a0 : 0.0f, r1 = a1 > 0.0f ? 127.0f / a1 : 0.0f;
    if (threadIdx.x == 0) {
        scale[row0] = a0 / 127.0f;
        if (two) scale[row0 + 1] = a1 / 127.0f;
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = threadIdx.x + i * NT;
        if (idx < nvec) {
            __builtin_nontemporal_store(quant8(k0[i], r0), (v2u*)code_dst(xq, row0, idx * 8, c_i, tiled));
            if (two) __builtin_nontemporal_store(quant8(k1[i], r1), (v2u*)code_dst(xq, row0 + 1, idx * 8, c_i, tiled));
        }
    }
}

// One row per wave (4 rows per workgroup): for narrow rows.
template <bool BF16, int NV>
__global__ __launch_bounds__(256) void quant_per_token_wave(const uint16_t* __restrict__ x, int64_t ldx, int c_i, int64_t t,
                                                           const float* __restrict__ inv_s, float* __restrict__ scale,
                                                           int8_t* __restrict__ xq, bool tiled)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= t) return;
    const v4u* xr = (const v4u*)(x + row * ldx);
    const int nvec = c_i >> 3;
    v4u raw[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        raw[i] = idx < nvec ? xr[idx] : v4u{0, 0, 0, 0};
    }
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        float f[8];
        unpack8<BF16>(raw[i], f);
        if (inv_s && idx < nvec) smooth8(f, inv_s, idx * 8);
        m = __builtin_fmaxf(m, absmax8(f));
    }
    const float a = wave_max(m);
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    if (lane == 0) scale[row] = a / 127.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            float f[8];
            unpack8<BF16>(raw[i], f);
            if (inv_s) smooth8(f, inv_s, idx * 8);
            *(v2u*)code_dst(xq, row, idx * 8, c_i, tiled) = quant8(f, r);
        }
    }
}

// Rows wider than the register-resident variants cover: two passes over the row (second one is
// served by the caches for any realistic width).
template <bool BF16>
__global__ __launch_bounds__(256) void quant_per_token_stream(const uint16_t* __restrict__ x, int64_t ldx, int c_i,
                                                             const float* __restrict__ inv_s, float* __restrict__ scale,
                                                             int8_t* __restrict__ xq, bool tiled)
{
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const v4u* xr = (const v4u*)(x + row * ldx);
    const int nvec = c_i >> 3;
    float m = 0.0f;
    for (int idx = threadIdx.x; idx < nvec; idx += 256) {
        float f[8];
        unpack8<BF16>(xr[idx], f);
        if (inv_s) smooth8(f, inv_s, idx * 8);
        m = __builtin_fmaxf(m, absmax8(f));
    }
    const float a = block_max_256(m, red);
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    if (threadIdx.x == 0) scale[row] = a / 127.0f;
    for (int idx = threadIdx.x; idx < nvec; idx += 256) {
        float f[8];
        unpack8<BF16>(xr[idx], f);
        if (inv_s) smooth8(f, inv_s, idx * 8);
        *(v2u*)code_dst(xq, row, idx * 8, c_i, tiled) = quant8(f, r);
    }
}

// ---- per-tensor

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// absmax over the whole [t, c_i] tensor -> *amax_bits (bit pattern of a non-negative float; the
// integer order of such patterns is the float order, so atomicMax on uint32 is exact).
template <bool BF16>
__global__ __launch_bounds__(256) void tensor_absmax_kernel(const uint16_t* __restrict__ x, int64_t ldx, int c_i, int64_t t,
                                                           const float* __restrict__ inv_s, uint32_t* amax_bits)
{
    __shared__ float red[4];
    const int nvec = c_i >> 3;
    const int64_t total = t * (int64_t)nvec;
    float m = 0.0f;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (int64_t)gridDim.x * 256) {
        const int64_t row = g / nvec;
        const int idx = (int)(g - row * nvec);
        float f[8];
        unpack8<BF16>(((const v4u*)(x + row * ldx))[idx], f);
        if (inv_s) smooth8(f, inv_s, idx * 8);
        m = __builtin_fmaxf(m, absmax8(f));
    }
    m = block_max_256(m, red);
    if (threadIdx.x == 0) atomicMax(amax_bits, __builtin_bit_cast(uint32_t, m));
}

// Elementwise quantization with one step for the whole tensor.  DYNAMIC: the step comes from the
// absmax pass (and is written to scale[0]); otherwise scale[0] holds the calibrated Delta.
template <bool BF16, bool DYNAMIC>
__global__ __launch_bounds__(256) void quant_per_tensor_kernel(const uint16_t* __restrict__ x, int64_t ldx, int c_i, int64_t t,
                                                              const float* __restrict__ inv_s, float* scale,
                                                              const uint32_t* amax_bits, int8_t* __restrict__ xq, bool tiled)
{
    float r;
    if (DYNAMIC) {
        const float a = __builtin_bit_cast(float, *amax_bits);
        r = a > 0.0f ? 127.0f / a : 0.0f;
        if (blockIdx.x == 0 && threadIdx.x == 0) scale[0] = a / 127.0f;
    } else {
        const float delta = scale[0];
        r = delta > 0.0f ? 1.0f / delta : 0.0f;
    }
    const int nvec = c_i >> 3;
    const int64_t total = t * (int64_t)nvec;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (int64_t)gridDim.x * 256) {
        const int64_t row = g / nvec;
        const int idx = (int)(g - row * nvec);
        float f[8];
        unpack8<BF16>(__builtin_nontemporal_load((const v4u*)(x + row * ldx) + idx), f);
        if (inv_s) smooth8(f, inv_s, idx * 8);
        __builtin_nontemporal_store(quant8(f, r), (v2u*)code_dst(xq, row, idx * 8, c_i, tiled));
    }
}

constexpr int kO2MaxGrid = 512;  // workgroups of the single-launch kernel (= partial maxima in the workspace)

// Workspace layout: bytes [0, 8) arrival cell {ticket : count}; bytes [256, 256 + 4 * kO2MaxGrid) partial maxima.
// spin_limit bounds the wait (0.5 to 2 us per poll); it is not reached unless a workgroup of the grid never gets to
// run, and if it is, scale[0] becomes NaN and nothing is quantized: every wave still leaves the kernel.
template <bool BF16, int NV>
__global__ __launch_bounds__(256) void quant_per_tensor_single_kernel(const uint16_t* __restrict__ x, int64_t ldx, int c_i, int64_t t,
                                                                     const float* __restrict__ inv_s, float* scale,
                                                                     unsigned char* ws, uint32_t ticket, uint32_t spin_limit,
                                                                     int8_t* __restrict__ xq, bool tiled)
{
    __shared__ float red[4];
    __shared__ uint32_t ok_flag;
    unsigned long long* cell = (unsigned long long*)ws;
    uint32_t* partial = (uint32_t*)(ws + 256);
    const int nvec = c_i >> 3;
    const int64_t total = t * (int64_t)nvec;
    const int64_t g0 = (int64_t)blockIdx.x * (256 * NV) + threadIdx.x;
    v4u raw[NV];
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int64_t g = g0 + i * 256;
        raw[i] = v4u{0, 0, 0, 0};
        if (g < total) {
            const int64_t row = g / nvec;
            const int idx = (int)(g - row * nvec);
            raw[i] = __builtin_nontemporal_load((const v4u*)(x + row * ldx) + idx);
            float f[8];
            unpack8<BF16>(raw[i], f);
            if (inv_s) smooth8(f, inv_s, idx * 8);
            m = __builtin_fmaxf(m, absmax8(f));
        }
    }
    m = block_max_256(m, red);
    if (threadIdx.x == 0) {
        __hip_atomic_store(partial + blockIdx.x, __builtin_bit_cast(uint32_t, m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ticket_open(cell, ticket);
        // release: the partial maximum above is visible device-wide before the count moves
        __hip_atomic_fetch_add(cell, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t spins = 0;
        bool ok = true;
        while ((uint32_t)__hip_atomic_load(cell, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < gridDim.x) {
            if (++spins > spin_limit) { ok = false; break; }
            if (spins < 16) __builtin_amdgcn_s_sleep(16); else __builtin_amdgcn_s_sleep(64);
        }
        ok_flag = ok ? 1u : 0u;
    }
    __syncthreads();
    if (!ok_flag) {  // the wait gave up (see above)
        if (threadIdx.x == 0) scale[0] = __builtin_nanf("");
        return;
    }
    float a = 0.0f;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += 256)
        a = __builtin_fmaxf(a, __builtin_bit_cast(float, __hip_atomic_load(partial + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
    __syncthreads();  // `red` is reused
    a = block_max_256(a, red);
    const float r = a > 0.0f ? 127.0f / a : 0.0f;
    if (blockIdx.x == 0 && threadIdx.x == 0) scale[0] = a / 127.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int64_t g = g0 + i * 256;
        if (g < total) {
            const int64_t row = g / nvec;
            const int idx = (int)(g - row * nvec);
            float f[8];
            unpack8<BF16>(raw[i], f);
            if (inv_s) smooth8(f, inv_s, idx * 8);
            __builtin_nontemporal_store(quant8(f, r), (v2u*)code_dst(xq, row, idx * 8, c_i, tiled));
        }
    }
}

// Per-channel calibration statistic: out_j = max_t |x_tj| (bit patterns, see above).
template <bool BF16>
__global__ __launch_bounds__(256) void act_absmax_per_channel_kernel(const uint16_t* __restrict__ x, int c_i, int64_t t,
                                                                    uint32_t* out_bits)
{
    const int nvec = c_i >> 3;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= nvec) return;
    float m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int64_t row = blockIdx.y; row < t; row += gridDim.y) {
        float f[8];
        unpack8<BF16>(((const v4u*)(x + row * (int64_t)c_i))[idx], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] = __builtin_fmaxf(m[e], __builtin_fabsf(f[e]));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) atomicMax(out_bits + idx * 8 + e, __builtin_bit_cast(uint32_t, m[e]));
}

template <bool BF16>
void launch_per_token(const uint16_t* x, int64_t ldx, int c_i, int64_t t, const float* inv_s, float* scale, int8_t* xq,
                      bool tiled, hipStream_t st)
{
    const int nvec = c_i >> 3;
#define SQ_WAVE(NV) sq_launch((quant_per_token_wave<BF16, NV>), dim3((unsigned)((t + 3) / 4)), dim3(256), 0, st, x, ldx, c_i, t, inv_s, scale, xq, tiled)
#define SQ_BLOCK(NV, NT)                                                                                                        \
    do {                                                                                                                        \
        if (inv_s && NV <= 6) sq_launch((quant_per_token_block<BF16, NV, NT, true>), dim3((unsigned)t), dim3(NT), 0, st, x, ldx, c_i, inv_s, scale, xq, tiled); \
        else sq_launch((quant_per_token_block<BF16, NV, NT, false>), dim3((unsigned)t), dim3(NT), 0, st, x, ldx, c_i, inv_s, scale, xq, tiled);                 \
    } while (0)
    if (nvec <= 64) SQ_WAVE(1);
    else if (nvec <= 128) SQ_WAVE(2);
    else if (nvec <= 256) SQ_BLOCK(1, 256);
    else if (nvec <= 512) SQ_BLOCK(2, 256);
    else if (nvec <= 1024) SQ_BLOCK(4, 256);
    // workgroup sizes that divide the row evenly (every thread the same number of vectors) measure 4-12 % faster
    // than the next power of two: the hidden sizes 9216 and 12288 and the 36864-wide FFN of the former
    // (with smoothing factors the 12288-wide row takes two rows per workgroup: 18.6 against 20.9 us at 2048 rows;
    //  the 9216-wide row measured no gain from it)
    else if (nvec == 1536 && inv_s) sq_launch((quant_per_token_block2<BF16, 2, 768>), dim3((unsigned)((t + 1) / 2)), dim3(768), 0, st, x, ldx, c_i, t, inv_s, scale, xq, tiled);
    else if (nvec == 1152) SQ_BLOCK(2, 576);
    else if (nvec == 1536) SQ_BLOCK(2, 768);
    else if (nvec == 4608) SQ_BLOCK(6, 768);
    else if (nvec <= 2048) SQ_BLOCK(2, 1024);  // measured: from 8192 channels on, 1024 threads per row beat 256
    else if (nvec <= 4096) SQ_BLOCK(4, 1024);
    else if (nvec <= 6144) SQ_BLOCK(6, 1024);
    else if (nvec <= 8192) SQ_BLOCK(8, 1024);
    else sq_launch((quant_per_token_stream<BF16>), dim3((unsigned)t), dim3(256), 0, st, x, ldx, c_i, inv_s, scale, xq, tiled);
#undef SQ_WAVE
#undef SQ_BLOCK
}

int grid_for(int64_t work_items)
{
    int64_t blocks = (work_items + 255) / 256;
    const int64_t cap = 256 * 16;
    return (int)(blocks < 1 ? 1 : (blocks > cap ? cap : blocks));
}

constexpr int kO2NV = 8;  // 16-byte vectors a thread holds: a workgroup covers 256 x 8 x 8 = 16384 elements

// Largest grid of the single-launch kernel: a quarter of the workgroups the device keeps resident (occupancy x
// compute units), at most kO2MaxGrid.
template <bool BF16> int single_launch_grid()
{
    static int limit = -1;
    if (limit < 0) {
        int dev = 0, cus = 0, per_cu = 0;
        limit = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0 &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, quant_per_tensor_single_kernel<BF16, kO2NV>, 256, 0) == hipSuccess &&
            per_cu > 0)
            limit = cus * per_cu / 4 < kO2MaxGrid ? cus * per_cu / 4 : kO2MaxGrid;
    }
    return limit;
}

}  // namespace

extern "C" {

// Workspace of the per-tensor dynamic mode: arrival cell + partial maxima of the single-launch kernel.
size_t sq_quantize_workspace_bytes(void) { return 256 + kO2MaxGrid * sizeof(uint32_t); }

sq_status sq_quantize_act(const void* x, sq_dtype dtype, int64_t t, int64_t c_i, int64_t ldx, const float* inv_s,
                          sq_act_mode mode, float* scale, int8_t* xq, sq_layout xq_layout, void* workspace,
                          size_t ws_bytes, void* stream)
{
    if (!x || !scale || !xq) return SQ_ERR_NULL;
    if (t <= 0 || c_i <= 0 || ldx < c_i || t >= ((int64_t)1 << 31) || c_i >= ((int64_t)1 << 31)) return SQ_ERR_SHAPE;
    if (dtype != SQ_F16 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (mode != SQ_PER_TOKEN_DYNAMIC && mode != SQ_PER_TENSOR_DYNAMIC && mode != SQ_PER_TENSOR_STATIC)
        return SQ_ERR_UNSUPPORTED;
    if (xq_layout != SQ_ROW_MAJOR && xq_layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if (xq_layout == SQ_TILED && (c_i & 63)) return SQ_ERR_ALIGN;
    const bool tiled = xq_layout == SQ_TILED;
    if ((c_i & 15) || (ldx & 7) || !sq_aligned16(x) || !sq_aligned16(xq) || (inv_s && !sq_aligned16(inv_s)))
        return SQ_ERR_ALIGN;
    if (mode == SQ_PER_TENSOR_DYNAMIC && (!workspace || ws_bytes < sizeof(uint32_t))) return SQ_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const uint16_t* xp = (const uint16_t*)x;
    const bool bf = dtype == SQ_BF16;
    if (mode == SQ_PER_TOKEN_DYNAMIC) {
        if (bf) launch_per_token<true>(xp, ldx, (int)c_i, t, inv_s, scale, xq, tiled, st);
        else launch_per_token<false>(xp, ldx, (int)c_i, t, inv_s, scale, xq, tiled, st);
        return sq_launch_status();
    }
    const int grid = grid_for(t * (c_i >> 3));
    if (mode == SQ_PER_TENSOR_DYNAMIC) {
        uint32_t* amax = (uint32_t*)workspace;
        const int64_t vecs = t * (c_i >> 3);
        const int64_t nwg = (vecs + 256 * kO2NV - 1) / (256 * kO2NV);  // workgroups that hold the whole tensor in registers
        const int limit = bf ? single_launch_grid<true>() : single_launch_grid<false>();
        // A stream that is being captured into a HIP graph records the three-launch version: a replay would reuse
        // the ticket.
        hipStreamCaptureStatus cap = hipStreamCaptureStatusActive;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess) cap = hipStreamCaptureStatusActive;
        if (cap == hipStreamCaptureStatusNone && nwg <= limit && ws_bytes >= sq_quantize_workspace_bytes() &&
            (reinterpret_cast<uintptr_t>(workspace) & 15u) == 0) {
            const uint32_t ticket = sq_next_ticket(), spin_limit = 1u << 21;
            if (bf) sq_launch((quant_per_tensor_single_kernel<true, kO2NV>), dim3((unsigned)nwg), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, scale, (unsigned char*)workspace, ticket, spin_limit, xq, tiled);
            else sq_launch((quant_per_tensor_single_kernel<false, kO2NV>), dim3((unsigned)nwg), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, scale, (unsigned char*)workspace, ticket, spin_limit, xq, tiled);
            return sq_launch_status();
        }
        sq_launch(fill_u32_kernel, dim3(1), dim3(64), 0, st, amax, 0u, 1);
        if (bf) {
            sq_launch(tensor_absmax_kernel<true>, dim3(grid), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, amax);
            sq_launch((quant_per_tensor_kernel<true, true>), dim3(grid), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, scale, amax, xq, tiled);
        } else {
            sq_launch(tensor_absmax_kernel<false>, dim3(grid), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, amax);
            sq_launch((quant_per_tensor_kernel<false, true>), dim3(grid), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, scale, amax, xq, tiled);
        }
    } else {
        if (bf) sq_launch((quant_per_tensor_kernel<true, false>), dim3(grid), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, scale, (const uint32_t*)nullptr, xq, tiled);
        else sq_launch((quant_per_tensor_kernel<false, false>), dim3(grid), dim3(256), 0, st, xp, ldx, (int)c_i, t, inv_s, scale, (const uint32_t*)nullptr, xq, tiled);
    }
    return sq_launch_status();
}

sq_status sq_act_absmax_per_channel(const void* x, sq_dtype dtype, int64_t t, int64_t c_i, float* out, void* stream)
{
    if (!x || !out) return SQ_ERR_NULL;
    if (t <= 0 || c_i <= 0 || t >= ((int64_t)1 << 31) || c_i >= ((int64_t)1 << 31)) return SQ_ERR_SHAPE;
    if (dtype != SQ_F16 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if ((c_i & 15) || !sq_aligned16(x) || !sq_aligned16(out)) return SQ_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    sq_launch(fill_u32_kernel, dim3((unsigned)((c_i + 255) / 256)), dim3(256), 0, st, (uint32_t*)out, 0u, (int)c_i);
    const int nvec = (int)(c_i >> 3);
    dim3 grid((unsigned)((nvec + 255) / 256), (unsigned)(t < 256 ? t : 256));
    if (dtype == SQ_BF16)
        sq_launch(act_absmax_per_channel_kernel<true>, grid, dim3(256), 0, st, (const uint16_t*)x, (int)c_i, t, (uint32_t*)out);
    else
        sq_launch(act_absmax_per_channel_kernel<false>, grid, dim3(256), 0, st, (const uint16_t*)x, (int)c_i, t, (uint32_t*)out);
    return sq_launch_status();
}

}  // extern "C"

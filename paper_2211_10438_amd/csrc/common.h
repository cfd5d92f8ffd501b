// Shared host/device helpers of the sqmi HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sqmi.h"

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

#define SQ_DEVICE static __device__ __forceinline__

// ---- 16-bit formats.  fp16 uses the hardware converts (round-to-nearest-even in the default
// mode); bf16 is widened by a shift and narrowed with the integer nearest-even rule.
SQ_DEVICE float f16_bits_to_f32(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }
SQ_DEVICE float bf16_bits_to_f32(uint32_t b) { return __builtin_bit_cast(float, b << 16); }
SQ_DEVICE uint32_t f32_to_f16_bits(float v) { return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v); }
SQ_DEVICE uint32_t f32_to_bf16_bits(float v)
{
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
template <bool BF16> SQ_DEVICE float load16_bits(uint32_t bits)
{
    return BF16 ? bf16_bits_to_f32(bits & 0xffffu) : f16_bits_to_f32(bits & 0xffffu);
}
template <bool BF16> SQ_DEVICE uint32_t store16_bits(float v)
{
    return BF16 ? f32_to_bf16_bits(v) : f32_to_f16_bits(v);
}

// Eq. 1 rounding and range: round-half-even of v, saturated to [-127, 127], as an int.
SQ_DEVICE int round_code(float v)
{
    float r = __builtin_rintf(v);
    r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// The same rounding with the code left in the low byte of a word (two's complement), three instructions:
// clamp to +-127 (v_med3_f32; clamping before or after rounding gives the same integer), then add 1.5 * 2^23:
// the adder's own round-to-nearest-even leaves the integer in the low mantissa bits.
SQ_DEVICE uint32_t code_bits(float v)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_fmed3f(v, -127.0f, 127.0f) + 12582912.0f);
}
// Low bytes of four words -> one word (byte e from word e), three v_perm_b32.
SQ_DEVICE uint32_t pack4_low_bytes(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3)
{
    const uint32_t lo = __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u), hi = __builtin_amdgcn_perm(b3, b2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Byte offset of element (r, c) of an int8 [rows, k] operand in the SQ_TILED layout (see sqmi.h).
SQ_DEVICE int64_t tiled_offset(int64_t r, int c, int k)
{
    const int rr = (int)(r & 15);
    const int sw = ((rr >> 1) & 3) ^ ((rr >> 3) & 1);
    return ((r >> 4) * (int64_t)(k >> 6) + (c >> 6)) * 1024 + rr * 64 + ((((c >> 4) & 3) ^ sw) << 4) + (c & 15);
}
// Destination of the codes starting at column c of row r (c % 8 == 0: 8 codes never straddle a chunk).
SQ_DEVICE int8_t* code_dst(int8_t* base, int64_t r, int c, int k, bool tiled)
{
    return base + (tiled ? tiled_offset(r, c, k) : r * (int64_t)k + c);
}

// Wave-wide max over 64 lanes (all lanes receive the result).
SQ_DEVICE float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
SQ_DEVICE float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---- host side
static inline bool sq_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline sq_status sq_launch_status()
{
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_HIP;
}

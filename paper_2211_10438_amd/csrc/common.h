// Shared host/device helpers of the sqmi HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>
#include <type_traits>

#include "sqmi.h"

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

#define SQ_DEVICE static __device__ __forceinline__

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose index is a constant
// expression inside the body (builtins that take immediates, register arrays indexed modulo something).
template <int... I, class F> SQ_DEVICE void static_for_impl(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> SQ_DEVICE void static_for(F&& f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

// ---- 16-bit formats.  fp16 uses the hardware converts (round-to-nearest-even in the default
// mode); bf16 is widened by a shift and narrowed with the integer nearest-even rule.
SQ_DEVICE float f16_bits_to_f32(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }
SQ_DEVICE float bf16_bits_to_f32(uint32_t b) { return __builtin_bit_cast(float, b << 16); }
// The value is made opaque before it is narrowed: left alone, the compiler merges a multiply or add that feeds a
// float -> half conversion into v_fma_mixlo_f16, which rounds the exact result once to fp16.  The arithmetic fixed for
// the outputs is "round to fp32, then round to the 16-bit type"; the two differ whenever the fp32 rounding lands on
// an fp16 tie point (about one output in 2^13).  (The barrier is an empty asm statement on purpose: the conversion
// itself stays an instruction the compiler schedules, so it also inserts the wait states the hardware wants between
// a transcendental result and its use; an asm v_cvt_f16_f32 fed directly by v_exp_f32 read garbage.)
SQ_DEVICE uint32_t f32_to_f16_bits(float v)
{
    asm("" : "+v"(v));
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v);
}
// bf16: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32, round-to-nearest-even like the integer rule
// u + 0x7fff + ((u >> 16) & 1) it replaces: one instruction for two values instead of three per value).
SQ_DEVICE uint32_t f32_to_bf16_bits(float v) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)v); }

// Two values narrowed at once (lo in bits 0..15): v_cvt_pk_f16_f32 / v_cvt_pk_bf16_f32.
typedef float sq_f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 sq_f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 sq_bf16x2 __attribute__((ext_vector_type(2)));
template <bool BF16> SQ_DEVICE uint32_t store16x2_bits(float lo, float hi)
{
    if constexpr (BF16) {
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(sq_f32x2{lo, hi}, sq_bf16x2));
    } else {
        asm("" : "+v"(lo));  // see f32_to_f16_bits
        asm("" : "+v"(hi));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(sq_f32x2{lo, hi}, sq_f16x2));
    }
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

// ---- ticketed 64-bit cells {ticket : value} in caller-owned scratch that nobody clears.  A cell whose upper half is
// not this call's ticket is stale: the first workgroup that sees it so replaces it by {ticket : 0} (one compare-and-
// swap; it fails only if another workgroup of the same call was faster, which is just as good).  After that the
// cell is updated with the hardware's 64-bit add / max, which never touch the ticket half.
SQ_DEVICE void ticket_open(unsigned long long* cell, uint32_t ticket)
{
    unsigned long long v = __hip_atomic_load(cell, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)(v >> 32) != ticket)
        __hip_atomic_compare_exchange_strong(cell, &v, (unsigned long long)ticket << 32, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
}

// ---- host side
// Ticket of one call that uses ticketed cells: a per-process counter started from the clock, never 0.
uint32_t sq_next_ticket();
static inline bool sq_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launch bookkeeping of one entry point, per host thread.  Every kernel of the library is launched through
// sq_launch, which keeps the status hipLaunchKernel itself returned for this launch (an error left behind by an
// unrelated earlier HIP call of the application is neither reported as ours nor cleared) and launches nothing
// more once a launch of the entry point has failed.  sq_launch_status closes the entry point: it returns that
// status and resets it for the next call.
inline thread_local hipError_t sq_tls_launch_error = hipSuccess;

template <typename... P, typename... A>
static inline void sq_launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st, A&&... args)
{
    static_assert(sizeof...(P) == sizeof...(A), "kernel argument count");
    if (sq_tls_launch_error != hipSuccess) return;
    std::tuple<std::decay_t<P>...> vals{static_cast<std::decay_t<P>>(args)...};
    std::apply(
        [&](auto&... v) {
            void* argv[] = {(void*)&v...};
            sq_tls_launch_error = hipLaunchKernel((const void*)kernel, grid, block, argv, lds_bytes, st);
        },
        vals);
}
static inline sq_status sq_launch_status()
{
    const hipError_t e = sq_tls_launch_error;
    sq_tls_launch_error = hipSuccess;
    return e == hipSuccess ? SQ_OK : SQ_ERR_HIP;
}

// Small device-side helpers: bf16 conversion, wavefront reductions, fault reporting.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "preserve.h"

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Round to nearest, ties to even.  NaN stays NaN (quiet bit forced).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Two floats -> two bf16 in one dword (lo in the low half).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

typedef __bf16 ps_bf16x2 __attribute__((ext_vector_type(2)));
typedef float ps_f32x2 __attribute__((ext_vector_type(2)));
// Two floats -> packed bf16 pair with the hardware conversion (round to nearest even).
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
    ps_f32x2 f = {lo, hi};
    ps_bf16x2 b = __builtin_convertvector(f, ps_bf16x2);
    return *reinterpret_cast<uint32_t*>(&b);
}

// XOR swizzle of the 16-byte chunks of a 128-byte LDS row: chunk c of row r lives at position
// c ^ lds_swz(r).  Any 8 consecutive rows, and any 16 consecutive rows taken modulo two rows, then
// fall in different banks for a 16-byte read per lane.  Depends on r mod 16 only.
__device__ __forceinline__ int lds_swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Record a fault found in device data: OR the flag, keep the smallest index.  first_bad holds
// (2^62 - index) so that a maximum over a zero-initialised word finds the smallest index.
// Faults are exceptional, so the two atomics are off the fast path.
__device__ __forceinline__ void report_fault(ps_status* st, int flag, int64_t index) {
    if (!st) return;
    atomicOr(&st->flags, flag);
    atomicMax((long long*)&st->first_bad, (long long)(((int64_t)1 << 62) - index));
}

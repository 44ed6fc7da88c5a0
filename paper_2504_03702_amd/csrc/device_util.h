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

// Four consecutive int32 (16-byte aligned) that will not be read again: the non-temporal hint keeps a stream
// from displacing what the caches hold (a read-only pass over 529 MB ran at 6.7 TB/s with it, 6.0 without).
__device__ __forceinline__ int4 load_stream_int4(const int32_t* p) {
    int4 v;
    v.x = __builtin_nontemporal_load(p);
    v.y = __builtin_nontemporal_load(p + 1);
    v.z = __builtin_nontemporal_load(p + 2);
    v.w = __builtin_nontemporal_load(p + 3);
    return v;
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

// erf-GELU x * Phi(x) with Phi(x) - 1/2 = x * Q(x^2) on |x| <= 4.5 (Q: degree-8 least-squares fit on Chebyshev
// nodes, coefficients taken to the variable x^2) and Phi clamped beyond; absolute error of the result below
// 6e-5, under the bf16 rounding of the stored value wherever the value is not itself tiny.  Eleven full-rate
// operations instead of the several dozen of a branching erff.
__device__ __forceinline__ float gelu_erf(float v) {
    const float xc = __builtin_amdgcn_fmed3f(v, -4.5f, 4.5f);
    const float s = xc * xc;
    float q = 2.917371829e-11f;
    q = fmaf(q, s, -3.208389305e-09f);
    q = fmaf(q, s, 1.551676639e-07f);
    q = fmaf(q, s, -4.373868311e-06f);
    q = fmaf(q, s, 8.053694228e-05f);
    q = fmaf(q, s, -1.031751237e-03f);
    q = fmaf(q, s, 9.564368315e-03f);
    q = fmaf(q, s, -6.595010928e-02f);
    q = fmaf(q, s, 3.986949891e-01f);
    return v * fmaf(xc, q, 0.5f);
}

// Record a fault found in device data: OR the flag, keep the smallest index.  first_bad holds
// (2^62 - index) so that a maximum over a zero-initialised word finds the smallest index.
// Faults are exceptional, so the two atomics are off the fast path.
__device__ __forceinline__ void report_fault(ps_status* st, int flag, int64_t index) {
    if (!st) return;
    atomicOr(&st->flags, flag);
    atomicMax((long long*)&st->first_bad, (long long)(((int64_t)1 << 62) - index));
}

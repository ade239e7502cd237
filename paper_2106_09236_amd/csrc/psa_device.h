// Device-side helpers for gfx950 (wave64): DPP lane exchanges, bf16 packing,
// wave-private LDS ordering.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psa_trace.h"

namespace psa {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// ---- DPP: data-parallel-primitive lane permutations inside a row of 16 lanes
// quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
// row_half_mirror = 0x141 (lane i <-> 7-i in each 8), row_mirror = 0x140 (i <-> 15-i).
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
    return __builtin_bit_cast(float,
        __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// Sum over aligned groups of 8 lanes; every lane of the group gets the total.
__device__ __forceinline__ float group_sum8(float x) {
    x += dpp_mov<0xB1>(x);
    x += dpp_mov<0x4E>(x);
    x += dpp_mov<0x141>(x);
    return x;
}
// Sum over aligned groups of 16 lanes.
__device__ __forceinline__ float group_sum16(float x) {
    x = group_sum8(x);
    x += dpp_mov<0x140>(x);
    return x;
}

// ---- bf16 <-> f32
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// two floats to a bf16 pair (lo in bits 0..15) with the hardware conversion, round-to-nearest-even
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---- ordering of LDS traffic between the lanes of ONE wave (no other wave
// touches the region): LDS executes a wave's instructions in order, so only
// the compiler has to be told not to move accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Work-group barrier that orders LDS traffic only.  __syncthreads() also waits
// for every outstanding global load of the wave (one counter covers loads and
// stores), which would serialise loads issued early on purpose; this one leaves
// them in flight.  Use it only where no global store needs to be seen by the
// other waves of the work-group.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Exchange with the lane 32 away (the other half of the wave).
__device__ __forceinline__ float swap_half(float x) { return __shfl_xor(x, 32, 64); }

// 2^x in float64 for x <= ~0 (anything below -1000, -inf included, gives 0):
// x = n + f with |f| <= 1/2, 2^f = e^(f ln 2) by its Taylor series to degree 7
// in Estrin form (truncation 5e-9 relative: the softmax weights need 1e-6, see
// the parity bound; degree 9 measured 1 % slower), scaled by 2^n.
__device__ __forceinline__ double exp2_f64(double x) {
    const double n = rint(x);
    const double z = (x - n) * 0.693147180559945309417;
    const double z2 = z * z, z4 = z2 * z2;
    const double p01 = fma(z, 1.0, 1.0);
    const double p23 = fma(z, 1.66666666666666666667e-1, 0.5);
    const double p45 = fma(z, 8.33333333333333333333e-3, 4.16666666666666666667e-2);
    const double p67 = fma(z, 1.98412698412698412698e-4, 1.38888888888888888889e-3);
    const double q0 = fma(z2, p23, p01);
    const double q1 = fma(z2, p67, p45);
    const double r = fma(z4, q1, q0);
    const double y = ldexp(r, (int)n);
    return x >= -1000.0 ? y : (x != x ? x : 0.0);
}

// Valid length of batch item b, clamped to [0, L].
__device__ __forceinline__ int valid_len(const int* lengths, int b, int L) {
    if (!lengths) return L;
    int n = lengths[b];
    return n < 0 ? 0 : (n > L ? L : n);
}

}  // namespace psa

// Cross-lane reductions of a 64-lane wave without the LDS crossbar.  `__shfl_xor` compiles to ds_bpermute_b32, a
// round trip through the LDS pipeline of well over a hundred cycles; a chain of them (six for a wave-wide sum, four
// per key tile in the attention kernels' soft-max) is pure latency on a wave that has nothing else to issue.  gfx950
// swaps 16-lane rows and 32-lane halves between two registers in one VALU instruction (v_permlane16_swap,
// v_permlane32_swap) and rotates within a row with a DPP modifier, each a few cycles.
//
// Every function pairs the same values in the same order as the xor butterfly it replaces, so results are identical
// bit for bit (checked on the device against the shuffle versions; a + b == b + a exactly).
#pragma once
#include <hip/hip_runtime.h>

namespace ee {

typedef unsigned int lanes_u32x2 __attribute__((ext_vector_type(2)));

// (lower 32 lanes' value, upper 32 lanes' value), each seen by both halves
__device__ __forceinline__ void halves_of(float v, float& lower, float& upper) {
    const lanes_u32x2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    lower = __uint_as_float(a[0]);
    upper = __uint_as_float(a[1]);
}

// (even 16-lane row's value, odd row's value), each seen by both rows of the pair
__device__ __forceinline__ void row_pair_of(float v, float& even, float& odd) {
    const lanes_u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    even = __uint_as_float(a[0]);
    odd = __uint_as_float(a[1]);
}

// lane i of a row receives lane (i - N) mod 16 of the same row
template <int N>
__device__ __forceinline__ float row_rotate(float v) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x120 + N, 0xf, 0xf, false));
}

// sum / max over the four 16-lane rows (lanes i, i+16, i+32, i+48), left in all four: (r0 + r1) + (r2 + r3)
__device__ __forceinline__ float rows4_sum(float v) {
    float a, b;
    row_pair_of(v, a, b);
    v = a + b;
    halves_of(v, a, b);
    return a + b;
}
__device__ __forceinline__ float rows4_max(float v) {
    float a, b;
    row_pair_of(v, a, b);
    v = fmaxf(a, b);
    halves_of(v, a, b);
    return fmaxf(a, b);
}

// sum over all 64 lanes, left in every lane; pairing order of the butterfly xor 32, 16, 8, 4, 2, 1
__device__ __forceinline__ float wave_sum(float v) {
    float a, b;
    halves_of(v, a, b);
    v = a + b;
    row_pair_of(v, a, b);
    v = a + b;
    v += row_rotate<8>(v);
    v += row_rotate<4>(v);
    v += row_rotate<2>(v);
    v += row_rotate<1>(v);
    return v;
}

}  // namespace ee

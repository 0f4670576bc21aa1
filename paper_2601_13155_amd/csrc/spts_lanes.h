// Lane-level helpers shared by the vector (non matrix-core) kernels of libspts: 16-byte chunk dot
// products, element access, wavefront and lane-group reductions.
#pragma once
#include "spts_internal.h"

namespace spts {

typedef __bf16 hbf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of T against 16 bytes of T, accumulated in fp32.  The bf16 pairs are taken out of the
// 8-element vector with constant shuffles (written out: indexing the dwords in a loop and
// bit-casting each made the compiler read element 0 four times).
typedef __bf16 hbf16x8 __attribute__((ext_vector_type(8)));
__device__ inline float dot16(u32x4 w, u32x4 x, float acc, bf16_t) {
    const hbf16x8 a = __builtin_bit_cast(hbf16x8, w), b = __builtin_bit_cast(hbf16x8, x);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), acc, false);
    return acc;
}
__device__ inline float dot16(u32x4 w, u32x4 x, float acc, float) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = fmaf(__uint_as_float(w[i]), __uint_as_float(x[i]), acc);
    return acc;
}
// element e of a 16-byte chunk as fp32
__device__ inline float chunk_elem(u32x4 v, int e, bf16_t) {
    const uint32_t w = v[e >> 1];
    return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
}
__device__ inline float chunk_elem(u32x4 v, int e, float) { return __uint_as_float(v[e]); }

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}


// Sum over aligned groups of LPK lanes (LPK = 2 .. 32), every lane of a group receiving the total.
// Steps 1, 2, 4, 8 stay inside a row of 16 lanes and use DPP operands (quad permutes, then mirror of
// 8 / 16 lanes: after the earlier steps both halves are uniform, so a mirror exchanges them); only a
// step of 16 crosses rows and goes through the LDS crossbar.
template <int LPK>
__device__ inline float group_sum(float v) {
    if (LPK >= 2) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    if (LPK >= 4) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    if (LPK >= 8) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));  // row_half_mirror
    if (LPK >= 16) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false)); // row_mirror
    if (LPK >= 32) v += __shfl_xor(v, 16);
    return v;
}

}  // namespace spts

// Signed base-256 digits of ring words and their byte transposition into digit planes, shared by
// the kernels that pack operands for the int8 matrix-core product.
#pragma once

#include "common.h"

namespace comet_gemm {

constexpr u64 DIGIT_BIAS = 0x0080808080808080ull;

__device__ __forceinline__ u64 to_digits(u64 x) { return (x + DIGIT_BIAS) ^ DIGIT_BIAS; }

// 4x4 byte transpose: in a0..a3 byte b of word j  ->  out word b, byte j
__device__ __forceinline__ void transpose4(u32 a0, u32 a1, u32 a2, u32 a3, u32& o0, u32& o1,
                                           u32& o2, u32& o3) {
    const u32 p01l = __builtin_amdgcn_perm(a1, a0, 0x05010400u);
    const u32 p01h = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
    const u32 p23l = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    const u32 p23h = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    o0 = __builtin_amdgcn_perm(p23l, p01l, 0x05040100u);
    o1 = __builtin_amdgcn_perm(p23l, p01l, 0x07060302u);
    o2 = __builtin_amdgcn_perm(p23h, p01h, 0x05040100u);
    o3 = __builtin_amdgcn_perm(p23h, p01h, 0x07060302u);
}

// Eight consecutive-k words (already in digit form) -> for each digit t one
// 8-byte group holding digit t of k0..k7.
__device__ __forceinline__ void digits_to_planes(const u64 (&v)[8], u64 (&plane)[8]) {
    u32 lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { lo[j] = (u32)v[j]; hi[j] = (u32)(v[j] >> 32); }
    u32 a[8], b[8];   // a: k0..3, b: k4..7, index = digit
    transpose4(lo[0], lo[1], lo[2], lo[3], a[0], a[1], a[2], a[3]);
    transpose4(hi[0], hi[1], hi[2], hi[3], a[4], a[5], a[6], a[7]);
    transpose4(lo[4], lo[5], lo[6], lo[7], b[0], b[1], b[2], b[3]);
    transpose4(hi[4], hi[5], hi[6], hi[7], b[4], b[5], b[6], b[7]);
#pragma unroll
    for (int t = 0; t < 8; ++t) plane[t] = (u64)a[t] | ((u64)b[t] << 32);
}

}  // namespace comet_gemm

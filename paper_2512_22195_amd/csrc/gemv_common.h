// Pieces of the bf16 K/V projection of a handful of token rows (a decode step), shared by the
// stand-alone GEMV kernel and by the fused decode step (paper Section III-B steps 2-3 for one
// new token): one wave per rotary pair (features j and j + D/2 of one head of K or of V),
// products on the packed bf16 dot instruction (exact products, fp32 accumulation), the 64-lane
// sum on DPP adds and register swaps, the rotation on the hardware sine / cosine with the angle
// kept in turns.
#pragma once
#include "device_util.h"

namespace matkv {
namespace gemv {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2v __attribute__((ext_vector_type(2)));

using dev::ldg16;
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ __forceinline__ float dot8(const uint4& a, const uint4& b, float c) {
    c = dot2(a.x, b.x, c); c = dot2(a.y, b.y, c); c = dot2(a.z, b.z, c); c = dot2(a.w, b.w, c);
    return c;
}
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(o);
}
__device__ __forceinline__ float wave_sum(float v, int lane) {
    v = dpp_add<0xB1>(v); v = dpp_add<0x4E>(v); v = dpp_add<0x141>(v); v = dpp_add<0x140>(v);   // 16-lane rows
    const unsigned x = __float_as_uint(v);
    const u32x2v r16 = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    v += __uint_as_float((lane & 16) ? r16.x : r16.y);
    const unsigned y = __float_as_uint(v);
    const u32x2v r32 = __builtin_amdgcn_permlane32_swap(y, y, false, false);
    v += __uint_as_float((lane & 32) ? r32.x : r32.y);
    return v;
}

// Dot products of R token rows (x + r * x_stride, rows past n_rows repeat the last) with the
// two weight rows w0, w1 of one rotary pair; Hd a multiple of 512 * NL (NL = 8: passes of 4096
// columns; NL = 6: of 3072).  All 2 * NL weight loads of a pass are issued before anything is
// consumed.  Sums are complete in every lane.
template <int R, int NL = 8>
__device__ __forceinline__ void pair_dots(const uint16_t* w0, const uint16_t* w1, const uint16_t* x, size_t x_stride,
                                          int n_rows, int Hd, int lane, float (&acc0)[R], float (&acc1)[R]) {
#pragma unroll
    for (int r = 0; r < R; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    w0 += lane * 8; w1 += lane * 8; x += lane * 8;
    for (int c0 = 0; c0 < Hd; c0 += 512 * NL) {
        uint4 wa[NL], wb[NL], xv[R][NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) { wa[i] = ldg16(w0 + c0 + 512 * i); wb[i] = ldg16(w1 + c0 + 512 * i); }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint16_t* xr = x + (size_t)min(r, n_rows - 1) * x_stride + c0;
#pragma unroll
            for (int i = 0; i < NL; ++i) xv[r][i] = ldg16(xr + 512 * i);
        }
#pragma unroll
        for (int i = 0; i < NL; ++i)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                acc0[r] = dot8(wa[i], xv[r][i], acc0[r]);
                acc1[r] = dot8(wb[i], xv[r][i], acc1[r]);
            }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) { acc0[r] = wave_sum(acc0[r], lane); acc1[r] = wave_sum(acc1[r], lane); }
}

// Rotation of the pair (r0, r1) by pos * theta_j: hi/lo split product in turns, whole turns
// dropped exactly, then the hardware sine / cosine (which take turns).
__device__ __forceinline__ void rotate_pair(const RopeEntry& e, float pos, float& r0, float& r1) {
    // no contraction: pos * turns_hi - rint(t) as one multiply-add would take the product exactly
    // and the rounding error of t, added back below, would count twice
#pragma clang fp contract(off)
    const float t = pos * e.turns_hi;
    const float err = fmaf(pos, e.turns_hi, -t);
    float fr = t - rintf(t);
    fr += fmaf(pos, e.turns_lo, err);
    const float c = __builtin_amdgcn_cosf(fr), s = __builtin_amdgcn_sinf(fr);
    const float k0 = r0 * c - r1 * s;
    const float k1 = r0 * s + r1 * c;
    r0 = k0; r1 = k1;
}

}  // namespace gemv
}  // namespace matkv

// Rotary embedding of one token's q and k heads (bf16, rotate-half pairs (j, j + d_head/2)): shared by the
// stand-alone rotary kernel and the launch that also transposes V.
#pragma once
#include "psd_internal.h"
#include "device_types.h"

// 8 pairs (x1, x2) = (a[e], b[e]) of bf16 values rotated by the angles whose cosines / sines are c0|c1 / s0|s1:
// (x1 cos - x2 sin, x2 cos + x1 sin), computed in fp32 and rounded to bf16 once.  Every kernel that applies the
// rotary embedding goes through this one function so that all of them produce the same bits.
__device__ __forceinline__ void rope_rotate8(const uint4 a, const uint4 b, const float4 c0, const float4 c1, const float4 s0,
                                             const float4 s1, uint4 &out_a, uint4 &out_b) {
    const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    const float sn[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
    const uint32_t au[4] = {a.x, a.y, a.z, a.w}, bu[4] = {b.x, b.y, b.z, b.w};
    uint32_t oa[4], ob[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float x1l = bf16_bits_to_float((uint16_t)(au[e] & 0xffff)), x1h = bf16_bits_to_float((uint16_t)(au[e] >> 16));
        const float x2l = bf16_bits_to_float((uint16_t)(bu[e] & 0xffff)), x2h = bf16_bits_to_float((uint16_t)(bu[e] >> 16));
        oa[e] = pack_bf16x2(x1l * cs[2 * e] - x2l * sn[2 * e], x1h * cs[2 * e + 1] - x2h * sn[2 * e + 1]);
        ob[e] = pack_bf16x2(x2l * cs[2 * e] + x1l * sn[2 * e], x2h * cs[2 * e + 1] + x1h * sn[2 * e + 1]);
    }
    out_a = make_uint4(oa[0], oa[1], oa[2], oa[3]);
    out_b = make_uint4(ob[0], ob[1], ob[2], ob[3]);
}

// a thread owns 8 consecutive pair indices j of one head (two 16-byte accesses each way); d_head % 16 == 0
__device__ __forceinline__ void rope_bf16_vec_token(bf16_t *__restrict__ row, int pos, int n_heads, int n_kv_heads, int d_head,
                                                    const float *__restrict__ cos_t, const float *__restrict__ sin_t) {
    const int half = d_head >> 1, groups = half >> 3;
    const int rot_heads = n_heads + n_kv_heads;
    for (int idx = threadIdx.x; idx < rot_heads * groups; idx += blockDim.x) {
        const int hd = idx / groups, j0 = (idx % groups) * 8;
        uint4 *p1 = reinterpret_cast<uint4 *>(row + hd * d_head + j0);
        uint4 *p2 = reinterpret_cast<uint4 *>(row + hd * d_head + j0 + half);
        const uint4 a = *p1, b = *p2;
        const float4 c0 = *reinterpret_cast<const float4 *>(cos_t + (int64_t)pos * half + j0);
        const float4 c1 = *reinterpret_cast<const float4 *>(cos_t + (int64_t)pos * half + j0 + 4);
        const float4 s0 = *reinterpret_cast<const float4 *>(sin_t + (int64_t)pos * half + j0);
        const float4 s1 = *reinterpret_cast<const float4 *>(sin_t + (int64_t)pos * half + j0 + 4);
        uint4 ra, rb;
        rope_rotate8(a, b, c0, c1, s0, s1, ra, rb);
        *p1 = ra;
        *p2 = rb;
    }
}

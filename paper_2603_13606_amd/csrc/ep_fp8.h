// FP8 (OCP E4M3) quantisation of token rows, shared by the kernels that quantise:
// per token and 128-channel group amax = max|x|, scale = amax / 448,
// q = e4m3(float(x) * (448 / amax)) rounded to nearest even and saturated at 448;
// amax == 0 gives scale 1 (the paper gives sizes only -- H bytes + H/128 float scales per
// row, Sec. IV-B payload; format and scale rule are this library's).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace ep {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Four float32 -> four E4M3 codes, packed low to high.  The conversion instruction of this
// part rounds to nearest even exactly as the rule above asks for magnitudes up to 448 and
// turns anything beyond 464 into NaN, so the value is clamped first (a product can exceed 448
// only through an overflowing 448 / amax); a NaN product stays NaN and gets the one NaN code
// this library writes, 0x7F.
__device__ __forceinline__ float clamp_e4m3(float p) {
    const float c = fminf(fmaxf(p, -448.0f), 448.0f);
    return p != p ? p : c;
}

__device__ __forceinline__ uint32_t pack4_e4m3(float f0, float f1, float f2, float f3) {
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(clamp_e4m3(f0), clamp_e4m3(f1), 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(clamp_e4m3(f2), clamp_e4m3(f3), r, true);
    const uint32_t u = (uint32_t)r;
    const uint32_t nan = ((u & 0x7f7f7f7fu) + 0x01010101u) & 0x80808080u;  // bit 7 of every byte that is +-NaN
    return u & ~nan;
}

// 16 consecutive bf16 channels (two 16-byte units) of a lane, as float32.
__device__ __forceinline__ void unpack16(const u32x4& in0, const u32x4& in1, float (&f)[16]) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        f[2 * c] = __uint_as_float(in0[c] << 16);
        f[2 * c + 1] = __uint_as_float(in0[c] & 0xffff0000u);
        f[8 + 2 * c] = __uint_as_float(in1[c] << 16);
        f[8 + 2 * c + 1] = __uint_as_float(in1[c] & 0xffff0000u);
    }
}

// Quantises the 16 channels of this lane; the 8 lanes lane & ~7 .. | 7 hold one group of 128
// channels and must all be active.  Returns the 16 codes, and the scale of the group.
__device__ __forceinline__ u32x4 quantize16(const u32x4& in0, const u32x4& in1, float* scale_out) {
    float f[16];
    unpack16(in0, in1, f);
    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
        const float v = fabsf(f[c]);
        amax = v > amax ? v : amax;
    }
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {  // the 8 lanes of a 128-channel group
        const float o = __shfl_xor(amax, off, kWave);
        amax = o > amax ? o : amax;
    }
    float scale = 1.0f, inv = 1.0f;
    if (amax != 0.0f) {
        scale = __fdiv_rn(amax, 448.0f);
        inv = __fdiv_rn(448.0f, amax);
    }
    u32x4 q;
#pragma unroll
    for (int c = 0; c < 4; ++c)
        q[c] = pack4_e4m3(__fmul_rn(f[4 * c], inv), __fmul_rn(f[4 * c + 1], inv), __fmul_rn(f[4 * c + 2], inv),
                          __fmul_rn(f[4 * c + 3], inv));
    *scale_out = scale;
    return q;
}

}  // namespace ep

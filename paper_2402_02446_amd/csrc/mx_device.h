// Device helpers for gfx950: MXINT block arithmetic on 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lqer {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// an 8-byte load from a 4-byte aligned address (exponent words of the compact weight records)
typedef u32x2 u32x2_a4 __attribute__((aligned(4)));

union Frag {            // one bf16 MFMA operand (16x16x32 or 32x32x16): 8 bf16 per lane
    bf16x8 v;
    u32x4 u;
    bf16x2 h[4];
};

__device__ __forceinline__ float f32_from_bits(uint32_t b) { return __builtin_bit_cast(float, b); }
__device__ __forceinline__ uint32_t f32_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// fp32 scale 2^(eb - 127 - 2 + 9) for a W block with exponent byte eb: the +9 undoes the 2^-9 of
// the fp8 subnormal encoding, the -2 is the MXINT4 fraction.  eb <= 247 is checked at import.
__device__ __forceinline__ float w_scale(uint32_t eb) { return f32_from_bits((eb + 7u) << 23); }

// 8 sign-magnitude 4-bit codes (layout in lqer_internal.h) -> 8 bf16 values code * 2^(e-2).
__device__ __forceinline__ bf16x8 unpack_w8(uint32_t w, float scale) {
    const uint32_t r0 = w & 0x87878787u;
    const uint32_t r1 = __builtin_amdgcn_alignbit(w, w, 4) & 0x87878787u;
    Frag f;
    f.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r0, scale, false);
    f.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r0, scale, true);
    f.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r1, scale, false);
    f.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r1, scale, true);
    return f.v;
}

// 2-bit weights: fp32 scale 2^(eb - 127 + 9) for a block with exponent byte eb (no fraction bits; the +9 undoes the
// 2^-9 of the fp8 subnormal encoding).  eb <= 245 is checked at import.
__device__ __forceinline__ float w2_scale(uint32_t eb) { return f32_from_bits((eb + 9u) << 23); }

// Eight of the 16 sign-and-magnitude 2-bit codes of a block word (layout in lqer_internal.h) -> 8 bf16 values
// code * 2^e: elements 8 half .. 8 half + 7.
__device__ __forceinline__ bf16x8 unpack_w8_b2(uint32_t w, int half, float scale) {
    const uint32_t r0 = (half ? __builtin_amdgcn_alignbit(w, w, 4) : w) & 0x81818181u;
    const uint32_t r1 = __builtin_amdgcn_alignbit(w, w, half ? 6 : 2) & 0x81818181u;
    Frag f;
    f.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r0, scale, false);
    f.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r0, scale, true);
    f.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r1, scale, false);
    f.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r1, scale, true);
    return f.v;
}

// Two fp32 values that are exactly representable in bf16 -> packed pair (a low, b high).
__device__ __forceinline__ uint32_t pack_bf16_exact(float a, float b) {
    return __builtin_amdgcn_perm(f32_bits(b), f32_bits(a), 0x07060302u);
}

// 4 int8 codes in a word, times an exact power-of-two scale -> 4 bf16 (exact), as two packed pairs.
__device__ __forceinline__ u32x2 int8x4_to_bf16(uint32_t w, float scale) {
    const float f0 = (float)(int)(int8_t)(w & 0xFF) * scale;
    const float f1 = (float)(int)(int8_t)((w >> 8) & 0xFF) * scale;
    const float f2 = (float)(int)(int8_t)((w >> 16) & 0xFF) * scale;
    const float f3 = (float)(int)(int8_t)(w >> 24) * scale;
    return u32x2{pack_bf16_exact(f0, f1), pack_bf16_exact(f2, f3)};
}

// One MXINT8 block (16 int8 codes) -> the two MFMA operands of its two K steps.
__device__ __forceinline__ void int8x16_to_frags(u32x4 cw, float scale, Frag& f0, Frag& f1) {
    const u32x2 a = int8x4_to_bf16(cw[0], scale), b = int8x4_to_bf16(cw[1], scale);
    const u32x2 c = int8x4_to_bf16(cw[2], scale), d = int8x4_to_bf16(cw[3], scale);
    f0.u = u32x4{a[0], a[1], b[0], b[1]};
    f1.u = u32x4{c[0], c[1], d[0], d[1]};
}

// fp32 scale 2^(eb - 127 - 6) of an MXINT8 block.  Below the normal range (eb < 7) the value is
// produced by a second exact multiply.
__device__ __forceinline__ float h_scale(uint32_t eb) {
    return (eb >= 7u) ? f32_from_bits((eb - 6u) << 23)
                      : f32_from_bits((eb + 18u) << 23) * 0x1p-24f;
}

// fp32 scale 2^(eb - 127 - frac) of an MXINT block with `frac` fraction bits (6 for 8-bit codes, 4 for 6-bit).
__device__ __forceinline__ float x_scale(uint32_t eb, int frac) {
    return (eb > (uint32_t)frac) ? f32_from_bits((eb - frac) << 23)
                                 : f32_from_bits((eb + 24u - frac) << 23) * 0x1p-24f;
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// D[i][j] += sum_k A[i][k] B[k][j], 32 x 32 x 16.  Lane (l % 32, l / 32) supplies A[l % 32][8 (l/32) ..+7]
// and B[8 (l/32) ..+7][l % 32]; accumulator register r of lane l is D[8 (r/4) + 4 (l/32) + r % 4][l % 32].
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Eight values of one MXINT8 block held by this lane (the other eight sit in lane ^ 32): the block's
// exponent byte from the maximum over both lanes, and this lane's codes as two words of four bytes.
__device__ __forceinline__ uint32_t requant_half_block(const float (&v)[8], uint32_t& w0, uint32_t& w1) {
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = __builtin_fmaxf(m, __builtin_fabsf(v[i]));
    m = __builtin_fmaxf(m, __shfl_xor(m, 32));
    const uint32_t eb = (f32_bits(m) >> 23) & 0xFFu;
    const int e = (int)eb - 127;
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float r = __builtin_rintf(__builtin_amdgcn_ldexpf(v[i], 6 - e));
        r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
        w[i >> 2] |= ((uint32_t)(int)r & 0xFFu) << (8 * (i & 3));
    }
    w0 = w[0];
    w1 = w[1];
    return eb;
}

// MXINT8 quantization of one value given the block's exponent byte: code = sat(rne(v * 2^(6-e))).
__device__ __forceinline__ int mx8_code(float v, int e_unbiased) {
    float r = __builtin_rintf(__builtin_amdgcn_ldexpf(v, 6 - e_unbiased));
    r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

}  // namespace lqer

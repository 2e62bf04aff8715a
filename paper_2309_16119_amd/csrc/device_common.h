// Device-side building blocks shared by every kernel of the library:
// bit-stream unpacking and the exact dequantization of one code.
//
// Dequantization follows Section 2.2 eq. (2) of the ModuLoRA paper in its
// integer-zero-point form,  w = (q - zero) * scale, materialized in bfloat16
// (Section 3.2 materializes in a 16-bit float).  The product is formed exactly
// in binary32 and rounded once, to nearest even, to bfloat16.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mlr {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// Make a value provably wave-uniform (it then lives in a scalar register).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Load from a wave-uniform base plus a per-lane 32-bit byte offset: the form that maps
// onto "scalar base + vector offset" addressing and needs no per-lane 64-bit arithmetic.
template <typename T>
__device__ __forceinline__ T load_at(const void *base, uint32_t byte_off) {
    return *reinterpret_cast<const T *>(static_cast<const char *>(base) + byte_off);
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
    _Float16 x;
    __builtin_memcpy(&x, &h, sizeof x);
    return (float)x;   // exact
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) {
    return __uint_as_float(((uint32_t)h) << 16);
}

// Two floats -> two bfloat16 (round to nearest even) packed in one register,
// `lo` in bits 0..15.  Compiles to v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    bf16x2 p = {(__bf16)lo, (__bf16)hi};
    uint32_t u;
    __builtin_memcpy(&u, &p, sizeof u);
    return u;
}

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    return (uint16_t)(pack_bf16x2(f, 0.0f) & 0xFFFFu);
}

// Per-(group, column) dequantization constants: w = fma(q, scale, bias) with
// bias = -zero * scale.  zero <= 255 and scale has an 11-bit significand, so
// bias is exact; q * scale is exact inside the fma and the sum (q - zero) * scale
// is representable, so the fma returns the exact product.
struct DqConst {
    float scale;
    float bias;
};

__device__ __forceinline__ DqConst make_dq(uint16_t scale_bits, uint8_t zero) {
    DqConst c;
    c.scale = half_bits_to_float(scale_bits);
    c.bias = -(float)zero * c.scale;
    return c;
}

__device__ __forceinline__ float dq_value(uint32_t q, const DqConst &c) {
    return __builtin_fmaf((float)q, c.scale, c.bias);
}

// Code i (0..7) of an 8-code chunk: chunk bits [i*BITS, i*BITS + BITS).
template <int BITS>
__device__ __forceinline__ uint32_t chunk_code(uint32_t chunk, int i) {
    return (chunk >> (i * BITS)) & ((1u << BITS) - 1u);
}

// The 8-code chunk number j (0..3) of a 32-code block held in BITS words
// (w[0] first): stream bits [8*BITS*j, 8*BITS*(j+1)) of the block, in the low
// 8*BITS bits of the result (higher bits are junk for BITS == 3 and are masked
// by chunk_code).
template <int BITS>
__device__ __forceinline__ uint32_t block_chunk(const uint32_t *w, int j) {
    if (BITS == 4) return w[j];
    if (BITS == 2) return (j & 1) ? (w[j >> 1] >> 16) : w[j >> 1];
    // BITS == 3: 24-bit chunks at stream bits 0, 24, 48, 72
    switch (j) {
        case 0: return w[0];
        case 1: return (w[0] >> 24) | (w[1] << 8);
        case 2: return (w[1] >> 16) | (w[2] << 16);
        default: return w[2] >> 8;
    }
}

// Dequantize the 8 codes of one chunk with one (scale, bias): 8 bfloat16 in
// 4 registers, code 0 in the low half of out[0].
template <int BITS>
__device__ __forceinline__ void dequant_chunk(uint32_t chunk, const DqConst &c, uint32_t out[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float lo = dq_value(chunk_code<BITS>(chunk, 2 * i), c);
        float hi = dq_value(chunk_code<BITS>(chunk, 2 * i + 1), c);
        out[i] = pack_bf16x2(lo, hi);
    }
}

// Dequantize a whole 32-code block (BITS words, one scale and zero): 32 bfloat16 in 16
// registers, code 0 in the low half of out[0].  For 4- and 2-bit codes the fields are
// first spread to one code per byte with a few AND/shift operations, so that each code
// then costs one byte->float conversion (v_cvt_f32_ubyteN) instead of extract + convert.
template <int BITS>
__device__ __forceinline__ void dequant_block(const uint32_t *w, const DqConst &c, uint32_t out[16]) {
    if (BITS == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo = w[j] & 0x0F0F0F0Fu, hi = (w[j] >> 4) & 0x0F0F0F0Fu;
#pragma unroll
            for (int i = 0; i < 4; ++i)   // codes 2i (lo byte i) and 2i+1 (hi byte i)
                out[j * 4 + i] = pack_bf16x2(dq_value((lo >> (8 * i)) & 0xFFu, c), dq_value((hi >> (8 * i)) & 0xFFu, c));
        }
    } else if (BITS == 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {     // word h holds codes 16h .. 16h+15
            uint32_t m[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) m[t] = (w[h] >> (2 * t)) & 0x03030303u;   // byte b of m[t] = code 4b + t
#pragma unroll
            for (int i = 0; i < 8; ++i) { // codes 2i, 2i+1 of the word
                const int c0 = 2 * i, c1 = 2 * i + 1;
                out[h * 8 + i] = pack_bf16x2(dq_value((m[c0 & 3] >> (8 * (c0 >> 2))) & 0xFFu, c),
                                             dq_value((m[c1 & 3] >> (8 * (c1 >> 2))) & 0xFFu, c));
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) dequant_chunk<BITS>(block_chunk<BITS>(w, j), c, out + 4 * j);
    }
}

// Exact three-way split of eight fp32 values into bfloat16 pairs: hi + mid + lo carry all 24
// significand bits, so three bf16 MFMAs against them reproduce the fp32 products.
__device__ __forceinline__ void split3(const float x[8], uint32_t hi[4], uint32_t mid[4], uint32_t lo[4]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float x0 = x[2 * p], x1 = x[2 * p + 1];
        hi[p] = pack_bf16x2(x0, x1);
        const float r0 = x0 - __uint_as_float(hi[p] << 16), r1 = x1 - __uint_as_float(hi[p] & 0xFFFF0000u);
        mid[p] = pack_bf16x2(r0, r1);
        const float s0 = r0 - __uint_as_float(mid[p] << 16), s1 = r1 - __uint_as_float(mid[p] & 0xFFFF0000u);
        lo[p] = pack_bf16x2(s0, s1);
    }
}

// Exact two-way split of eight binary16 values (four registers of pairs) into bfloat16 pairs: the
// upper 8 significand bits and the remaining (at most 3), so two bf16 MFMAs against them reproduce
// the products with the binary16 values.  Truncation, not rounding: both parts are exact.
__device__ __forceinline__ void split_f16x8(const uint32_t h[4], uint32_t hi[4], uint32_t lo[4]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float x0 = half_bits_to_float((uint16_t)(h[p] & 0xFFFFu)), x1 = half_bits_to_float((uint16_t)(h[p] >> 16));
        const uint32_t t0 = __float_as_uint(x0) & 0xFFFF0000u, t1 = __float_as_uint(x1) & 0xFFFF0000u;
        hi[p] = (t0 >> 16) | t1;
        const float r0 = x0 - __uint_as_float(t0), r1 = x1 - __uint_as_float(t1);
        lo[p] = (__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xFFFF0000u);
    }
}

}  // namespace mlr

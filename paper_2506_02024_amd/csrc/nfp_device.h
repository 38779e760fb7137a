// Device-side helpers shared by the NestedFP HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nfp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int intx8 __attribute__((ext_vector_type(8)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// ---- FP16 reconstruction, four weights per 32-bit word (Sec. 4.2, Alg. 1) ----------
// u, l: four upper / lower bytes of consecutive weights (byte j <-> weight j).
// Returns the upper bytes with the rounding undone: S | 0 | E[3:0] | M1 M2 per byte.
// The subtraction never borrows across bytes for planes made by the decomposition:
// the checksum bit is set only when the stored 7-bit field is at least 1.
__device__ __forceinline__ uint32_t undo_rounding4(uint32_t u, uint32_t l) {
    uint32_t sub = (l >> 7) & 0x01010101u;
    uint32_t t = ((u - sub) >> 1) & 0x3f3f3f3fu;
    return t | (u & 0x80808080u);
}

// v_perm_b32: result byte i = byte sel[i] of the 8-byte value {hi:lo} (lo = bytes 0..3).
__device__ __forceinline__ uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// Interleave: weights 0,1 -> w01 = {l0,h0,l1,h1}, weights 2,3 -> w23 (little-endian FP16 pairs).
__device__ __forceinline__ void merge4(uint32_t u, uint32_t l, uint32_t &w01, uint32_t &w23) {
    uint32_t h = undo_rounding4(u, l);
    w01 = byte_perm(h, l, 0x05010400u);
    w23 = byte_perm(h, l, 0x07030602u);
}

// 16 weights: four dwords of upper bytes + four of lower bytes -> two 16-byte vectors of FP16 words.
__device__ __forceinline__ void merge16(const u32x4 &u, const u32x4 &l, u32x4 &w_lo, u32x4 &w_hi) {
    uint32_t a, b;
    merge4(u.x, l.x, a, b);  w_lo.x = a;  w_lo.y = b;
    merge4(u.y, l.y, a, b);  w_lo.z = a;  w_lo.w = b;
    merge4(u.z, l.z, a, b);  w_hi.x = a;  w_hi.y = b;
    merge4(u.w, l.w, a, b);  w_hi.z = a;  w_hi.w = b;
}

// ---- Decomposition of two FP16 words packed in 32 bits (Sec. 4.1) -------------------
// Each 16-bit half: magnitude field m = bits & 0x7fff; E[3:0]|M[1:3] rounded to nearest
// even = (m + 0x3f + bit7(m)) >> 7; in-range magnitudes (<= 0x3f00) cannot carry into
// the neighbouring half.  Out-of-range halves yield (0,0) and are counted.
__device__ __forceinline__ void decompose2(uint32_t w, uint32_t &up2, uint32_t &lo2, uint32_t &bad) {
    uint32_t m = w & 0x7fff7fffu;
    uint32_t m_lo = m & 0xffffu, m_hi = m >> 16;
    uint32_t ok_lo = (m_lo <= 0x3f00u) ? 0x0000ffffu : 0u;
    uint32_t ok_hi = (m_hi <= 0x3f00u) ? 0xffff0000u : 0u;
    uint32_t ok = ok_lo | ok_hi;
    bad += (ok_lo == 0u) + (ok_hi == 0u);
    w &= ok;
    m &= ok;
    uint32_t r = (m + 0x003f003fu + ((m >> 7) & 0x00010001u)) >> 7;  // per half, <= 0x7e
    up2 = (r & 0x00ff00ffu) | ((w >> 8) & 0x00800080u);             // byte in each half
    lo2 = w & 0x00ff00ffu;
}

// pack bytes {a.b0, a.b2, b.b0, b.b2}
__device__ __forceinline__ uint32_t pack_even_bytes(uint32_t a, uint32_t b) {
    return byte_perm(b, a, 0x06040200u);
}

// 16 FP16 words (two 16-byte vectors) -> 16 upper bytes and 16 lower bytes, in order.
__device__ __forceinline__ void decompose16(const u32x4 &a, const u32x4 &b, u32x4 &up, u32x4 &lo, uint32_t &bad) {
    uint32_t u[8], l[8];
    decompose2(a.x, u[0], l[0], bad);
    decompose2(a.y, u[1], l[1], bad);
    decompose2(a.z, u[2], l[2], bad);
    decompose2(a.w, u[3], l[3], bad);
    decompose2(b.x, u[4], l[4], bad);
    decompose2(b.y, u[5], l[5], bad);
    decompose2(b.z, u[6], l[6], bad);
    decompose2(b.w, u[7], l[7], bad);
    up.x = pack_even_bytes(u[0], u[1]);  lo.x = pack_even_bytes(l[0], l[1]);
    up.y = pack_even_bytes(u[2], u[3]);  lo.y = pack_even_bytes(l[2], l[3]);
    up.z = pack_even_bytes(u[4], u[5]);  lo.z = pack_even_bytes(l[4], l[5]);
    up.w = pack_even_bytes(u[6], u[7]);  lo.w = pack_even_bytes(l[6], l[7]);
}

// ---- E4M3 encode (OCP "FN": bias 7, max 448, no Inf) from binary32 -----------------
// Round-to-nearest-even in integer arithmetic; |r| must already be clamped to <= 448.
__device__ __forceinline__ uint32_t e4m3_from_float_sw(float r) {
    uint32_t b = __float_as_uint(r);
    uint32_t sign = (b >> 24) & 0x80u;
    uint32_t a = b & 0x7fffffffu;
    uint32_t code;
    if (a >= 0x3c800000u) {                    // |r| >= 2^-6: normal E4M3
        uint32_t q = (a + 0x7ffffu + ((a >> 20) & 1u)) >> 20;   // exp|m3, RNE
        code = q - (120u << 3);                // rebias 127 -> 7
    } else {                                   // subnormal: multiples of 2^-9
        code = (uint32_t)__float2int_rn(__uint_as_float(a) * 512.0f);
    }
    return sign | code;
}

// Four floats -> four E4M3 bytes with the hardware converter (v_cvt_pk_fp8_f32).
__device__ __forceinline__ uint32_t e4m3x4_from_float_hw(float a, float b, float c, float d) {
    int v = 0;
    v = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, v, false);
    v = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, v, true);
    return (uint32_t)v;
}

__device__ __forceinline__ float clamp448(float r) {
    return fminf(fmaxf(r, -448.0f), 448.0f);
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
    union { uint16_t u; _Float16 f; } cvt;
    cvt.u = (uint16_t)h16;
    return (float)cvt.f;
}

// Correctly rounded binary32 quotient a / s from y = RN(1 / s) (itself one IEEE division per
// token row): q0 = RN(a*y), r = a - q0*s exactly (FMA), q = RN(q0 + r*y).  With a correctly
// rounded reciprocal this is the correctly rounded quotient whenever nothing over- or
// underflows (Markstein's theorem); here |a| is a finite FP16 value and s lies far inside the
// binary32 range, and the identity is also checked exhaustively against the oracle's division.
__device__ __forceinline__ float div_by_scale(float a, float s, float y) {
    float q0 = a * y;
    float r = __builtin_fmaf(-q0, s, a);
    return __builtin_copysignf(__builtin_fmaf(r, y, q0), a);       // s > 0; keeps -0 / s = -0
}

// Four FP16 activations (two packed dwords) -> four E4M3 bytes at scale s (Sec. 2.2, per-token
// scaling): quotient correctly rounded in binary32, clamp to +-448, RNE.  y = 1.0f / s.
template <bool HW>
__device__ __forceinline__ uint32_t quant4(uint32_t w01, uint32_t w23, float s, float y) {
    float a = clamp448(div_by_scale(half_bits_to_float(w01 & 0xffffu), s, y));
    float b = clamp448(div_by_scale(half_bits_to_float(w01 >> 16), s, y));
    float c = clamp448(div_by_scale(half_bits_to_float(w23 & 0xffffu), s, y));
    float d = clamp448(div_by_scale(half_bits_to_float(w23 >> 16), s, y));
    if (HW) return e4m3x4_from_float_hw(a, b, c, d);
    return e4m3_from_float_sw(a) | (e4m3_from_float_sw(b) << 8) | (e4m3_from_float_sw(c) << 16) |
           (e4m3_from_float_sw(d) << 24);
}

// FP8-mode outputs are the FP32 sum times the FP32 scale, rounded to FP32, then converted to FP16,
// in every kernel: the empty asm keeps the compiler from fusing product and conversion into a single
// rounding in some kernels and not in others, so that every launch shape gives the same bits.
__device__ __forceinline__ float scale_f32(float x, float s) {
    float y = x * s;
    asm("" : "+v"(y));
    return y;
}

__device__ __forceinline__ uint32_t float2_to_half2_bits(float a, float b) {
    union { _Float16 f[2]; uint32_t u; } cvt;
    cvt.f[0] = (_Float16)a;
    cvt.f[1] = (_Float16)b;
    return cvt.u;
}

}  // namespace nfp

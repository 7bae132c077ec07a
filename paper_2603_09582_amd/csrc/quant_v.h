// Device helpers shared by the operand-preparation kernels and the single-launch
// short-sequence kernel: the key order inside a block image, the per-channel absmax of V
// and the 8-bit quantiser psi of Eq. 7.
#pragma once

#include "binattn_internal.h"

namespace binattn {

typedef unsigned u4 __attribute__((ext_vector_type(4)));

// Eq. 5 for 8 bf16 values: bit i = (x_i >= 0) under IEEE rules (-0.0 -> 1, NaN -> 0, Sec. 3);
// adds their magnitudes to asum.
__device__ __forceinline__ unsigned sign_bits8_abs(u4 w, float &asum) {
    unsigned bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(w[i] << 16);
        const float hi = __uint_as_float(w[i] & 0xffff0000u);
        bits |= (lo >= 0.0f ? 1u : 0u) << (2 * i);
        bits |= (hi >= 0.0f ? 1u : 0u) << (2 * i + 1);
        asum += fabsf(lo) + fabsf(hi);
    }
    return bits;
}

// Row position inside a key block <-> key offset.  The fused kernel's lane
// (g = lane / 32) holds, for MFMA tile t and accumulator register r, the key
// j0 + 64 g + 16 t + r; the MFMA puts accumulator register r of lane group g
// at tile row m = 8 (r / 4) + 4 g + (r % 4).  Rows are stored at position
// 32 t + m so that the A operand reads consecutive LDS rows.
__device__ __forceinline__ int key_of_position(int pos) {
    const int t = pos >> 5, m = pos & 31;
    const int g = (m >> 2) & 1;
    const int r = ((m >> 3) << 2) | (m & 3);
    return 64 * g + 16 * t + r;
}

__device__ __forceinline__ void unpack8(u4 w, float f[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// Running absmax of 8 bf16 values per lane on their bit patterns: with the sign bit
// cleared, bf16 magnitudes order like 16-bit unsigned integers (two values per instruction).
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void absmax_acc(unsigned m[4], u4 w) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const us2 a = __builtin_bit_cast(us2, m[i]);
        const us2 b = __builtin_bit_cast(us2, w[i] & 0x7FFF7FFFu);
        m[i] = __builtin_bit_cast(unsigned, __builtin_elementwise_max(a, b));
    }
}
__device__ __forceinline__ void absmax_floats(const unsigned m[4], float f[8]) {
    unpack8(u4{m[0], m[1], m[2], m[3]}, f);
}

// Eq. 7 scale: absmax / 127 (IEEE fp32 division); 1 for an all-zero channel.
__device__ __forceinline__ float delta_of_absmax(float a) {
    return (a == 0.0f) ? 1.0f : __fdiv_rn(a, 127.0f);
}

// Eq. 7: code = round-to-nearest-even(y), clamped to [-127, 127], with y the IEEE fp32
// quotient v / delta.  Fast form: with r = fp32(1 / delta), the bracketing multipliers
// r_lo = fp32(r (1 - 2^-22)) and r_hi = fp32(r (1 + 2^-22)) satisfy
// r_lo <= (1 / delta)(1 - 2^-23) and r_hi >= (1 / delta)(1 + 2^-23), so y (relative error
// 2^-24) lies between v r_lo and v r_hi.  fma(v, r, 1.5 * 2^23) rounds the exact product v r
// to an integer (ties to even) and leaves its two's complement code in the low byte;
// rounding is monotone, so when the two brackets round alike that integer is the code of y.
// |v| <= absmax makes |y| <= 127 (1 + 2^-23), which rounds to at most 127: no clamp needed
// there.  When they differ (v / delta within 6e-5 of a half-integer, or a non-finite
// input) the code comes from the division itself.  A channel whose 1 / delta is not finite
// gets r_lo = 0, r_hi = inf, which never agree.
constexpr float QMAGIC = 12582912.0f;  // 1.5 * 2^23
__device__ __forceinline__ float quant_exact(float v, float delta) {
    return fminf(fmaxf(rintf(__fdiv_rn(v, delta)), -127.0f), 127.0f) + QMAGIC;
}
// The constants of 8 consecutive channels, read from LDS with 16-byte loads up front (the
// arrays must be 16-byte aligned).
struct QuantConsts8 {
    float dl[8], lo[8], hi[8];
};
__device__ __forceinline__ QuantConsts8 load_quant_consts8(const float *sdelta, const float *srlo,
                                                          const float *srhi, int c) {
    QuantConsts8 k;
    const float4 *a = reinterpret_cast<const float4 *>(sdelta + 8 * c);
    const float4 *b = reinterpret_cast<const float4 *>(srlo + 8 * c);
    const float4 *e = reinterpret_cast<const float4 *>(srhi + 8 * c);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float4 x = a[h], y = b[h], z = e[h];
        k.dl[4 * h] = x.x; k.dl[4 * h + 1] = x.y; k.dl[4 * h + 2] = x.z; k.dl[4 * h + 3] = x.w;
        k.lo[4 * h] = y.x; k.lo[4 * h + 1] = y.y; k.lo[4 * h + 2] = y.z; k.lo[4 * h + 3] = y.w;
        k.hi[4 * h] = z.x; k.hi[4 * h + 1] = z.y; k.hi[4 * h + 2] = z.z; k.hi[4 * h + 3] = z.w;
    }
    return k;
}
// codes of 4 tokens x 8 channels (w[k]: token k), one dword per channel, token k in byte k;
// one test per channel (4 values) decides between the bracketed and the exact form.  Both
// bracket results are integers within 128 of 1.5 * 2^23 (finite V), so they are equal iff
// their bits are, and their bit differences are small numbers.
__device__ __forceinline__ void quant_quad(const u4 w[4], const QuantConsts8 &kc, unsigned packed[8]) {
    float f[4][8];
#pragma unroll
    for (int k = 0; k < 4; ++k) unpack8(w[k], f[k]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float s[4];
        unsigned diff = 0u;  // sum of the bit differences (each below 2^9): one xor-add per value
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            s[k] = fmaf(f[k][i], kc.lo[i], QMAGIC);
            diff += __float_as_uint(s[k]) ^ __float_as_uint(fmaf(f[k][i], kc.hi[i], QMAGIC));
        }
        if (diff != 0u) {
#pragma unroll
            for (int k = 0; k < 4; ++k) s[k] = quant_exact(f[k][i], kc.dl[i]);
        }
        const unsigned b01 = __builtin_amdgcn_perm(__float_as_uint(s[1]), __float_as_uint(s[0]), 0x0c0c0400u);
        const unsigned b23 = __builtin_amdgcn_perm(__float_as_uint(s[3]), __float_as_uint(s[2]), 0x0c0c0400u);
        packed[i] = b01 | (b23 << 16);
    }
}
// per-channel constants of the quantiser from the channel's absmax
__device__ __forceinline__ void quant_consts(float a, float *dl, float *r_lo, float *r_hi) {
    *dl = delta_of_absmax(a);
    const float r = __fdiv_rn(1.0f, *dl);
    const bool ok = r < 3.0e38f;
    *r_lo = ok ? __fmul_rn(r, 1.0f - 0x1p-22f) : 0.0f;
    *r_hi = ok ? __fmul_rn(r, 1.0f + 0x1p-22f) : INFINITY;
}

}  // namespace binattn

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

// Eq. 7: code = round-to-nearest-even(v / delta), clamped to [-127, 127], where the
// quotient is the IEEE fp32 one.  t = v * (1 / delta) is within 2.3e-5 of that quotient
// (|v / delta| <= 127), so its rounding is already decided unless t sits that close to a
// half-integer; only then is the exact division needed.  Clamping t first is equivalent
// (the bounds are integers).  Rounding is the fp32 addition of 1.5 * 2^23, whose result
// carries the two's complement code in its low byte.  thr = 0.4999 normally; a channel whose
// 1 / delta is not finite passes thr < 0 and rcp = 0, which sends every element to the division.
constexpr float QMAGIC = 12582912.0f;  // 1.5 * 2^23
__device__ __forceinline__ unsigned quant_bits(float v, float delta, float rcp_delta, float thr) {
    const float t = __builtin_amdgcn_fmed3f(v * rcp_delta, -127.0f, 127.0f);
    float s = t + QMAGIC;
    const float q = s - QMAGIC;
    if (fabsf(t - q) > thr) {
        const float e = fminf(fmaxf(rintf(__fdiv_rn(v, delta)), -127.0f), 127.0f);
        s = e + QMAGIC;
    }
    return __float_as_uint(s);
}
// codes of 4 tokens x 8 channels (w[k]: token k), one dword per channel, token k in byte k
__device__ __forceinline__ void quant_quad(const u4 w[4], const float *sdelta, const float *srcp,
                                           const float *sthr, int c, unsigned packed[8]) {
    float f[4][8];
#pragma unroll
    for (int k = 0; k < 4; ++k) unpack8(w[k], f[k]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float dl = sdelta[8 * c + i], rc = srcp[8 * c + i], th = sthr[8 * c + i];
        unsigned b[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) b[k] = quant_bits(f[k][i], dl, rc, th);
        const unsigned lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
        const unsigned hi = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
        packed[i] = lo | (hi << 16);
    }
}
// per-channel constants of the quantiser from the channel's absmax
__device__ __forceinline__ void quant_consts(float a, float *dl, float *rc, float *th) {
    *dl = delta_of_absmax(a);
    const float r = __fdiv_rn(1.0f, *dl);
    const bool ok = r < 3.0e38f;
    *rc = ok ? r : 0.0f;
    *th = ok ? 0.4999f : -1.0f;
}

}  // namespace binattn

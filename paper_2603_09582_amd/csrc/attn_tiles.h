// Device routines shared by the fused attention kernel and the logits export:
// the per-block operand image, its asynchronous copy into LDS, and the QK tile
// on the matrix cores.
//
// Register/lane convention (wave64, 32x32 MFMA tiles, D = A*B + C):
//   lane L feeds row (A) / column (B) number (L & 31) with the k-slots of group
//   g = L >> 5.  A and B use the same slot numbering, so any consistent
//   assignment of channels (or keys) to slots gives the same contraction.
//   D: lane L holds column (L & 31); register r holds row 8(r/4) + 4g + (r%4).
// The kernels put KEYS (resp. value channels) on the A side and QUERIES on the
// B side, so that every lane owns one query row: all softmax statistics are
// lane-local, and the P tile a lane produces is already in B-operand order for
// the P.V contraction (no LDS round trip).
//
// QK runs as v_mfma_f32_32x32x64_f8f6f4 with FP4 (e2m1) operands: +1.0 and -1.0
// are exact in FP4, the products and the fp32 accumulation of at most 128 of
// them are exact, so the result is the integer logit of Sec. 4.1 already in
// fp32 (no int->float conversion), and the accumulator input carries the bias
// term of Eq. 6 for free.  An int8 form of the same tile is kept for comparison.
#pragma once

#include "binattn_internal.h"

namespace binattn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));  // 16-byte register

constexpr int FUSED_THREADS = 256;
constexpr int KT = BV / 32;  // MFMA key tiles per block

// B operand of the QK tile for this lane's query row: FP4 codes of channels
// 64 s + 32 g + [0, 32) in 16 bytes, zero beyond d.  q_words: the row's sign words
// (zero-filled up to 2 * DK2).  `flip` negates the row, `zero` clears it (used for a
// non-positive or vanishing logit multiplier).
template <int DK2>
__device__ __forceinline__ void load_q_operand(const unsigned q_words[2 * DK2], int d, int g,
                                               bool flip, bool zero, v4i qB[DK2]) {
#pragma unroll
    for (int s = 0; s < DK2; ++s) {
        unsigned word = g ? q_words[2 * s + 1] : q_words[2 * s];
        if (flip) word = ~word;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c0 = 32 * (2 * s + g) + 8 * i;
            qB[s][i] = (c0 < d && !zero) ? (int)fp4_pm1_from_bits8((word >> (8 * i)) & 0xFFu) : 0;
        }
    }
}

// A operand rows of QK tile t for this lane (LDS reads only).
template <int DK>
__device__ __forceinline__ void load_k_operand(const char *img, int t, int m, int g,
                                               v4i ka[(DK + 1) / 2]) {
    using L = Image<DK>;
#pragma unroll
    for (int s = 0; s < L::DK2; ++s)
        ka[s] = *reinterpret_cast<const v4i *>(img + L::K_OFF + (32 * t + m) * L::KP +
                                               16 * k_chunk(m, 2 * s + g, L::KP));
}

// QK tile: for this lane's query, register r of the result is
// cin[r] + (s_i . t_j) with key j = block start + 64 g + 16 t + r.
template <int DK2>
__device__ __forceinline__ v16f qk_mfma(const v4i ka[DK2], const v4i qB[DK2], v16f cin) {
#pragma unroll
    for (int s = 0; s < DK2; ++s) {
        const v8i a8 = {ka[s][0], ka[s][1], ka[s][2], ka[s][3], 0, 0, 0, 0};
        const v8i b8 = {qB[s][0], qB[s][1], qB[s][2], qB[s][3], 0, 0, 0, 0};
        cin = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, cin, 4, 4, 0, 0, 0, 0);
    }
    return cin;
}

template <int DK>
__device__ __forceinline__ v16f qk_tile(const char *img, int t, int m, int g,
                                        const v4i qB[(DK + 1) / 2], v16f cin) {
    v4i ka[(DK + 1) / 2];
    load_k_operand<DK>(img, t, m, g, ka);
    return qk_mfma<(DK + 1) / 2>(ka, qB, cin);
}

// LDS byte offset of a pointer into a __shared__ array.
__device__ __forceinline__ unsigned lds_offset(const void *p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) const char *)p;
}

// A pointer that is the same in every lane, moved into scalar registers.
template <class T>
__device__ __forceinline__ const T *uniform_ptr(const T *p) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    // (the builtin returns int: widen through unsigned, or the low half is sign-extended)
    const uint64_t u = (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)a) |
                       ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(a >> 32)) << 32);
    return reinterpret_cast<const T *>(u);
}

// One asynchronous 16-byte-per-lane copy global -> LDS: lane L's 16 bytes, read from
// sbase + voff (sbase wave-uniform, kept in scalar registers; voff this lane's byte offset),
// land at lds_base + 16 L (lds_base wave-uniform).  Issued through inline assembly so that
// the compiler does not serialise later LDS reads of OTHER buffers against it; the callers
// order it by hand (wait_vmem + barrier before the data is read).
__device__ __forceinline__ void dma16(const void *sbase, unsigned voff, unsigned lds_base) {
    const uint64_t u = reinterpret_cast<uint64_t>(uniform_ptr(static_cast<const char *>(sbase)));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(voff), "s"(u)
                 : "memory", "m0");
}

// Asynchronous copy of one block image (L::BYTES, a multiple of 1 KiB) from
// global memory straight into LDS by NW waves (wave = 0 .. NW - 1), each of
// which moves 1 KiB per instruction.
template <int DK, int NW = 4>
__device__ __forceinline__ void dma_image(const char *__restrict__ gsrc, unsigned ldst, int wave, int lane) {
    using L = Image<DK>;
    constexpr int NCH = L::BYTES / 1024;
#pragma unroll
    for (int i = 0; i < (NCH + NW - 1) / NW; ++i) {
        const int c = wave + NW * i;
        if (c < NCH) dma16(gsrc + c * 1024, lane * 16, ldst + c * 1024);
    }
}

__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// max / sum over the two lanes L and L ^ 32 (they share a query row), on the vector ALU.
__device__ __forceinline__ float pair_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace binattn

// Device routines shared by the fused attention kernel and the logits export:
// the LDS tile layout of one key/value block and the +-1 int8 QK MFMA tile.
//
// Register/lane convention (wave64, v_mfma_i32_32x32x32_i8, D = A*B + C):
//   A is 32 x 32 (rows x k), B is 32 x 32 (k x cols); lane L feeds row/col
//   (L & 31) with the 16 k-slots of group g = L >> 5.  A and B use the same
//   slot numbering, so any consistent assignment of channels (or keys) to
//   slots gives the same contraction.
//   D: lane L holds column (L & 31); register r holds row 8(r/4) + 4g + (r%4).
// The kernels put KEYS (resp. value channels) on the A side and QUERIES on the
// B side, so that every lane owns one query row: all softmax statistics are
// lane-local, and the P tile a lane produces is already in B-operand order for
// the P.V contraction (no LDS round trip).
#pragma once

#include "binattn_internal.h"

namespace binattn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));  // 16-byte staging register

constexpr int FUSED_THREADS = 256;
constexpr int KT = BV / 32;  // MFMA key tiles per block

template <int DK>
struct Tiles {
    static constexpr int DKP = 32 * DK;
    static constexpr int KP = DKP + 16;  // K row pitch (bytes); +16 keeps b128 reads conflict-free
    static constexpr int VP = BV + 16;   // V^T row pitch (bytes)
    int8_t k8[BV * KP];    // [position in block][channel]  +-1 / 0
    int8_t vt[DKP * VP];   // [channel][key offset]         V codes
    int cs[DKP];           // 128 * sum over the block's keys of the V codes
};

// 4 sign bits -> 4 bytes holding +1 (bit set) or -1 (bit clear).
__device__ __forceinline__ unsigned pm1_bytes(unsigned nib) {
    unsigned x = (nib * 0x00204081u) & 0x01010101u;
    return x | ((x ^ 0x01010101u) * 0xFFu);
}

// B operand of the QK tile for this lane's query row: +-1 bytes of channels
// 32 s + 16 g + [0, 16), zero beyond d.
template <int DK>
__device__ __forceinline__ void load_q_operand(const uint32_t *__restrict__ q_words, int d, int g,
                                               v4i qB[DK]) {
#pragma unroll
    for (int s = 0; s < DK; ++s) {
        const unsigned half = (q_words[s] >> (16 * g)) & 0xffffu;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c0 = 32 * s + 16 * g + 4 * i;
            qB[s][i] = c0 < d ? (int)pm1_bytes((half >> (4 * i)) & 0xFu) : 0;
        }
    }
}

// Integer logits of MFMA tile t of the block in LDS: for this lane's query,
// register r is the +-1 inner product with key (block start + 64 g + 16 t + r).
template <int DK>
__device__ __forceinline__ v16i qk_tile(const Tiles<DK> &T, int t, int m, int g, const v4i qB[DK]) {
    v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < DK; ++s) {
        const v4i a = *reinterpret_cast<const v4i *>(T.k8 + (32 * t + m) * Tiles<DK>::KP + 32 * s +
                                                     16 * g);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qB[s], acc, 0, 0, 0);
    }
    return acc;
}

// Cooperative copy of the K part of block `blk` (contiguous in the workspace).
template <int DK>
__device__ __forceinline__ void load_k_regs(const int8_t *__restrict__ k8_head, int blk,
                                            u4v kreg[DK]) {
    const u4v *src = reinterpret_cast<const u4v *>(k8_head + (int64_t)blk * BV * (32 * DK));
#pragma unroll
    for (int i = 0; i < DK; ++i) kreg[i] = src[threadIdx.x + FUSED_THREADS * i];
}

template <int DK>
__device__ __forceinline__ void store_k_regs(Tiles<DK> &T, const u4v kreg[DK]) {
#pragma unroll
    for (int i = 0; i < DK; ++i) {
        const int ch = threadIdx.x + FUSED_THREADS * i;
        const int row = ch / (2 * DK), part = ch % (2 * DK);
        *reinterpret_cast<u4v *>(T.k8 + row * Tiles<DK>::KP + 16 * part) = kreg[i];
    }
}

}  // namespace binattn

// Integer logits I_ij = s_i . t_j (Sec. 4.1) exported to memory, three ways:
//   * vector-ALU form: d - 2 * popcount(q XOR k) straight from the sign words
//   * int8 matrix-core form: +-1 bytes on v_mfma_i32_32x32x32_i8
//   * FP4 matrix-core form: the QK tile routine of the fused kernel
//     (v_mfma_f32_32x32x64_f8f6f4 on +-1.0 FP4 codes, exact in fp32)
// All are exact; they exist so that the forms can be compared and timed, and so
// that the fused kernel's tile routine is checked bit for bit.  Each also has a
// row-sum form (sum_j I_ij per query row instead of the N x N matrix): without the
// 4-byte-per-pair store stream the kernels are bound by how they compute the logits,
// which is what a comparison of the three forms is about.
#include "attn_tiles.h"

namespace binattn {

// One thread per (row, key).
__global__ void logits_popcount_kernel(const uint32_t *__restrict__ q_bits,
                                       const uint32_t *__restrict__ k_bits, int N, int d, int W,
                                       int row_begin, int nrows, int nper,
                                       int32_t *__restrict__ logits) {
    const int bh = blockIdx.x / nper;
    const int64_t i = (int64_t)(blockIdx.x % nper) * blockDim.x + threadIdx.x;
    if (i >= (int64_t)nrows * N) return;
    const int r = (int)(i / N), j = (int)(i % N);
    const uint32_t *qw = q_bits + ((int64_t)bh * N + row_begin + r) * W;
    const uint32_t *kw = k_bits + ((int64_t)bh * N + j) * W;
    int ham = 0;
    for (int w = 0; w < W; ++w) ham += __popc(qw[w] ^ kw[w]);
    logits[(int64_t)bh * nrows * N + i] = d - 2 * ham;
}

// Row sums only (no N x N store): one thread per query row walks all keys; the key words are
// the same for every lane of a wave (scalar loads), the per-pair work is one XOR and one
// population count per sign word (v_bcnt_u32_b32 accumulates).  sum_j I_ij = d N - 2 sum_j ham.
template <int W>
__global__ __launch_bounds__(256) void logits_popcount_rowsum_kernel(
    const uint32_t *__restrict__ q_bits, const uint32_t *__restrict__ k_bits, int N, int d,
    int row_begin, int nrows, int nper, int32_t *__restrict__ sums) {
    const int bh = blockIdx.x / nper;
    const int r = (blockIdx.x % nper) * 256 + threadIdx.x;
    const int q = min(row_begin + r, N - 1);
    uint32_t qw[W];
#pragma unroll
    for (int w = 0; w < W; ++w) qw[w] = q_bits[((int64_t)bh * N + q) * W + w];
    const uint32_t *kb = k_bits + (int64_t)bh * N * W;
    int ham = 0;
#pragma unroll 16
    for (int j = 0; j < N; ++j) {
#pragma unroll
        for (int w = 0; w < W; ++w) ham += __popc(qw[w] ^ kb[(int64_t)j * W + w]);
    }
    if (r < nrows) sums[(int64_t)bh * nrows + r] = d * N - 2 * ham;
}

// FP4 form.  One workgroup per (head, 128-row block); loops over key blocks,
// reading the operand images binattn's key preparation wrote.
template <int DK, bool ROWSUM>
__global__ __launch_bounds__(FUSED_THREADS) void logits_fp4_kernel(
    const uint32_t *__restrict__ q_bits, const char *__restrict__ img, int N, int d, int nblk,
    int row_begin, int nrows, int nrb, int32_t *__restrict__ logits) {
    using L = Image<DK>;
    __shared__ __attribute__((aligned(1024))) char buf[L::BYTES];
    const int rb = blockIdx.x % nrb, bh = blockIdx.x / nrb;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = lane & 31, g = lane >> 5;
    const int r = rb * BR + wave * ROWS_PER_WAVE + m;  // row inside [0, nrows)
    const int q = min(row_begin + r, N - 1);
    const int W = (d + 31) / 32;
    v4i qB[L::DK2];
    unsigned qw[2 * L::DK2];
#pragma unroll
    for (int w = 0; w < 2 * L::DK2; ++w) qw[w] = w < W ? q_bits[((int64_t)bh * N + q) * W + w] : 0u;
    load_q_operand<L::DK2>(qw, d, g, false, false, qB);
    const char *imgs = img + (int64_t)bh * nblk * L::BYTES;
    int32_t *orow = logits + ((int64_t)bh * nrows + r) * N;
    float rs = 0.0f;  // ROWSUM: sum of this lane's logits (exact: |sum| <= 128 N < 2^24)
    for (int blk = 0; blk < nblk; ++blk) {
        __syncthreads();  // previous block's reads are done
        dma_image<DK>(imgs + (int64_t)blk * L::BYTES, lds_offset(buf), wave, lane);
        wait_vmem();
        __syncthreads();
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const v16f zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            const v16f acc = qk_tile<DK>(buf, t, m, g, qB, zero);
            const int k0 = blk * BV + 64 * g + 16 * t;
            if (ROWSUM) {  // keys beyond N are zero rows of the image: they add nothing
#pragma unroll
                for (int i = 0; i < 16; ++i) rs += acc[i];
            } else if (r < nrows) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (k0 + i < N) orow[k0 + i] = (int32_t)acc[i];
            }
        }
    }
    if (ROWSUM) {
        rs += __shfl_xor(rs, 32, 64);  // the two halves of the keys
        if (g == 0 && r < nrows) logits[(int64_t)bh * nrows + r] = (int32_t)rs;
    }
}

// 4 sign bits -> 4 bytes holding +1 (bit set) or -1 (bit clear).
__device__ __forceinline__ unsigned pm1_bytes(unsigned nib) {
    unsigned x = (nib * 0x00204081u) & 0x01010101u;
    return x | ((x ^ 0x01010101u) * 0xFFu);
}

// int8 form: +-1 bytes are expanded from the sign words inside the kernel.
// Lane layout as in the fused kernel (keys on the A side, one query per lane).
template <int DK, bool ROWSUM>
__global__ __launch_bounds__(FUSED_THREADS) void logits_i8_kernel(
    const uint32_t *__restrict__ q_bits, const uint32_t *__restrict__ k_bits, int N, int d,
    int nblk, int row_begin, int nrows, int nrb, int32_t *__restrict__ logits) {
    constexpr int KP = 32 * DK + 16;
    __shared__ __attribute__((aligned(16))) char k8[BV * KP];
    const int rb = blockIdx.x % nrb, bh = blockIdx.x / nrb;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, g = lane >> 5;
    const int r = rb * BR + wave * ROWS_PER_WAVE + m;
    const int q = min(row_begin + r, N - 1);
    v4i qB[DK];
#pragma unroll
    for (int s = 0; s < DK; ++s) {
        const unsigned half = (q_bits[((int64_t)bh * N + q) * DK + s] >> (16 * g)) & 0xffffu;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            qB[s][i] = (32 * s + 16 * g + 4 * i < d) ? (int)pm1_bytes((half >> (4 * i)) & 0xFu) : 0;
    }
    const uint32_t *kb = k_bits + (int64_t)bh * N * DK;
    int32_t *orow = logits + ((int64_t)bh * nrows + r) * N;
    int rs = 0;  // ROWSUM: sum of this lane's logits
    for (int blk = 0; blk < nblk; ++blk) {
        __syncthreads();
        // row `pos` of the tile holds key blk*BV + pos (natural order)
        for (int i = threadIdx.x; i < BV * DK; i += FUSED_THREADS) {
            const int pos = i / DK, w = i % DK;
            const int key = blk * BV + pos;
            const uint32_t word = key < N ? kb[(int64_t)key * DK + w] : 0u;
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const bool live = key < N && 32 * w + 4 * n < d;
                *reinterpret_cast<unsigned *>(k8 + pos * KP + 32 * w + 4 * n) =
                    live ? pm1_bytes((word >> (4 * n)) & 0xFu) : 0u;
            }
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < DK; ++s) {
                const v4i a = *reinterpret_cast<const v4i *>(k8 + (32 * t + m) * KP + 32 * s + 16 * g);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qB[s], acc, 0, 0, 0);
            }
            // register i of lane group g is tile row 8 (i/4) + 4 g + (i%4)
            if (ROWSUM) {  // keys beyond N are zero rows of the tile
#pragma unroll
                for (int i = 0; i < 16; ++i) rs += acc[i];
            } else if (r < nrows) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = blk * BV + 32 * t + 8 * (i >> 2) + 4 * g + (i & 3);
                    if (key < N) orow[key] = acc[i];
                }
            }
        }
    }
    if (ROWSUM) {
        rs += __shfl_xor(rs, 32, 64);
        if (g == 0 && r < nrows) logits[(int64_t)bh * nrows + r] = rs;
    }
}

int launch_logits_popcount(const uint32_t *q_bits, const uint32_t *k_bits, const Shape &s,
                           int row_begin, int row_end, int32_t *logits, bool rowsum, hipStream_t stream) {
    const int nrows = row_end - row_begin;
    if (nrows == 0) return BINATTN_OK;
    if (rowsum) {
        const int nper = (nrows + 255) / 256;
        const dim3 grid((unsigned)nper * s.BH), block(256);
        switch (s.W) {
#define CASE(K) case K: hipLaunchKernelGGL(logits_popcount_rowsum_kernel<K>, grid, block, 0, stream, q_bits, \
                                           k_bits, s.N, s.d, row_begin, nrows, nper, logits); break;
            CASE(1) CASE(2) CASE(3) CASE(4)
#undef CASE
            default: return BINATTN_ERR_SHAPE;
        }
        return check_launch();
    }
    const int nper = (int)(((int64_t)nrows * s.N + 255) / 256);
    hipLaunchKernelGGL(logits_popcount_kernel, dim3((unsigned)nper * s.BH), dim3(256), 0, stream,
                       q_bits, k_bits, s.N, s.d, s.W, row_begin, nrows, nper, logits);
    return check_launch();
}

int launch_logits_fp4(const uint32_t *q_bits, const char *ws, const Workspace &w, const Shape &s,
                      int row_begin, int row_end, int32_t *logits, bool rowsum, hipStream_t stream) {
    const int nrows = row_end - row_begin;
    if (nrows == 0) return BINATTN_OK;
    const int nrb = (nrows + BR - 1) / BR;
    const dim3 grid((unsigned)nrb * s.BH), block(FUSED_THREADS);
    switch (s.DK) {
#define CASE(K) case K: if (rowsum) hipLaunchKernelGGL((logits_fp4_kernel<K, true>), grid, block, 0, stream, q_bits, \
                                           ws + w.img, s.N, s.d, s.nblk, row_begin, nrows, nrb, logits); \
                        else hipLaunchKernelGGL((logits_fp4_kernel<K, false>), grid, block, 0, stream, q_bits, \
                                           ws + w.img, s.N, s.d, s.nblk, row_begin, nrows, nrb, logits); break;
        CASE(1) CASE(2) CASE(3) CASE(4)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
    return check_launch();
}

int launch_logits_i8(const uint32_t *q_bits, const uint32_t *k_bits, const Shape &s, int row_begin,
                     int row_end, int32_t *logits, bool rowsum, hipStream_t stream) {
    const int nrows = row_end - row_begin;
    if (nrows == 0) return BINATTN_OK;
    const int nrb = (nrows + BR - 1) / BR;
    const dim3 grid((unsigned)nrb * s.BH), block(FUSED_THREADS);
    switch (s.DK) {
#define CASE(K) case K: if (rowsum) hipLaunchKernelGGL((logits_i8_kernel<K, true>), grid, block, 0, stream, q_bits, k_bits, \
                                           s.N, s.d, s.nblk, row_begin, nrows, nrb, logits); \
                        else hipLaunchKernelGGL((logits_i8_kernel<K, false>), grid, block, 0, stream, q_bits, k_bits, \
                                           s.N, s.d, s.nblk, row_begin, nrows, nrb, logits); break;
        CASE(1) CASE(2) CASE(3) CASE(4)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
    return check_launch();
}

}  // namespace binattn

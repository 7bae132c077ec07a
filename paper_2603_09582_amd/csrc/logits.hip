// Integer logits I_ij = s_i . t_j (Sec. 4.1) exported to memory, two ways:
//   * vector-ALU form: d - 2 * popcount(q XOR k) straight from the sign words
//   * matrix-core form: the +-1 int8 MFMA tile routine of the fused kernel
// Both are exact; they exist so that the two can be compared and timed.
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

// One workgroup per (head, 128-row block); loops over key blocks.
template <int DK>
__global__ __launch_bounds__(FUSED_THREADS) void logits_mfma_kernel(
    const uint32_t *__restrict__ q_bits, const int8_t *__restrict__ k8, int N, int d, int nblk,
    int row_begin, int nrows, int nrb, int32_t *__restrict__ logits) {
    __shared__ __attribute__((aligned(16))) Tiles<DK> T;
    const int rb = blockIdx.x % nrb, bh = blockIdx.x / nrb;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, g = lane >> 5;
    const int r = rb * BR + wave * ROWS_PER_WAVE + m;  // row inside [0, nrows)
    const int q = min(row_begin + r, N - 1);
    v4i qB[DK];
    load_q_operand<DK>(q_bits + ((int64_t)bh * N + q) * DK, d, g, qB);
    const int8_t *k8h = k8 + (int64_t)bh * nblk * BV * (32 * DK);
    int32_t *orow = logits + ((int64_t)bh * nrows + r) * N;
    for (int blk = 0; blk < nblk; ++blk) {
        u4v kreg[DK];
        load_k_regs<DK>(k8h, blk, kreg);
        __syncthreads();  // previous block's reads are done
        store_k_regs<DK>(T, kreg);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const v16i acc = qk_tile<DK>(T, t, m, g, qB);
            const int k0 = blk * BV + 64 * g + 16 * t;
            if (r < nrows) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (k0 + i < N) orow[k0 + i] = acc[i];
            }
        }
    }
}

int launch_logits_popcount(const uint32_t *q_bits, const uint32_t *k_bits, const Shape &s,
                           int row_begin, int row_end, int32_t *logits, hipStream_t stream) {
    const int nrows = row_end - row_begin;
    if (nrows == 0) return BINATTN_OK;
    const int nper = (int)(((int64_t)nrows * s.N + 255) / 256);
    hipLaunchKernelGGL(logits_popcount_kernel, dim3((unsigned)nper * s.BH), dim3(256), 0, stream,
                       q_bits, k_bits, s.N, s.d, s.W, row_begin, nrows, nper, logits);
    return check_launch();
}

int launch_logits_mfma(const uint32_t *q_bits, const int8_t *k8, const Shape &s, int row_begin,
                       int row_end, int32_t *logits, hipStream_t stream) {
    const int nrows = row_end - row_begin;
    if (nrows == 0) return BINATTN_OK;
    const int nrb = (nrows + BR - 1) / BR;
    const dim3 grid((unsigned)nrb * s.BH), block(FUSED_THREADS);
    switch (s.DK) {
#define CASE(K) case K: hipLaunchKernelGGL(logits_mfma_kernel<K>, grid, block, 0, stream, q_bits, k8, \
                                           s.N, s.d, s.nblk, row_begin, nrows, nrb, logits); break;
        CASE(1) CASE(2) CASE(3) CASE(4)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
    return check_launch();
}

}  // namespace binattn

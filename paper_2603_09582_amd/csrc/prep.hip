// Operand preparation for the fused kernel.  Both kernels write straight into
// the per-block operand images (see Image<DK>) that the attention kernel copies
// into LDS:
//   * K sign words -> FP4 codes of +-1, rows in the order the QK MFMA tile
//     wants them
//   * psi of Alg. 1 (Eq. 7): per-channel absmax of V, delta_v, signed 8-bit
//     codes stored channel-major, and the accumulator seed of the P.V
//     contraction (128 * column sums per key block, see fused_impl.h)
// All are HBM-bound streaming kernels.
#include "quant_v.h"

namespace binattn {

constexpr int PREP_THREADS = 256;

// Key block `blk` of one head: sign words -> FP4 rows of the block image.
// One thread per (row position, sign word): 32 channels -> 16 bytes of FP4 codes.
__device__ __forceinline__ void expand_k_block(const uint32_t *__restrict__ kb, int N, int d, int W,
                                               int blk, int KP, char *__restrict__ dst) {
    const int W2 = 2 * ((W + 1) / 2);  // words per row incl. the zero word that pads to 64 channels
    for (int i = threadIdx.x; i < BV * W2; i += PREP_THREADS) {
        const int pos = i / W2, w = i % W2;
        const int key = blk * BV + key_of_position(pos);
        const bool live = key < N && w < W;
        const uint32_t word = live ? kb[(int64_t)key * W + w] : 0u;
        const int valid = live ? d - 32 * w : 0;  // real channels in this word
        u4 o;
#pragma unroll
        for (int n = 0; n < 4; ++n)
            o[n] = (8 * n < valid) ? fp4_pm1_from_bits8((word >> (8 * n)) & 0xFFu) : 0u;
        *reinterpret_cast<u4 *>(dst + (int64_t)pos * KP + 16 * k_chunk(pos, w, KP)) = o;
    }
}

__global__ __launch_bounds__(PREP_THREADS) void expand_k_kernel(const uint32_t *__restrict__ k_bits,
                                                                int N, int d, int W, int nblk,
                                                                int img_bytes, int KP,
                                                                char *__restrict__ img) {
    const int blk = blockIdx.x % nblk, bh = blockIdx.x / nblk;
    expand_k_block(k_bits + (int64_t)bh * N * W, N, d, W, blk, KP,
                   img + ((int64_t)bh * nblk + blk) * img_bytes);
}

// absmax over token rows [n0, n1) of one head, all threads of the workgroup:
// on return thread c < 8 * C16 holds max_n |v[n][c]| (other threads 0).
// smax: LDS scratch of (PREP_THREADS / C16) * 8 * C16 floats.
template <int C16>
__device__ __forceinline__ float absmax_rows(const uint16_t *__restrict__ vb, int64_t stride_n,
                                             int n0, int n1, float *smax) {
    constexpr int RT = PREP_THREADS / C16;  // token rows per pass
    constexpr int D = 8 * C16;
    const int c = threadIdx.x % C16, r0 = threadIdx.x / C16;
    if (r0 < RT) {
        unsigned mb[4] = {0u, 0u, 0u, 0u};
        // four rows per trip, their loads issued together (the loop is latency-bound)
        const u4 zero4 = {0u, 0u, 0u, 0u};
        for (int n = n0 + r0; n < n1; n += 4 * RT) {
            u4 w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                w[k] = (n + k * RT < n1)
                           ? *reinterpret_cast<const u4 *>(vb + (int64_t)(n + k * RT) * stride_n + 8 * c)
                           : zero4;
#pragma unroll
            for (int k = 0; k < 4; ++k) absmax_acc(mb, w[k]);
        }
        float m[8];
        absmax_floats(mb, m);
#pragma unroll
        for (int i = 0; i < 8; ++i) smax[r0 * D + 8 * c + i] = m[i];
    }
    __syncthreads();
    float a = 0.0f;
    if (threadIdx.x < D)
        for (int r = 0; r < RT; ++r) a = fmaxf(a, smax[r * D + threadIdx.x]);
    return a;
}

// Key block `blk` of one head: codes (channel-major) and the accumulator seeds
// into the block image.  sdelta (LDS) holds the head's per-channel scales;
// tile is LDS scratch of 128 * (BV + 16) bytes.
template <int C16>
__device__ __forceinline__ void quant_v_block(const uint16_t *__restrict__ vb, int64_t stride_n,
                                              int N, int DKP, int blk, const float *sdelta,
                                              const float *srlo, const float *srhi, int8_t *tile,
                                              int v_off, int cs_off, char *__restrict__ dst) {
    constexpr int LDT = BV + 16;  // LDS row pitch in bytes = Image::VP
    for (int i = threadIdx.x; i < DKP * LDT / 4; i += PREP_THREADS)
        reinterpret_cast<uint32_t *>(tile)[i] = 0u;
    __syncthreads();

    // One thread per (4 consecutive tokens, 8-channel chunk); consecutive lanes take
    // consecutive chunks of the same tokens, so every load instruction reads whole token
    // rows.  The transposed 4-byte LDS writes of a wave (8 token quads x 8 chunks at d = 64)
    // would fall on 16 banks; XOR-ing bits of the chunk index into the quad's column spreads
    // them over all 64 (the copy-out below undoes it at 16-byte granularity).
    const int j0 = blk * BV;
    const int nrow = min(BV, N - j0);
    for (int e = threadIdx.x; e < C16 * (BV / 4); e += PREP_THREADS) {
        const int c = e % C16, jq = e / C16;
        unsigned packed[8];
        u4 w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {  // rows beyond the block's end read as zeros: code 0
            w[k] = u4{0u, 0u, 0u, 0u};
            if (4 * jq + k < nrow)
                w[k] = *reinterpret_cast<const u4 *>(vb + (int64_t)(j0 + 4 * jq + k) * stride_n + 8 * c);
        }
        quant_quad(w, load_quant_consts8(sdelta, srlo, srhi, c), packed);
        const int col = jq ^ (((c >> 1) & 3) << 3);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<unsigned *>(tile + (8 * c + i) * LDT + 4 * col) = packed[i];
    }
    __syncthreads();

    for (int i = threadIdx.x; i < DKP * (BV / 16); i += PREP_THREADS) {
        const int c = i / (BV / 16), part = i % (BV / 16);
        const int spart = part ^ (((c >> 4) & 3) << 1);  // where the writer put this token group
        const u4 val = *reinterpret_cast<const u4 *>(tile + c * LDT + 16 * spart);
        *reinterpret_cast<u4 *>(dst + v_off + c * LDT + 16 * part) = val;
    }
    if (threadIdx.x < DKP) {  // column sums: 16 bytes per read, four signed bytes per dot
        int sum = 0;
#pragma unroll
        for (int j = 0; j < BV / 16; ++j) {
            const u4 w = *reinterpret_cast<const u4 *>(tile + threadIdx.x * LDT + 16 * j);
#pragma unroll
            for (int n = 0; n < 4; ++n) sum = __builtin_amdgcn_sdot4((int)w[n], 0x01010101, sum, false);
        }
        reinterpret_cast<int *>(dst + cs_off)[threadIdx.x] = PV_MAGIC_BITS + 128 * sum;
    }
}

// Long sequences, step 1: partial absmax over VCHUNK token rows, amax[bh][chunk][c].
template <int C16>
__global__ __launch_bounds__(PREP_THREADS) void v_absmax_kernel(const uint16_t *__restrict__ v,
                                                                Strides3 vs, int H, int N, int DKP,
                                                                int nchunk,
                                                                float *__restrict__ amax) {
    __shared__ float smax[(PREP_THREADS / C16) * 8 * C16];
    const int chunk = blockIdx.x % nchunk, bh = blockIdx.x / nchunk;
    const int b = bh / H, h = bh % H;
    const uint16_t *vb = v + (int64_t)b * vs.b + (int64_t)h * vs.h;
    const float a = absmax_rows<C16>(vb, vs.n, chunk * VCHUNK, min(N, chunk * VCHUNK + VCHUNK), smax);
    if (threadIdx.x < 8 * C16) amax[((int64_t)bh * nchunk + chunk) * DKP + threadIdx.x] = a;
}

// Longer sequences, step 2: one key block of one head (V codes and, if k_bits is
// not null, the key operand).
// Optional last step of Eq. 5's abs-means in v_quant_kernel: the per-chunk partial sums of |q|
// and |k| written by phi_psi1_kernel are added in a FIXED order (each lane its chunks in
// ascending order, then a fixed shuffle tree), so the means are the same bits on every run.
struct MuReduce {
    const float *psum;          // [BH][nchunk][2], or null: nothing to do
    float *mu_q, *mu_k;         // [BH]
    float *mu_q_out, *mu_k_out; // optional copies for the caller
    float inv_count;
};

template <int C16>
__global__ __launch_bounds__(PREP_THREADS) void v_quant_kernel(
    const uint16_t *__restrict__ v, Strides3 vs, const uint32_t *__restrict__ k_bits, int H, int N,
    int d, int DKP, int nchunk, int nblk, const float *__restrict__ amax, float *__restrict__ delta,
    int img_bytes, int KP, int v_off, int cs_off, char *__restrict__ img, MuReduce mr, int bpw) {
    // A workgroup takes bpw consecutive key blocks of one head (more than one for long
    // sequences, where re-reading all absmax partials for every single block would cost more
    // than the block itself).
    __shared__ __attribute__((aligned(16))) float sdelta[8 * C16], srlo[8 * C16], srhi[8 * C16];
    __shared__ __attribute__((aligned(16))) int8_t tile[128 * (BV + 16)];
    const int ngrp = (nblk + bpw - 1) / bpw;
    const int blk0 = (blockIdx.x % ngrp) * bpw, bh = blockIdx.x / ngrp;
    const int b = bh / H, h = bh % H;
    const uint16_t *vb = v + (int64_t)b * vs.b + (int64_t)h * vs.h;
    if (k_bits != nullptr) {
        const int W = (d + 31) / 32;
        for (int blk = blk0; blk < min(nblk, blk0 + bpw); ++blk)
            expand_k_block(k_bits + (int64_t)bh * N * W, N, d, W, blk, KP, img + ((int64_t)bh * nblk + blk) * img_bytes);
    }
    if (mr.psum != nullptr && blk0 == 0 && threadIdx.x < 64) {
        const float *ps = mr.psum + (int64_t)bh * nchunk * 2;
        float sq = 0.0f, sk = 0.0f;
        for (int j = threadIdx.x; j < nchunk; j += 64) {
            sq += ps[2 * j];
            sk += ps[2 * j + 1];
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            sq += __shfl_down(sq, off, 64);
            sk += __shfl_down(sk, off, 64);
        }
        if (threadIdx.x == 0) {
            const float mq = sq * mr.inv_count, mk = sk * mr.inv_count;
            mr.mu_q[bh] = mq;
            mr.mu_k[bh] = mk;
            if (mr.mu_q_out) mr.mu_q_out[bh] = mq;
            if (mr.mu_k_out) mr.mu_k_out[bh] = mk;
        }
    }
    // The head's absmax from the per-chunk partials: all threads load (independent,
    // coalesced), the maximum is taken in LDS on the bit patterns (non-negative floats
    // order like integers).
    __shared__ int sabs[8 * C16];
    if (threadIdx.x < 8 * C16) sabs[threadIdx.x] = 0;
    __syncthreads();
    {
        const float *am = amax + (int64_t)bh * nchunk * DKP;
        const int total = nchunk * DKP;
        for (int i0 = threadIdx.x; i0 < total; i0 += 4 * PREP_THREADS) {
            float a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * PREP_THREADS;
                a[u] = i < total ? am[i] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = (i0 + u * PREP_THREADS) % DKP;
                if (c < 8 * C16 && a[u] > 0.0f) atomicMax(&sabs[c], __float_as_int(a[u]));
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < 8 * C16) {
        float dl;
        quant_consts(__int_as_float(sabs[threadIdx.x]), &dl, &srlo[threadIdx.x], &srhi[threadIdx.x]);
        sdelta[threadIdx.x] = dl;
        if (blk0 == 0) delta[(int64_t)bh * DKP + threadIdx.x] = dl;
    }
    for (int blk = blk0; blk < min(nblk, blk0 + bpw); ++blk) {
        quant_v_block<C16>(vb, vs.n, N, DKP, blk, sdelta, srlo, srhi, tile, v_off, cs_off,
                           img + ((int64_t)bh * nblk + blk) * img_bytes);
        __syncthreads();  // the tile is reused
    }
}

// Inverse of key_of_position: where key offset o (0 <= o < BV) sits in a block image.
__device__ __forceinline__ int position_of_key(int o) {
    const int g = o >> 6, t = (o >> 4) & 3, r = o & 15;
    return 32 * t + 8 * (r >> 2) + 4 * g + (r & 3);
}

// phi of Alg. 1 (Eq. 5) for Q and K and the first half of psi (Eq. 7) in ONE pass over the bf16
// inputs, for the entry point that takes Q, K and V themselves: a workgroup owns the BV = 128
// tokens of one key block of one head (many small workgroups: the loads of one overlap the
// arithmetic of its neighbours on the compute unit) and
//   * packs the sign words of its queries (assembled per token in LDS, stored as whole words),
//   * turns the signs of its keys straight into the FP4 rows of the block images (the key
//     sign words never exist in memory),
//   * reduces the per-channel absmax of its V rows (the partials the quantisation launch
//     combines), and
//   * leaves its partial sums of |q| and |k| for the fixed-order reduction of the abs-means.
// A thread owns one 8-channel chunk of every RT-th token, so consecutive lanes read whole
// rows; all of a thread's loads go out before the first is used.
struct PhiPsi1Args {
    const uint16_t *q, *k, *v;
    Strides3 qs, ks, vs;
    uint32_t *q_bits;   // [BH][N][W]
    char *img;          // block images
    float *amax;        // [BH][nblk][DKP]: one partial per key block
    float *psum;        // [BH][nblk][2]
    int H, N, d, DKP, nblk, img_bytes;
};

template <int C16>
__global__ __launch_bounds__(PREP_THREADS) void phi_psi1_kernel(const PhiPsi1Args a) {
    constexpr int W = (C16 + 3) / 4;
    constexpr int RT = PREP_THREADS / C16;            // tokens per pass
    constexpr int NP = (BV + RT - 1) / RT;            // passes
    constexpr int D = 8 * C16;
    constexpr int KW = 8 * ((W + 1) / 2);             // 4-byte words (8 channels each) per image row
    __shared__ uint32_t words[BV * W];
    __shared__ float smax[RT * D];
    __shared__ float wsum[2][PREP_THREADS / 64];
    const int chunk = blockIdx.x % a.nblk, bh = blockIdx.x / a.nblk;  // chunk = key block
    const int b = bh / a.H, h = bh % a.H;
    const int N = a.N, n0 = chunk * BV, n1 = min(N, n0 + BV);
    char *image = a.img + ((int64_t)bh * a.nblk + chunk) * a.img_bytes;
    const uint16_t *qb = a.q + (int64_t)b * a.qs.b + (int64_t)h * a.qs.h;
    const uint16_t *kb = a.k + (int64_t)b * a.ks.b + (int64_t)h * a.ks.h;
    const uint16_t *vb = a.v + (int64_t)b * a.vs.b + (int64_t)h * a.vs.h;
    const int c = threadIdx.x % C16, r0 = threadIdx.x / C16;
    const bool on = r0 < RT;

    // (unconditional loads from clamped rows, masked where they are used)
    u4 xq[NP], xk[NP], xv[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int tok = min(n0 + r0 + p * RT, N - 1);
        xq[p] = *reinterpret_cast<const u4 *>(qb + (int64_t)tok * a.qs.n + 8 * c);
        xk[p] = *reinterpret_cast<const u4 *>(kb + (int64_t)tok * a.ks.n + 8 * c);
        xv[p] = *reinterpret_cast<const u4 *>(vb + (int64_t)tok * a.vs.n + 8 * c);
    }
    for (int i = threadIdx.x; i < BV * W; i += PREP_THREADS) words[i] = 0u;
    // image words no key of the sequence fills: channels beyond d, positions beyond N
    for (int i = threadIdx.x; i < BV * KW; i += PREP_THREADS) {
        const int pos = i / KW, w4 = i % KW;
        const int key = n0 + key_of_position(pos);
        if (key >= N || w4 >= C16)
            *reinterpret_cast<unsigned *>(image + pos * (4 * KW) + 16 * k_chunk(pos, w4 >> 2, 4 * KW) + 4 * (w4 & 3)) = 0u;
    }
    __syncthreads();

    float qsum = 0.0f, ksum = 0.0f;
    unsigned mb[4] = {0u, 0u, 0u, 0u};
    uint8_t *bytes = reinterpret_cast<uint8_t *>(words);
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int tok = n0 + r0 + p * RT;
        if (on && r0 + p * RT < BV && tok < n1) {
            bytes[(tok - n0) * (4 * W) + c] = (uint8_t)sign_bits8_abs(xq[p], qsum);
            const unsigned kbits = sign_bits8_abs(xk[p], ksum);
            const int pos = position_of_key(tok - n0);
            *reinterpret_cast<unsigned *>(image + pos * (4 * KW) + 16 * k_chunk(pos, c >> 2, 4 * KW) + 4 * (c & 3)) =
                fp4_pm1_from_bits8(kbits);
            absmax_acc(mb, xv[p]);
        }
    }
    if (on) {
        float m[8];
        absmax_floats(mb, m);
#pragma unroll
        for (int i = 0; i < 8; ++i) smax[r0 * D + 8 * c + i] = m[i];
    }
    // the two partial sums of the workgroup, in a fixed order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        qsum += __shfl_down(qsum, off, 64);
        ksum += __shfl_down(ksum, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        wsum[0][threadIdx.x >> 6] = qsum;
        wsum[1][threadIdx.x >> 6] = ksum;
    }
    __syncthreads();
    if (threadIdx.x < D) {
        float m = 0.0f;
        for (int r = 0; r < RT; ++r) m = fmaxf(m, smax[r * D + threadIdx.x]);
        a.amax[((int64_t)bh * a.nblk + chunk) * a.DKP + threadIdx.x] = m;
    }
    if (threadIdx.x < 2) {
        float t = 0.0f;
        for (int i = 0; i < PREP_THREADS / 64; ++i) t += wsum[threadIdx.x][i];
        a.psum[((int64_t)bh * a.nblk + chunk) * 2 + threadIdx.x] = t;
    }
    uint32_t *ob = a.q_bits + ((int64_t)bh * N + n0) * W;
    for (int i = threadIdx.x; i < (n1 - n0) * W; i += PREP_THREADS) ob[i] = words[i];
}

// Short sequences (at most two key blocks): everything for one head in ONE launch and ONE
// pass over V.  All of the head's V rows go into registers first (a thread owns quads of
// consecutive tokens of one 8-channel chunk; consecutive lanes take consecutive chunks, so a
// load instruction reads whole token rows), the absmax is reduced through LDS, and the codes
// are made from the same registers; nothing is read twice and only one load latency is paid.
template <int C16>
__global__ __launch_bounds__(PREP_THREADS) void prep_head_kernel(
    const uint16_t *__restrict__ v, Strides3 vs, const uint32_t *__restrict__ k_bits, int H, int N,
    int d, int DKP, int nblk, float *__restrict__ delta, int img_bytes, int KP, int v_off, int cs_off,
    char *__restrict__ img) {
    constexpr int RT = PREP_THREADS / C16;  // thread groups = token quads per pass
    constexpr int D = 8 * C16;
    constexpr int NQ = 2 * BV / 4;          // token quads of two key blocks
    constexpr int MAXQ = (NQ + RT - 1) / RT;
    constexpr int LDT = BV + 16;            // = Image::VP
    __shared__ float smax[RT * D];
    __shared__ __attribute__((aligned(16))) float sdelta[D], srlo[D], srhi[D];
    __shared__ __attribute__((aligned(16))) int8_t tile[2 * 128 * LDT];
    const int bh = blockIdx.x, b = bh / H, h = bh % H;
    const int W = (d + 31) / 32;
    const uint16_t *vb = v + (int64_t)b * vs.b + (int64_t)h * vs.h;
    char *dst = img + (int64_t)bh * nblk * img_bytes;
    const int c = threadIdx.x % C16, r0 = threadIdx.x / C16;
    const bool on = r0 < RT;

    u4 w[MAXQ][4];
#pragma unroll
    for (int k = 0; k < MAXQ; ++k)
#pragma unroll
        for (int t = 0; t < 4; ++t) {  // rows beyond N read as zeros: no effect on a maximum, code 0
            const int row = 4 * (r0 + k * RT) + t;
            w[k][t] = u4{0u, 0u, 0u, 0u};
            if (on && row < N) w[k][t] = *reinterpret_cast<const u4 *>(vb + (int64_t)row * vs.n + 8 * c);
        }
    for (int blk = 0; blk < nblk; ++blk)
        expand_k_block(k_bits + (int64_t)bh * N * W, N, d, W, blk, KP, dst + (int64_t)blk * img_bytes);
    for (int i = threadIdx.x; i < nblk * DKP * LDT / 4; i += PREP_THREADS)
        reinterpret_cast<uint32_t *>(tile)[i] = 0u;

    if (on) {
        unsigned mb[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < MAXQ; ++k)
#pragma unroll
            for (int t = 0; t < 4; ++t) absmax_acc(mb, w[k][t]);
        float m[8];
        absmax_floats(mb, m);
#pragma unroll
        for (int i = 0; i < 8; ++i) smax[r0 * D + 8 * c + i] = m[i];
    }
    __syncthreads();
    if (threadIdx.x < D) {
        float a = 0.0f;
        for (int r = 0; r < RT; ++r) a = fmaxf(a, smax[r * D + threadIdx.x]);
        float dl;
        quant_consts(a, &dl, &srlo[threadIdx.x], &srhi[threadIdx.x]);
        sdelta[threadIdx.x] = dl;
        delta[(int64_t)bh * DKP + threadIdx.x] = dl;
    }
    __syncthreads();

    if (on) {
        const QuantConsts8 kc = load_quant_consts8(sdelta, srlo, srhi, c);
#pragma unroll
        for (int k = 0; k < MAXQ; ++k) {
            const int quad = r0 + k * RT;
            if (4 * quad < N && quad < NQ) {
                unsigned packed[8];
                quant_quad(w[k], kc, packed);
                const int blk = quad / (BV / 4), jq = quad % (BV / 4);
                const int col = jq ^ (((c >> 1) & 3) << 3);  // see quant_v_block
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    *reinterpret_cast<unsigned *>(tile + (blk * DKP + 8 * c + i) * LDT + 4 * col) = packed[i];
            }
        }
    }
    __syncthreads();

    for (int i = threadIdx.x; i < nblk * DKP * (BV / 16); i += PREP_THREADS) {
        const int row = i / (BV / 16), part = i % (BV / 16);  // row = blk * DKP + channel
        const int blk = row / DKP, ch = row % DKP;
        const int spart = part ^ (((ch >> 4) & 3) << 1);
        const u4 val = *reinterpret_cast<const u4 *>(tile + row * LDT + 16 * spart);
        *reinterpret_cast<u4 *>(dst + (int64_t)blk * img_bytes + v_off + ch * LDT + 16 * part) = val;
    }
    if (threadIdx.x < nblk * DKP) {  // column sums: 16 bytes per read, four signed bytes per dot
        const int blk = threadIdx.x / DKP, ch = threadIdx.x % DKP;
        int sum = 0;
#pragma unroll
        for (int j = 0; j < BV / 16; ++j) {
            const u4 x = *reinterpret_cast<const u4 *>(tile + threadIdx.x * LDT + 16 * j);
#pragma unroll
            for (int n = 0; n < 4; ++n) sum = __builtin_amdgcn_sdot4((int)x[n], 0x01010101, sum, false);
        }
        reinterpret_cast<int *>(dst + (int64_t)blk * img_bytes + cs_off)[ch] = PV_MAGIC_BITS + 128 * sum;
    }
}

// Codes and delta from the private layout into [B,H,N,d] / [B,H,d].
__global__ void export_vq_kernel(const char *__restrict__ img, const float *__restrict__ dl, int N,
                                 int d, int DKP, int nblk, int img_bytes, int v_off, int nper,
                                 int8_t *__restrict__ vq, float *__restrict__ delta) {
    const int bh = blockIdx.x / nper;
    const int64_t i = (int64_t)(blockIdx.x % nper) * blockDim.x + threadIdx.x;
    if (i < (int64_t)N * d) {
        const int n = (int)(i / d), c = (int)(i % d);
        const char *src = img + ((int64_t)bh * nblk + n / BV) * img_bytes + v_off;
        vq[(int64_t)bh * N * d + i] = (int8_t)src[c * (BV + 16) + (n % BV)];
    }
    if (i < d) delta[(int64_t)bh * d + i] = dl[(int64_t)bh * DKP + i];
}

static void image_offsets(int DK, int *KP, int *v_off, int *cs_off) {
    switch (DK) {
#define CASE(K) case K: *KP = Image<K>::KP; *v_off = Image<K>::V_OFF; *cs_off = Image<K>::CS_OFF; break;
        CASE(1) CASE(2) CASE(3) default: CASE(4)
#undef CASE
    }
}

int launch_expand_k(const uint32_t *k_bits, const Shape &s, char *ws, const Workspace &w,
                    hipStream_t stream) {
    int KP, v_off, cs_off;
    image_offsets(s.DK, &KP, &v_off, &cs_off);
    hipLaunchKernelGGL(expand_k_kernel, dim3((unsigned)s.nblk * s.BH), dim3(PREP_THREADS), 0,
                       stream, k_bits, s.N, s.d, s.W, s.nblk, w.img_bytes, KP, ws + w.img);
    return check_launch();
}

// Sequences up to this many key blocks take the single-launch path (one workgroup per
// head); longer ones take absmax partials + one more launch.
constexpr int PREP_FUSED_MAX_BLOCKS = 2;

template <int C16>
static void launch_quant_v_t(const void *v, Strides3 vs, const uint32_t *k_bits, const Shape &s,
                             char *ws, const Workspace &w, hipStream_t stream) {
    const uint16_t *vp = static_cast<const uint16_t *>(v);
    float *amax = reinterpret_cast<float *>(ws + w.amax);
    float *delta = reinterpret_cast<float *>(ws + w.delta);
    int KP, v_off, cs_off;
    image_offsets(s.DK, &KP, &v_off, &cs_off);
    if (k_bits != nullptr && s.nblk <= PREP_FUSED_MAX_BLOCKS) {
        hipLaunchKernelGGL(prep_head_kernel<C16>, dim3((unsigned)s.BH), dim3(PREP_THREADS), 0, stream,
                           vp, vs, k_bits, s.H, s.N, s.d, s.DKP, s.nblk, delta, w.img_bytes, KP,
                           v_off, cs_off, ws + w.img);
        return;
    }
    hipLaunchKernelGGL(v_absmax_kernel<C16>, dim3((unsigned)s.nchunk * s.BH), dim3(PREP_THREADS),
                       0, stream, vp, vs, s.H, s.N, s.DKP, s.nchunk, amax);
    hipLaunchKernelGGL(v_quant_kernel<C16>, dim3((unsigned)s.nblk * s.BH), dim3(PREP_THREADS), 0,
                       stream, vp, vs, k_bits, s.H, s.N, s.d, s.DKP, s.nchunk, s.nblk, amax, delta,
                       w.img_bytes, KP, v_off, cs_off, ws + w.img, MuReduce{nullptr, nullptr, nullptr, nullptr, nullptr, 0.0f}, 1);
}

// phi + psi for the entry point that takes Q, K, V: two launches (see phi_psi1_kernel).
template <int C16>
static void launch_phi_psi_t(const void *q, Strides3 qs, const void *k, Strides3 ks, const void *v, Strides3 vs,
                             const Shape &s, char *ws, const Workspace &w, float *mu_q_out, float *mu_k_out,
                             hipStream_t stream) {
    int KP, v_off, cs_off;
    image_offsets(s.DK, &KP, &v_off, &cs_off);
    float *amax = reinterpret_cast<float *>(ws + w.amax);
    float *delta = reinterpret_cast<float *>(ws + w.delta);
    float *psum = reinterpret_cast<float *>(ws + w.psum);
    float *mu = reinterpret_cast<float *>(ws + w.mu);
    PhiPsi1Args a;
    a.q = static_cast<const uint16_t *>(q); a.k = static_cast<const uint16_t *>(k); a.v = static_cast<const uint16_t *>(v);
    a.qs = qs; a.ks = ks; a.vs = vs;
    a.q_bits = reinterpret_cast<uint32_t *>(ws + w.qbits);
    a.img = ws + w.img; a.amax = amax; a.psum = psum;
    a.H = s.H; a.N = s.N; a.d = s.d; a.DKP = s.DKP; a.nblk = s.nblk;
    a.img_bytes = w.img_bytes;
    hipLaunchKernelGGL(phi_psi1_kernel<C16>, dim3((unsigned)s.nblk * s.BH), dim3(PREP_THREADS), 0, stream, a);
    const MuReduce mr = {psum, mu, mu + s.BH, mu_q_out, mu_k_out, (float)(1.0 / ((double)s.N * (double)s.d))};
    // long sequences: several key blocks per workgroup while the grid still fills the chip
    int bpw = 1;
    while (bpw < 8 && s.nblk >= 16 * bpw && (int64_t)s.BH * (s.nblk / (2 * bpw)) >= 1024) bpw *= 2;
    const int ngrp = (s.nblk + bpw - 1) / bpw;
    hipLaunchKernelGGL(v_quant_kernel<C16>, dim3((unsigned)ngrp * s.BH), dim3(PREP_THREADS), 0, stream,
                       a.v, vs, static_cast<const uint32_t *>(nullptr), s.H, s.N, s.d, s.DKP, /*partials per head*/ s.nblk,
                       s.nblk, amax, delta, w.img_bytes, KP, v_off, cs_off, ws + w.img, mr, bpw);
}

int launch_phi_psi(const void *q, Strides3 qs, const void *k, Strides3 ks, const void *v, Strides3 vs,
                   const Shape &s, char *ws, const Workspace &w, float *mu_q_out, float *mu_k_out,
                   hipStream_t stream) {
    switch (s.d / 8) {
#define CASE(c) case c: launch_phi_psi_t<c>(q, qs, k, ks, v, vs, s, ws, w, mu_q_out, mu_k_out, stream); break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
    return check_launch();
}

// V quantisation and (if k_bits is not null) the key operand into the block images.
int launch_prepare(const void *v, Strides3 vs, const uint32_t *k_bits, const Shape &s, char *ws,
                   const Workspace &w, hipStream_t stream) {
    switch (s.d / 8) {
#define CASE(c) case c: launch_quant_v_t<c>(v, vs, k_bits, s, ws, w, stream); break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
    return check_launch();
}

int launch_export_vq(const Shape &s, const char *ws, const Workspace &w, int8_t *vq, float *delta,
                     hipStream_t stream) {
    const int64_t total = (int64_t)s.N * s.d;
    const int nper = (int)((total + 255) / 256);
    int KP, v_off, cs_off;
    image_offsets(s.DK, &KP, &v_off, &cs_off);
    hipLaunchKernelGGL(export_vq_kernel, dim3((unsigned)nper * s.BH), dim3(256), 0, stream,
                       ws + w.img, reinterpret_cast<const float *>(ws + w.delta), s.N, s.d, s.DKP,
                       s.nblk, w.img_bytes, v_off, nper, vq, delta);
    return check_launch();
}

}  // namespace binattn

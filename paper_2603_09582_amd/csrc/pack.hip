// phi of Alg. 1 (Eq. 5): sign bits and the abs-mean scale of Q or K.
//
// HBM-bound streaming kernel: every lane loads 16 contiguous bytes (8 bf16
// channels of one token), turns them into 8 sign bits and one partial |x| sum.
// The sign bytes of a tile of tokens are assembled in LDS and written out as
// whole uint32 words, fully coalesced.  Q and K go through one launch.
#include "quant_v.h"

namespace binattn {

constexpr int PACK_THREADS = 256;
constexpr int PACK_TOKENS = 128;  // tokens per workgroup

__global__ void zero_f32_kernel(float *a, float *b, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        a[i] = 0.0f;
        b[i] = 0.0f;
    }
}

typedef u4 u4p;

struct PackSide {
    const uint16_t *x;
    Strides3 xs;
    uint32_t *bits;
    float *mu;
};

// One tile of PACK_TOKENS tokens of one head: sign bytes assembled in LDS, then
// written as whole words.  Returns this thread's partial sum of |x|.
template <int C16, int PACK_THREADS, int PACK_TOKENS>
__device__ __forceinline__ float pack_tile(const uint16_t *__restrict__ xb, int64_t stride_n, int n0,
                                           int ntok, uint32_t *__restrict__ ob, uint32_t *words) {
    constexpr int W = (C16 + 3) / 4;  // words per token
    for (int i = threadIdx.x; i < PACK_TOKENS * W; i += PACK_THREADS) words[i] = 0u;
    __syncthreads();
    uint8_t *bytes = reinterpret_cast<uint8_t *>(words);
    float asum = 0.0f;
    // all loads of this thread go out before the first is used (the tile is latency-bound)
    constexpr int PER = (PACK_TOKENS * C16 + PACK_THREADS - 1) / PACK_THREADS;
    u4p v[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int e = threadIdx.x + k * PACK_THREADS;
        if (e < ntok * C16)
            v[k] = *reinterpret_cast<const u4p *>(xb + (int64_t)(n0 + e / C16) * stride_n + 8 * (e % C16));
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int e = threadIdx.x + k * PACK_THREADS;
        if (e < ntok * C16)
            bytes[(e / C16) * (4 * W) + (e % C16)] =
                (uint8_t)sign_bits8_abs(v[k], asum);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < ntok * W; i += PACK_THREADS) ob[i] = words[i];
    return asum;
}

template <int PACK_THREADS>
__device__ __forceinline__ float block_sum(float v, float *wsum) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.0f;
    for (int i = 0; i < PACK_THREADS / 64; ++i) t += wsum[i];
    return t;
}

// Long sequences: streaming form without LDS staging.  A lane owns one 16-byte chunk
// (8 channels) of a token; a token takes 4 W consecutive lanes (slots past d stay idle), so
// the four chunks of one 32-channel word sit in one lane quad and the word is assembled
// with three quad broadcasts.  A workgroup streams PACK_STREAM_TOKENS tokens of one
// (tensor, head), four loads in flight per lane; mu through one float atomic per workgroup
// into a zeroed buffer.
constexpr int PACK_STREAM_TOKENS = 512;

template <int K>
__device__ __forceinline__ unsigned quad_bcast(unsigned x) {  // value of lane K of this lane's quad
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, K * 0x55, 0xf, 0xf, true);
}

template <int C16>
__global__ __launch_bounds__(PACK_THREADS) void pack_stream_kernel(PackSide q, PackSide k, int BH,
                                                                   int H, int N, int nseg,
                                                                   float inv_count) {
    constexpr int W = (C16 + 3) / 4;
    constexpr int SLOTS = 4 * W;      // lanes per token
    constexpr int TPW = 64 / SLOTS;   // tokens per wave and load
    constexpr int U = 4;              // loads in flight per lane
    __shared__ float wsum[PACK_THREADS / 64];
    const int side = blockIdx.x / (BH * nseg);
    const int rem = blockIdx.x % (BH * nseg);
    const PackSide &S = side ? k : q;
    const int bh = rem / nseg, t0 = (rem % nseg) * PACK_STREAM_TOKENS;
    const int tend = min(N, t0 + PACK_STREAM_TOKENS);
    const int b = bh / H, h = bh % H;
    const uint16_t *xb = S.x + (int64_t)b * S.xs.b + (int64_t)h * S.xs.h;
    uint32_t *ob = S.bits + (int64_t)bh * N * W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tl = lane / SLOTS, slot = lane % SLOTS;
    const bool lane_on = tl < TPW && slot < C16;
    float asum = 0.0f;
    for (int base = t0 + wave * TPW; base < tend; base += U * 4 * TPW) {
        u4p v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tok = base + u * 4 * TPW + tl;
            v[u] = u4p{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};  // -0.0: |x| = 0; bits masked below
            if (lane_on && tok < tend)
                v[u] = *reinterpret_cast<const u4p *>(xb + (int64_t)tok * S.xs.n + 8 * slot);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tok = base + u * 4 * TPW + tl;
            const bool on = lane_on && tok < tend;
            unsigned bits = sign_bits8_abs(v[u], asum);
            bits = on ? bits : 0u;  // padding bits are 0
            const unsigned word = quad_bcast<0>(bits) | (quad_bcast<1>(bits) << 8) |
                                  (quad_bcast<2>(bits) << 16) | (quad_bcast<3>(bits) << 24);
            if ((slot & 3) == 0 && tl < TPW && tok < tend) ob[(int64_t)tok * W + (slot >> 2)] = word;
        }
    }
    const float t = block_sum<PACK_THREADS>(asum, wsum);
    if (threadIdx.x == 0) atomicAdd(S.mu + bh, t * inv_count);
}

// Short sequences: one workgroup per (tensor, head) walks all token tiles and
// stores mu itself: one launch, no atomics, no zero fill, deterministic.
// Two shapes: 256 threads and 128-token tiles for heads of fewer than 512 tokens (several
// workgroups per CU), 1024 threads and 512-token tiles from there on (one workgroup per CU,
// which then keeps up to 4.5 loads of 16 bytes per thread in flight: 13.3 -> 9.9 us at
// dit_xl2_512, 44 -> 35 us at head dimension 128 and 2048 tokens).
template <int C16, int PACK_THREADS, int PACK_TOKENS>
__global__ __launch_bounds__(PACK_THREADS) void pack_head_kernel(PackSide q, PackSide k, int BH,
                                                                 int H, int N, float inv_count) {
    constexpr int W = (C16 + 3) / 4;
    __shared__ uint32_t words[PACK_TOKENS * W];
    __shared__ float wsum[PACK_THREADS / 64];
    const int side = blockIdx.x / BH, bh = blockIdx.x % BH;
    const PackSide &S = side ? k : q;
    const int b = bh / H, h = bh % H;
    const uint16_t *xb = S.x + (int64_t)b * S.xs.b + (int64_t)h * S.xs.h;
    float a = 0.0f;
    for (int n0 = 0; n0 < N; n0 += PACK_TOKENS) {
        a += pack_tile<C16, PACK_THREADS, PACK_TOKENS>(xb, S.xs.n, n0, min(PACK_TOKENS, N - n0),
                            S.bits + ((int64_t)bh * N + n0) * W, words);
        __syncthreads();
    }
    const float t = block_sum<PACK_THREADS>(a, wsum);
    if (threadIdx.x == 0) S.mu[bh] = t * inv_count;
}

int launch_zero_f32(float *a, float *b, int n, hipStream_t stream) {
    hipLaunchKernelGGL(zero_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, a, b, n);
    return check_launch();
}

// Heads of at most this many tokens are packed by one workgroup each.
constexpr int PACK_HEAD_MAX_TOKENS = 2048;

template <int C16>
static int launch_pack_t(const PackSide &q, const PackSide &k, const Shape &s, hipStream_t stream) {
    const float inv = (float)(1.0 / ((double)s.N * (double)s.d));
    if (s.N <= PACK_HEAD_MAX_TOKENS) {
        if (s.N >= 512)
            hipLaunchKernelGGL((pack_head_kernel<C16, 1024, 512>), dim3(2u * s.BH), dim3(1024), 0, stream, q, k,
                               s.BH, s.H, s.N, inv);
        else
            hipLaunchKernelGGL((pack_head_kernel<C16, PACK_THREADS, PACK_TOKENS>), dim3(2u * s.BH),
                               dim3(PACK_THREADS), 0, stream, q, k, s.BH, s.H, s.N, inv);
        return check_launch();
    }
    int rc = launch_zero_f32(q.mu, k.mu, s.BH, stream);
    if (rc != BINATTN_OK) return rc;
    const int nseg = (s.N + PACK_STREAM_TOKENS - 1) / PACK_STREAM_TOKENS;
    hipLaunchKernelGGL(pack_stream_kernel<C16>, dim3(2u * s.BH * nseg), dim3(PACK_THREADS), 0, stream,
                       q, k, s.BH, s.H, s.N, nseg, inv);
    return check_launch();
}

int launch_pack_qk(const void *q, Strides3 qs, const void *k, Strides3 ks, const Shape &s,
                   uint32_t *q_bits, uint32_t *k_bits, float *mu_q, float *mu_k,
                   hipStream_t stream) {
    const PackSide Q = {static_cast<const uint16_t *>(q), qs, q_bits, mu_q};
    const PackSide K = {static_cast<const uint16_t *>(k), ks, k_bits, mu_k};
    switch (s.d / 8) {
#define CASE(c) case c: return launch_pack_t<c>(Q, K, s, stream);
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
}

}  // namespace binattn

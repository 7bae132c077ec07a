// phi of Alg. 1 (Eq. 5): sign bits and the abs-mean scale of Q or K.
//
// HBM-bound streaming kernel: every lane loads 16 contiguous bytes (8 bf16
// channels of one token), turns them into 8 sign bits and one partial |x| sum.
// The sign bytes of a tile of tokens are assembled in LDS and written out as
// whole uint32 words, fully coalesced.  One float atomic per workgroup feeds
// mu (pre-divided by N*d, so the buffer holds the mean when the grid drains).
#include "binattn_internal.h"

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

// bit = (x >= 0) under IEEE rules, so -0.0 -> 1 and NaN -> 0 (Sec. 3).
__device__ __forceinline__ unsigned sign_bits8(uint4 w, float &asum) {
    unsigned bits = 0;
    const unsigned dw[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float lo = __uint_as_float(dw[i] << 16);
        float hi = __uint_as_float(dw[i] & 0xffff0000u);
        bits |= (lo >= 0.0f ? 1u : 0u) << (2 * i);
        bits |= (hi >= 0.0f ? 1u : 0u) << (2 * i + 1);
        asum += fabsf(lo) + fabsf(hi);
    }
    return bits;
}

// C16 = d / 8 = 16-byte chunks per token.
template <int C16>
__global__ __launch_bounds__(PACK_THREADS) void pack_kernel(const uint16_t *__restrict__ x,
                                                            Strides3 xs, int H, int N,
                                                            int ntile,
                                                            uint32_t *__restrict__ bits,
                                                            float *__restrict__ mu,
                                                            float inv_count) {
    constexpr int W = (C16 + 3) / 4;           // words per token
    __shared__ uint32_t words[PACK_TOKENS * W];
    __shared__ float wsum[PACK_THREADS / 64];

    const int bh = blockIdx.x / ntile;
    const int b = bh / H, h = bh % H;
    const int n0 = (blockIdx.x % ntile) * PACK_TOKENS;
    const int ntok = min(PACK_TOKENS, N - n0);
    const uint16_t *xb = x + (int64_t)b * xs.b + (int64_t)h * xs.h;

    for (int i = threadIdx.x; i < PACK_TOKENS * W; i += PACK_THREADS) words[i] = 0u;
    __syncthreads();

    uint8_t *bytes = reinterpret_cast<uint8_t *>(words);
    float asum = 0.0f;
    for (int e = threadIdx.x; e < ntok * C16; e += PACK_THREADS) {
        const int tok = e / C16, c = e % C16;
        const uint4 v = *reinterpret_cast<const uint4 *>(xb + (int64_t)(n0 + tok) * xs.n + 8 * c);
        bytes[tok * (4 * W) + c] = (uint8_t)sign_bits8(v, asum);
    }
    __syncthreads();

    uint32_t *ob = bits + ((int64_t)bh * N + n0) * W;
    for (int i = threadIdx.x; i < ntok * W; i += PACK_THREADS) ob[i] = words[i];

    // workgroup reduction of the |x| partial sums
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) asum += __shfl_down(asum, off, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = asum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.0f;
        for (int i = 0; i < PACK_THREADS / 64; ++i) t += wsum[i];
        atomicAdd(mu + bh, t * inv_count);
    }
}

int launch_zero_f32(float *a, float *b, int n, hipStream_t stream) {
    hipLaunchKernelGGL(zero_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, a, b, n);
    return check_launch();
}

template <int C16>
static void launch_pack_t(const void *x, Strides3 xs, const Shape &s, uint32_t *bits, float *mu,
                          hipStream_t stream) {
    const int ntile = (s.N + PACK_TOKENS - 1) / PACK_TOKENS;
    dim3 grid((unsigned)ntile * (unsigned)s.BH);
    float inv = (float)(1.0 / ((double)s.N * (double)s.d));
    hipLaunchKernelGGL(pack_kernel<C16>, grid, dim3(PACK_THREADS), 0, stream,
                       static_cast<const uint16_t *>(x), xs, s.H, s.N, ntile, bits, mu, inv);
}

int launch_pack(const void *x, Strides3 xs, const Shape &s, uint32_t *bits, float *mu,
                hipStream_t stream) {
    switch (s.d / 8) {
#define CASE(c) case c: launch_pack_t<c>(x, xs, s, bits, mu, stream); break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
        default: return BINATTN_ERR_SHAPE;
    }
    return check_launch();
}

}  // namespace binattn

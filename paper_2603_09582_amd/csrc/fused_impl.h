// The fused loop of Alg. 1 for one (batch, head, 128-query block) per
// workgroup: QK logits on the int8 matrix cores, scale + bias (Eq. 6), online
// softmax, unsigned 8-bit P, int8 P.V with int32 accumulation, fp32 carry.
//
// One wave owns 32 query rows; a lane owns ONE query row and half of the keys
// of every block (g = lane / 32 selects keys [64 g, 64 g + 64) of the block).
// Per key block of BV = 128 keys:
//   1. four 32x32 QK tiles -> 64 integer logits per lane (registers)
//   2. S = alpha * I + b; block max (one cross-lane exchange with lane ^ 32)
//   3. p = 255 * exp(S - m) through one FMA + v_exp_f32 in base 2; row sum;
//      p rounded to a byte by v_cvt_pk_u8_f32
//   4. P.V: the int8 MFMA is signed x signed, so the operand is P - 128 and the
//      accumulator starts from 128 * (column sums of the V block), which the V
//      quantisation kernel precomputed: exact in int32
//   5. O = exp(m_old - m_new) * O + int32 block result (Alg. 1 rescale line,
//      read as a multiplication)
// Final: O / (sum of 255 * P_hat) * delta_v (Alg. 1 last line; the factor 255
// is already inside the row sum).
#pragma once

#include "attn_tiles.h"

namespace binattn {

constexpr float LOG2E_F = 1.44269504088896340736f;
constexpr float LOG2_255_F = 7.99435343685885793770f;

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ unsigned f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // keep NaN a NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <int DK, int MODE>
__global__ __launch_bounds__(FUSED_THREADS, 2) void fused_kernel(const FusedParams p) {
    using TL = Tiles<DK>;
    constexpr int DKP = 32 * DK;
    __shared__ __attribute__((aligned(16))) TL tiles[2];

    // Workgroup -> work item.  Consecutive workgroup ids go to different XCDs, so
    // the id is first turned into (xcd, slot) and work items that share a bias
    // slab (same head and row block, different batch entry) are given to one XCD
    // back to back: they then share that slab through the XCD's L2.
    const int per_xcd = (p.total_wg + 7) >> 3;
    const int u = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (u >= p.total_wg) return;
    const int b = u % p.B;
    const int rb = (u / p.B) % p.nrb;
    const int h = u / (p.B * p.nrb);
    const int bh = b * p.H + h;
    const int N = p.N, d = p.d;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, g = lane >> 5;
    const int q = rb * BR + wave * ROWS_PER_WAVE + m;  // this lane's query row
    const int qc = min(q, N - 1);                      // clamped for loads

    float alpha = p.scale;
    if (p.mu_q) alpha *= p.mu_q[bh];
    if (p.mu_k) alpha *= p.mu_k[bh];

    v4i qB[DK];
    load_q_operand<DK>(p.q_bits + ((int64_t)bh * N + qc) * DK, d, g, qB);

    const int8_t *k8h = p.k8 + (int64_t)bh * p.npad * DKP;
    const int8_t *vth = p.vt8 + (int64_t)bh * DKP * p.npad;
    const int *csh = p.cs128 + (int64_t)bh * p.nblk * DKP;

    // ---- global -> register -> LDS staging of one key/value block ----------
    u4v kreg[DK], vreg[DK];
    v4i csreg = {0, 0, 0, 0};
#define BINATTN_LOAD_BLOCK(blk)                                                                   \
    do {                                                                                          \
        load_k_regs<DK>(k8h, (blk), kreg);                                                        \
        _Pragma("unroll") for (int i_ = 0; i_ < DK; ++i_) {                                       \
            const int ch_ = threadIdx.x + FUSED_THREADS * i_;                                     \
            vreg[i_] = *reinterpret_cast<const u4v *>(vth + (int64_t)(ch_ >> 3) * p.npad +      \
                                                        (blk) * BV + 16 * (ch_ & 7));             \
        }                                                                                         \
        if (threadIdx.x < DKP / 4)                                                                \
            csreg = *reinterpret_cast<const v4i *>(csh + (int64_t)(blk) * DKP + 4 * threadIdx.x); \
    } while (0)
#define BINATTN_STORE_BLOCK(T_)                                                                   \
    do {                                                                                          \
        store_k_regs<DK>((T_), kreg);                                                             \
        _Pragma("unroll") for (int i_ = 0; i_ < DK; ++i_) {                                       \
            const int ch_ = threadIdx.x + FUSED_THREADS * i_;                                     \
            *reinterpret_cast<u4v *>((T_).vt + (ch_ >> 3) * TL::VP + 16 * (ch_ & 7)) = vreg[i_]; \
        }                                                                                         \
        if (threadIdx.x < DKP / 4) *reinterpret_cast<v4i *>((T_).cs + 4 * threadIdx.x) = csreg;  \
    } while (0)

    // ---- bias row of this lane ------------------------------------------------
    const int bsb = (MODE == BIAS_F32_VEC || MODE == BIAS_F32_ANY) ? 4 : 2;  // bytes per element
    const char *brow = nullptr;
    if (MODE != BIAS_NONE)
        brow = static_cast<const char *>(p.bias) +
               ((int64_t)b * p.bs.b + (int64_t)h * p.bs.h + (int64_t)qc * p.bs.n) * bsb;
    uint4 braw[8];  // BIAS_BF16_VEC: the 64 bias values of the current block
    auto load_bias_vec = [&](int blk) {
        const int k0 = blk * BV + 64 * g;
        const uint16_t *src = reinterpret_cast<const uint16_t *>(brow) + k0;
        if (blk * BV + BV <= N) {
#pragma unroll
            for (int i = 0; i < 8; ++i) braw[i] = *reinterpret_cast<const uint4 *>(src + 8 * i);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (k0 + 8 * i + 8 <= N) {
                    braw[i] = *reinterpret_cast<const uint4 *>(src + 8 * i);
                } else {
                    unsigned e[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) e[j] = (k0 + 8 * i + j < N) ? src[8 * i + j] : 0u;
                    braw[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16),
                                         e[4] | (e[5] << 16), e[6] | (e[7] << 16));
                }
            }
        }
    };
    // bias of tile t for this lane: keys blk*BV + 64 g + 16 t + [0, 16)
    auto bias_tile = [&](int blk, int t, float bt[16]) {
        const int k0 = blk * BV + 64 * g + 16 * t;
        if (MODE == BIAS_NONE) {
#pragma unroll
            for (int r = 0; r < 16; ++r) bt[r] = 0.0f;
        } else if (MODE == BIAS_BF16_VEC) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint4 w = braw[2 * t + i];
                const unsigned dw[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bt[8 * i + 2 * j] = bf16_lo(dw[j]);
                    bt[8 * i + 2 * j + 1] = bf16_hi(dw[j]);
                }
            }
        } else if (MODE == BIAS_BF16_ANY) {
            const uint16_t *src = reinterpret_cast<const uint16_t *>(brow) + k0;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                bt[r] = (k0 + r < N) ? __uint_as_float((unsigned)src[r] << 16) : 0.0f;
        } else if (MODE == BIAS_F32_VEC) {
            const float *src = reinterpret_cast<const float *>(brow) + k0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (k0 + 4 * i + 4 <= N) {
                    const float4 w = *reinterpret_cast<const float4 *>(src + 4 * i);
                    bt[4 * i] = w.x; bt[4 * i + 1] = w.y; bt[4 * i + 2] = w.z; bt[4 * i + 3] = w.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) bt[4 * i + j] = (k0 + 4 * i + j < N) ? src[4 * i + j] : 0.0f;
                }
            }
        } else {
            const float *src = reinterpret_cast<const float *>(brow) + k0;
#pragma unroll
            for (int r = 0; r < 16; ++r) bt[r] = (k0 + r < N) ? src[r] : 0.0f;
        }
    };

    // ---- prologue ---------------------------------------------------------------
    BINATTN_LOAD_BLOCK(0);
    if (MODE == BIAS_BF16_VEC) load_bias_vec(0);
    BINATTN_STORE_BLOCK(tiles[0]);
    __syncthreads();

    float m_run = -INFINITY;  // running row maximum (Alg. 1: m)
    float l_run = 0.0f;       // running sum of 255 * exp(S - m) over this lane's keys
    float Of[DK][16];         // fp32 carry of the output, channel 32cb + 8(r/4) + 4g + r%4
#pragma unroll
    for (int cb = 0; cb < DK; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) Of[cb][r] = 0.0f;

    for (int it = 0; it < p.nblk; ++it) {
        const bool more = it + 1 < p.nblk;
        if (more) BINATTN_LOAD_BLOCK(it + 1);
        const TL &T = tiles[it & 1];

        // 1-2. logits of the block: S = alpha * (s_i . t_j) + b_ij  (Eq. 6)
        float S[KT][16];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const v16i acc = qk_tile<DK>(T, t, m, g, qB);
            float bt[16];
            bias_tile(it, t, bt);
#pragma unroll
            for (int r = 0; r < 16; ++r) S[t][r] = fmaf((float)acc[r], alpha, bt[r]);
        }
        if (MODE == BIAS_BF16_VEC && more) load_bias_vec(it + 1);
        if (it * BV + BV > N) {  // ragged last block: keys beyond N never count
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (it * BV + 64 * g + 16 * t + r >= N) S[t][r] = -INFINITY;
        }

        // running maximum (Alg. 1: m_ij = max(m_i,j-1, rowmax S_ij))
        float mx = S[0][0];
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[t][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;  // whole row masked so far
        const float resc = __builtin_amdgcn_exp2f((m_run - m_use) * LOG2E_F);  // e^{m_old - m_new}
        const float cexp = LOG2_255_F - m_use * LOG2E_F;
        m_run = m_new;

        // 3. p = 255 * exp(S - m), its row sum, and the byte codes (Eq. 7, scale 1/255)
        float lsum = 0.0f;
        v4i pk[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                unsigned w = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(S[t][4 * i + j], LOG2E_F, cexp));
                    lsum += pe;
                    w = __builtin_amdgcn_cvt_pk_u8_f32(pe, j, w);
                }
                pk[t][i] = (int)(w ^ 0x80808080u);  // code - 128 as signed bytes
            }
        }
        l_run = fmaf(l_run, resc, lsum);

        // 4-5. O = e^{m_old - m_new} O + P~ . V~   (int8 MFMA, int32 accumulate)
#pragma unroll
        for (int cb = 0; cb < DK; ++cb) {
            v16i acc;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int4 c4 = *reinterpret_cast<const int4 *>(T.cs + 32 * cb + 8 * q4 + 4 * g);
                acc[4 * q4] = c4.x; acc[4 * q4 + 1] = c4.y; acc[4 * q4 + 2] = c4.z; acc[4 * q4 + 3] = c4.w;
            }
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const v4i a = *reinterpret_cast<const v4i *>(T.vt + (32 * cb + m) * TL::VP + 64 * g + 16 * t);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, pk[t], acc, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) Of[cb][r] = fmaf(Of[cb][r], resc, (float)acc[r]);
        }

        if (more) BINATTN_STORE_BLOCK(tiles[(it + 1) & 1]);
        __syncthreads();
    }

    // ---- epilogue: O / (255 l) * delta_v, bf16 store ----------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (q < N) {
        uint16_t *orow = p.out + (int64_t)b * p.os.b + (int64_t)h * p.os.h + (int64_t)q * p.os.n;
        const float *dl = p.delta + (int64_t)bh * DKP;
#pragma unroll
        for (int cb = 0; cb < DK; ++cb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int c = 32 * cb + 8 * q4 + 4 * g;
                if (c < d) {
                    const float4 d4 = *reinterpret_cast<const float4 *>(dl + c);
                    const unsigned y0 = f32_to_bf16_rne(Of[cb][4 * q4 + 0] * inv * d4.x);
                    const unsigned y1 = f32_to_bf16_rne(Of[cb][4 * q4 + 1] * inv * d4.y);
                    const unsigned y2 = f32_to_bf16_rne(Of[cb][4 * q4 + 2] * inv * d4.z);
                    const unsigned y3 = f32_to_bf16_rne(Of[cb][4 * q4 + 3] * inv * d4.w);
                    *reinterpret_cast<uint2 *>(orow + c) = make_uint2(y0 | (y1 << 16), y2 | (y3 << 16));
                }
            }
    }
}

#undef BINATTN_LOAD_BLOCK
#undef BINATTN_STORE_BLOCK

template <int DK>
int launch_fused_dk(const FusedParams &p, int mode, hipStream_t stream) {
    const dim3 grid((unsigned)(((p.total_wg + 7) / 8) * 8)), block(FUSED_THREADS);
    switch (mode) {
#define CASE(M) case M: hipLaunchKernelGGL((fused_kernel<DK, M>), grid, block, 0, stream, p); break;
        CASE(BIAS_NONE) CASE(BIAS_BF16_VEC) CASE(BIAS_BF16_ANY) CASE(BIAS_F32_VEC) CASE(BIAS_F32_ANY)
#undef CASE
        default: return BINATTN_ERR_DTYPE;
    }
    return check_launch();
}

}  // namespace binattn

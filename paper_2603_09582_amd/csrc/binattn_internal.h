// Internal declarations shared by the HIP translation units of libbinattn.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "binattn.h"

namespace binattn {

// Key/value block of Alg. 1 (B_v): 128 keys, i.e. four 32-key MFMA tiles.
constexpr int BV = 128;
// Query rows per workgroup (B_r of Alg. 1): 4 waves x 32 rows.
constexpr int BR = 128;
constexpr int ROWS_PER_WAVE = 32;
// Token rows reduced by one workgroup of the V absmax kernel.
constexpr int VCHUNK = 256;

struct Shape {
    int B, H, N, d;
    int BH;    // B * H
    int W;     // sign words per token = ceil(d / 32)
    int DK;    // 32-channel groups = W
    int DKP;   // padded channel count = 32 * DK
    int nblk;  // key blocks = ceil(N / BV)
    int npad;  // nblk * BV
    int nchunk;  // V absmax partials per head = ceil(N / VCHUNK)
};

inline Shape make_shape(int B, int H, int N, int d) {
    Shape s;
    s.B = B; s.H = H; s.N = N; s.d = d;
    s.BH = B * H;
    s.W = (d + 31) / 32;
    s.DK = s.W;
    s.DKP = 32 * s.DK;
    s.nblk = (N + BV - 1) / BV;
    s.npad = s.nblk * BV;
    s.nchunk = (N + VCHUNK - 1) / VCHUNK;
    return s;
}

// Operand image of one key/value block (BV keys) of one head, stored in the
// workspace exactly as the attention kernel wants it in LDS, so that a block is
// one flat asynchronous copy:
//   K  [BV positions][KP bytes]  FP4 codes of the +-1 keys (0 beyond d / beyond N),
//                                32 bytes per 64 channels, rows in MFMA order; the
//                                16-byte chunks of a row are XOR-swizzled (k_chunk)
//   VT [DKP channels][VP bytes]  V codes, channel-major, BV key bytes per row + 16 pad
//   CS [DKP] int32               PV_MAGIC + 128 * (sum of the block's V codes)
// Swizzle and padding make the 16-byte reads of 16 consecutive rows fall into 16
// different 16-byte bank groups of the 256-byte LDS row.
template <int DK>
struct Image {
    static constexpr int DK2 = (DK + 1) / 2;       // 64-channel groups of the QK contraction
    static constexpr int DKP = 32 * DK;            // padded channel count of V
    static constexpr int KP = 32 * DK2;
    static constexpr int VP = BV + 16;
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = BV * KP;
    static constexpr int CS_OFF = V_OFF + DKP * VP;
    static constexpr int BYTES = (CS_OFF + DKP * 4 + 1023) / 1024 * 1024;
};

// Where 16-byte chunk `chunk` (of KP / 16) of K row `pos` is stored inside the row.
__host__ __device__ inline int k_chunk(int pos, int chunk, int KP) {
    return KP == 32 ? (chunk ^ ((pos >> 3) & 1)) : (chunk ^ ((pos >> 2) & 3));
}

// FP4 e2m1 codes of +1.0 and -1.0
constexpr unsigned FP4_PLUS1 = 0x2u, FP4_MINUS1 = 0xAu;

// 8 sign bits -> 8 FP4 nibbles (bit i -> nibble i): +1.0 where set, -1.0 where clear.
__device__ __forceinline__ unsigned fp4_pm1_from_bits8(unsigned b) {
    unsigned x = (b | (b << 12)) & 0x000F000Fu;  // 4 bits per half word
    x = (x | (x << 6)) & 0x03030303u;            // 2 bits per byte
    x = (x | (x << 3)) & 0x11111111u;            // 1 bit per nibble, at its lowest position
    return 0xAAAAAAAAu - (x << 3);               // 0xA - 8 = 0x2 where the bit is set
}

inline int image_bytes(int DK) {
    switch (DK) {
        case 1: return Image<1>::BYTES;
        case 2: return Image<2>::BYTES;
        case 3: return Image<3>::BYTES;
        default: return Image<4>::BYTES;
    }
}

// The int32 P.V accumulator of a block starts from PV_MAGIC + 128 * colsum: read
// as fp32 bits the finished accumulator is then 1.5 * 2^23 + (block result),
// exact while |block result| < 2^22 (128 keys * 255 * 127 = 4 145 280 fits).
constexpr int PV_MAGIC_BITS = 0x4B400000;
constexpr float PV_MAGIC_F = 12582912.0f;

// Private workspace layout (all offsets 256-byte aligned).
//   img   bytes [BH][nblk][Image<DK>::BYTES]
//   delta f32   [BH][DKP]
//   amax  f32   [BH][nblk][DKP]             partial absmax of V (per 256 tokens, or per key
//                                           block on the path that takes Q, K, V themselves)
// and, for that path:
//   mu    f32   [2][BH]                     abs-means of Q and K
//   psum  f32   [BH][nblk][2]               their partial sums per key block
//   qbits u32   [BH][N][W]                  query sign words
struct Workspace {
    size_t img, delta, amax, mu, psum, qbits, total;
    int img_bytes;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline Workspace make_workspace(const Shape &s) {
    Workspace w;
    w.img_bytes = image_bytes(s.DK);
    size_t off = 0;
    w.img = off;   off = align256(off + (size_t)s.BH * s.nblk * w.img_bytes);
    w.delta = off; off = align256(off + (size_t)s.BH * s.DKP * 4);
    w.amax = off;  off = align256(off + (size_t)s.BH * s.nblk * s.DKP * 4);
    w.mu = off;    off = align256(off + (size_t)2 * s.BH * 4);
    w.psum = off;  off = align256(off + (size_t)s.BH * s.nblk * 2 * 4);
    w.qbits = off; off = align256(off + (size_t)s.BH * s.N * s.W * 4);
    w.total = off;
    return w;
}

struct Strides3 {
    int64_t b, h, n;
};

// Launchers (each returns BINATTN_OK or BINATTN_ERR_LAUNCH).
int launch_pack_qk(const void *q, Strides3 qs, const void *k, Strides3 ks, const Shape &s,
                   uint32_t *q_bits, uint32_t *k_bits, float *mu_q, float *mu_k,
                   hipStream_t stream);
int launch_expand_k(const uint32_t *k_bits, const Shape &s, char *ws, const Workspace &w,
                    hipStream_t stream);
int launch_prepare(const void *v, Strides3 vs, const uint32_t *k_bits, const Shape &s, char *ws,
                   const Workspace &w, hipStream_t stream);
int launch_phi_psi(const void *q, Strides3 qs, const void *k, Strides3 ks, const void *v, Strides3 vs,
                   const Shape &s, char *ws, const Workspace &w, float *mu_q_out, float *mu_k_out,
                   hipStream_t stream);
int launch_export_vq(const Shape &s, const char *ws, const Workspace &w, int8_t *vq, float *delta,
                     hipStream_t stream);
int launch_logits_popcount(const uint32_t *q_bits, const uint32_t *k_bits, const Shape &s,
                           int row_begin, int row_end, int32_t *logits, bool rowsum, hipStream_t stream);
int launch_logits_fp4(const uint32_t *q_bits, const char *ws, const Workspace &w, const Shape &s,
                      int row_begin, int row_end, int32_t *logits, bool rowsum, hipStream_t stream);
int launch_logits_i8(const uint32_t *q_bits, const uint32_t *k_bits, const Shape &s, int row_begin,
                     int row_end, int32_t *logits, bool rowsum, hipStream_t stream);

int launch_probe_valu(int op, int iters, int blocks, float *out, hipStream_t stream);

enum BiasMode {
    BIAS_NONE = 0,
    BIAS_BF16_VEC = 1,  // any element-aligned rows: 16-byte loads into registers, one block ahead
    BIAS_F32_VEC = 3,   // fp32 bias, 16-byte loads at use
    BIAS_BF16_LDS = 5,  // rows 16-byte aligned, N % 8 == 0: tile staged global -> LDS asynchronously
    BIAS_AXIAL = 7,     // b_ij = y[iy - jy] + x[ix - jx] on a Gy x Gx token grid, tables held in LDS
    BIAS_TABLE = 9,     // b_ij = t[iy - jy][ix - jx]: the full relative-position table of the head in LDS
    BIAS_TABLE_BLK = 13, // the same table for larger grids: only the rows a key block needs, staged per block
    BIAS_LUT = 11       // no bias: 255 exp(S - m) read from a per-head table indexed by (m - I) / 2
};

// largest grid side of BIAS_AXIAL (the tables of one head live in LDS)
constexpr int AXIAL_MAX_G = 256;
// largest grid side of BIAS_TABLE ((2 G - 1)^2 entries per head held in LDS); larger grids
// (up to AXIAL_MAX_G) take BIAS_TABLE_BLK
constexpr int TABLE_MAX_G = 32;

struct FusedParams {
    const uint32_t *q_bits;
    const float *mu_q, *mu_k;  // may be null (taken as 1)
    const void *bias;          // may be null
    Strides3 bs;               // bias element strides (batch, head, row)
    float scale;
    uint16_t *out;
    Strides3 os;
    const char *img;     // block images
    const float *delta;
    int B, H, N, d, nblk, nrb, total_wg;
    int nb;              // batch entries per workgroup (1 or 2)
    int wide;            // 0; 1 / 3: single-launch forms (8 / 4 waves); 2: 8-wave workgroups over row-block pairs (nrb counts pairs)
    // single-launch short-sequence kernel: the bf16 inputs, whether mu is applied, optional mu exports
    const uint16_t *xq, *xk, *xv;
    Strides3 xqs, xks, xvs;
    int use_mu;
    float *mu_q_out, *mu_k_out;
    const float *ax_y, *ax_x;  // BIAS_AXIAL: fp32 [H][2 Gy - 1], [H][2 Gx - 1]
    const float *table;        // BIAS_TABLE: fp32 [H][2 Gy - 1][2 Gx - 1]
    int Gy, Gx, gx_shift;      // BIAS_AXIAL / BIAS_TABLE: token grid, Gx = 1 << gx_shift
};

// Defined (and explicitly instantiated) in fused_dk<DK>.hip, DK = ceil(d / 32).
template <int DK>
int launch_fused_dk(const FusedParams &p, int mode, hipStream_t stream);
// The single-launch form for at most two key blocks (nb must be 2, total_wg = B * H).
// single-launch form: calls with more heads than this use 4-wave workgroups (two per compute unit)
constexpr int ONEHEAD4_MIN_HEADS = 256;
// ... in the variants whose 256-thread prologue holds a head's loads in registers without spilling
constexpr bool onehead4_built(int DK, int mode) {
    return DK <= 2 || (DK == 3 && (mode == BIAS_NONE || mode == BIAS_F32_VEC || mode == BIAS_BF16_LDS || mode == BIAS_AXIAL));
}

template <int DK>
int launch_onehead_dk(const FusedParams &p, int mode, hipStream_t stream);

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? BINATTN_OK : BINATTN_ERR_LAUNCH;
}

}  // namespace binattn

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

// Private workspace layout (all offsets 256-byte aligned).
//   k8    int8  [BH][nblk][BV rows in MFMA order][DKP]   +-1 keys, 0 in padding
//   vt8   int8  [BH][DKP][npad]                          V codes, channel-major
//   cs128 int32 [BH][nblk][DKP]                          128 * column sums of a key block
//   delta f32   [BH][DKP]
//   amax  f32   [BH][nchunk][DKP]                        partial absmax of V
struct Workspace {
    size_t k8, vt8, cs128, delta, amax, total;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline Workspace make_workspace(const Shape &s) {
    Workspace w;
    size_t off = 0;
    w.k8 = off;    off = align256(off + (size_t)s.BH * s.npad * s.DKP);
    w.vt8 = off;   off = align256(off + (size_t)s.BH * s.DKP * s.npad);
    w.cs128 = off; off = align256(off + (size_t)s.BH * s.nblk * s.DKP * 4);
    w.delta = off; off = align256(off + (size_t)s.BH * s.DKP * 4);
    w.amax = off;  off = align256(off + (size_t)s.BH * s.nchunk * s.DKP * 4);
    w.total = off;
    return w;
}

struct Strides3 {
    int64_t b, h, n;
};

// Launchers (each returns BINATTN_OK or BINATTN_ERR_LAUNCH).
int launch_pack(const void *x, Strides3 xs, const Shape &s, uint32_t *bits, float *mu,
                hipStream_t stream);
int launch_zero_f32(float *a, float *b, int n, hipStream_t stream);
int launch_expand_k(const uint32_t *k_bits, const Shape &s, int8_t *k8, hipStream_t stream);
int launch_quant_v(const void *v, Strides3 vs, const Shape &s, char *ws, const Workspace &w,
                   hipStream_t stream);
int launch_export_vq(const Shape &s, const char *ws, const Workspace &w, int8_t *vq, float *delta,
                     hipStream_t stream);
int launch_logits_popcount(const uint32_t *q_bits, const uint32_t *k_bits, const Shape &s,
                           int row_begin, int row_end, int32_t *logits, hipStream_t stream);
int launch_logits_mfma(const uint32_t *q_bits, const int8_t *k8, const Shape &s, int row_begin,
                       int row_end, int32_t *logits, hipStream_t stream);

enum BiasMode {
    BIAS_NONE = 0,
    BIAS_BF16_VEC = 1,  // rows 16-byte aligned: 16-byte loads, prefetched one block ahead
    BIAS_BF16_ANY = 2,  // any alignment: element loads
    BIAS_F32_VEC = 3,
    BIAS_F32_ANY = 4
};

struct FusedParams {
    const uint32_t *q_bits;
    const float *mu_q, *mu_k;  // may be null (taken as 1)
    const void *bias;          // may be null
    Strides3 bs;               // bias element strides (batch, head, row)
    float scale;
    uint16_t *out;
    Strides3 os;
    const int8_t *k8;
    const int8_t *vt8;
    const int *cs128;
    const float *delta;
    int B, H, N, d, nblk, npad, nrb, total_wg;
};

// Defined (and explicitly instantiated) in fused_dk<DK>.hip, DK = ceil(d / 32).
template <int DK>
int launch_fused_dk(const FusedParams &p, int mode, hipStream_t stream);

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? BINATTN_OK : BINATTN_ERR_LAUNCH;
}

}  // namespace binattn

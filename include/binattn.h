/*
 * binattn -- BinaryAttention forward for AMD MI355X (gfx950), C ABI.
 *
 * The library computes one attention layer the way the paper's Alg. 1 does:
 *   phi:  Q, K -> sign bits + scales mu_q, mu_k              (Eq. 5)
 *   psi:  V    -> signed 8-bit codes + per-channel delta_v   (Eq. 7)
 *   S_ij  = scale * mu_q * mu_k * (s_i . t_j) + b_ij         (Eq. 6)
 *   online softmax over key blocks, P quantised to unsigned 8 bits with
 *   scale 1/255 relative to the running row maximum, integer P~.V~ with
 *   32-bit accumulation, O = O / (255 l) * delta_v           (Alg. 1)
 * with (B, H) independent problems of N tokens and head dimension d.
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers owned by the caller (the library
 *    never allocates, frees or synchronises); `stream` is a hipStream_t passed
 *    as void* (NULL = the default stream).  Work is enqueued asynchronously.
 *  - Stride arrays hold ELEMENT strides for the (batch, head, row) axes; the
 *    innermost (channel / column) stride is always 1.
 *  - Return value 0 on success, a negative BINATTN_ERR_* otherwise.  All
 *    arguments are validated before anything is launched, so a failing call
 *    leaves every output untouched.  Inputs are never modified.
 *  - Supported shapes: B, H, N >= 1 with B*H < 2^31 / 128 and N <= 2^24;
 *    d a multiple of 8 with 8 <= d <= 128.  Accuracy does not degrade with N: the
 *    running output of Alg. 1 is carried in fp32 and rounded by at most 4 units of
 *    the integer P~.V~ scale per 128-key block (against a final divisor of at
 *    least 255), whatever the number of blocks.
 *  - Q, K, V and the output are bf16; their base pointers must be 16-byte
 *    aligned and every stride a multiple of 8 elements.
 *  - Calls on one stream are ordered; the entry points keep no global mutable
 *    state, so calls on different streams with disjoint buffers are
 *    independent.
 */
#ifndef BINATTN_H
#define BINATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    BINATTN_OK = 0,
    BINATTN_ERR_NULL = -1,      /* a required pointer is NULL                      */
    BINATTN_ERR_SHAPE = -2,     /* B, H, N or d outside the supported range        */
    BINATTN_ERR_STRIDE = -3,    /* a stride is negative, too small or misaligned   */
    BINATTN_ERR_ALIGN = -4,     /* a base pointer is not aligned as required       */
    BINATTN_ERR_WORKSPACE = -5, /* workspace missing, misaligned or too small      */
    BINATTN_ERR_DTYPE = -6,     /* unknown bias dtype                              */
    BINATTN_ERR_LAUNCH = -7,    /* the HIP runtime refused a launch                */
    BINATTN_ERR_VARIANT = -8,   /* unknown logits variant                          */
    BINATTN_ERR_RANGE = -9,     /* row range outside [0, N]                        */
    BINATTN_ERR_TOO_LARGE = -10, /* shape needs more than the static scratch holds (binattn_forward_static) */
    BINATTN_ERR_DEVICE = -11    /* current device / static buffer could not be resolved */
};

enum { BINATTN_BIAS_BF16 = 1, BINATTN_BIAS_F32 = 2 };

/* flags of binattn_forward */
enum {
    BINATTN_FLAG_NO_MU = 1,   /* ignore mu_q, mu_k (ablation row "no scale", Tab. 5) */
    BINATTN_FLAG_NO_BIAS = 2, /* ignore bias (ablation rows without bias, Tab. 5)    */
    BINATTN_FLAG_LUT = 4,     /* bias-free calls only: read 255 exp(S - m) from a per-head table
                                 of its d + 1 possible values instead of computing every
                                 exponential.  Same results up to the rounding of one fp32
                                 exponential; measured slower than the exponentials on MI355X
                                 (the table read costs more than the FMA + v_exp_f32 it
                                 replaces), so it is opt-in and kept for comparison         */
    BINATTN_FLAG_WIDE8 = 8,   /* single-launch forms only: one 8-wave workgroup per head even
                                 when the call has more heads than the chip has compute units
                                 (by default such calls use 4-wave workgroups, two per compute
                                 unit).  Same results; kept for comparison                    */
};

/* variants of binattn_logits_debug */
enum {
    BINATTN_LOGITS_POPCOUNT = 0, /* d - 2*popcount(q XOR k) on the vector ALU (Sec. 4.1)   */
    BINATTN_LOGITS_MFMA_I8 = 1,  /* +-1 int8 contraction on the matrix cores                */
    BINATTN_LOGITS_MFMA_FP4 = 2, /* +-1.0 FP4 contraction, fp32 accumulate (exact); the form
                                    the fused kernel uses                                   */
    BINATTN_LOGITS_ROWSUM = 0x100 /* OR-ed to a variant: write sum_j I_ij per query row, int32
                                    [B, H, row_end - row_begin], instead of the matrix (no
                                    4-byte-per-pair store stream: the form for timing)      */
};

int binattn_version(void);
const char *binattn_strerror(int code);

/*
 * phi of Alg. 1 / Eq. 5 for Q and K in one launch sequence.
 *   q, k      : bf16 [B, H, N, d] with element strides q_strides / k_strides.
 *   q_bits,
 *   k_bits    : out, uint32 [B, H, N, W] contiguous, W = ceil(d / 32).  Bit
 *               (c & 31) of word (c >> 5) is 1 iff x[c] >= 0 under IEEE
 *               comparison (+0 and -0 give 1, NaN gives 0); unused bits are 0.
 *   mu_q, mu_k: out, float32 [B, H]: mean of |x| over the N*d elements of the
 *               head (Eq. 5 text).  For N > 2048 the sum goes through float
 *               atomics, so the last bits may differ between runs.
 */
int binattn_pack_qk(const void *q, const void *k, int B, int H, int N, int d,
                    const int64_t q_strides[3], const int64_t k_strides[3],
                    uint32_t *q_bits, uint32_t *k_bits, float *mu_q, float *mu_k,
                    void *stream);

/* Bytes of scratch binattn_prepare_kv / binattn_attend / binattn_forward (and the
 * debug entry points) need for this shape
 * (0 if the shape is unsupported).  The workspace must be 256-byte aligned; its
 * contents are private to the library and overwritten by every call. */
size_t binattn_workspace_bytes(int B, int H, int N, int d);

/*
 * psi of Alg. 1 (Eq. 7) plus the operand set-up of the key side: quantises V
 * to signed 8-bit codes with per-channel delta_v and lays the +-1 keys and the
 * codes out in `workspace` the way the attention kernel reads them.
 *   k_bits : as written by binattn_pack_qk.
 *   v      : bf16 [B, H, N, d], strides v_strides.  Must be finite.
 */
int binattn_prepare_kv(const uint32_t *k_bits, const void *v, const int64_t v_strides[3], int B,
                       int H, int N, int d, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The fused loop of Alg. 1 (logits of Eq. 6, online softmax, 8-bit P, integer
 * P~.V~, final rescale) over a workspace filled by binattn_prepare_kv for the
 * SAME (B, H, N, d).
 *   q_bits     : as written by binattn_pack_qk.
 *   mu_q, mu_k : float32 [B, H]; either may be NULL (taken as 1).
 *   bias       : [.., N, N] of bias_dtype, element strides bias_strides for
 *                (batch, head, row); a batch stride of 0 shares one bias over
 *                the batch.  May be NULL (no bias).  Rows need only element
 *                alignment; the fastest path (tiles staged through LDS) needs
 *                bf16, a 16-byte aligned base, strides that keep every row
 *                16-byte aligned, and either N a multiple of 8 or a row stride of
 *                at least N rounded up to a multiple of 8 (e.g. N = 197 in rows
 *                of 200 elements: the padding elements of every row, the last
 *                one included, are then read - they must be inside the
 *                allocation - and ignored); and N > 128 if d > 96.
 *   scale      : multiplies the +-1 inner product (1/sqrt(d) in Eq. 6); the
 *                effective multiplier is scale * mu_q[b,h] * mu_k[b,h].
 *   out        : bf16 [B, H, N, d], strides out_strides, rounded to nearest even
 *                from fp32.
 *   flags      : BINATTN_FLAG_*.
 */
int binattn_attend(const uint32_t *q_bits, const float *mu_q, const float *mu_k, const void *bias,
                   int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                   int d, void *out, const int64_t out_strides[3], const void *workspace,
                   size_t workspace_bytes, unsigned flags, void *stream);

/*
 * binattn_attend with a DECOMPOSED relative-position bias generated inside the kernel
 * instead of a dense [N, N] matrix.  Sec. 4.2 allows the bias of Eq. 6 to depend on position
 * only, and the memory study of the ablations (Sec. 5.6) points to a bias that splits into a
 * sum over the spatial directions as the way to avoid the dense matrix's footprint.  Tokens
 * form a Gy x Gx grid in row-major order, n = iy * Gx + ix, with Gy * Gx = N, and
 *     b_ij = bias_y[h][iy - jy + Gy - 1] + bias_x[h][ix - jx + Gx - 1].
 *   bias_y : float32 [H, 2 Gy - 1] contiguous, shared over the batch.
 *   bias_x : float32 [H, 2 Gx - 1] contiguous.
 *   Gx     : a power of two in [16, 256];  Gy in [1, 256]  (BINATTN_ERR_SHAPE otherwise).
 * Everything else as binattn_attend; BINATTN_FLAG_NO_BIAS ignores the tables.
 */
int binattn_attend_axial(const uint32_t *q_bits, const float *mu_q, const float *mu_k,
                         const float *bias_y, const float *bias_x, int Gy, int Gx, float scale, int B,
                         int H, int N, int d, void *out, const int64_t out_strides[3],
                         const void *workspace, size_t workspace_bytes, unsigned flags, void *stream);

/*
 * binattn_attend with the full learnable relative-position table as bias (the bias the
 * ablations of Sec. 5.6 train), generated inside the kernel: tokens form a Gy x Gx grid in
 * row-major order, n = iy * Gx + ix, with Gy * Gx = N, and
 *     b_ij = table[h][iy - jy + Gy - 1][ix - jx + Gx - 1].
 *   table : float32 [H, 2 Gy - 1, 2 Gx - 1] contiguous, shared over the batch, finite values.
 *   Gx    : a power of two in [16, 256];  Gy in [1, 256]  (BINATTN_ERR_SHAPE otherwise).
 *           Up to 32 x 32 the head's whole table is held in LDS; larger grids stage, per key
 *           block, only the table rows that block touches.
 * Everything else as binattn_attend; BINATTN_FLAG_NO_BIAS ignores the table.
 */
int binattn_attend_relpos(const uint32_t *q_bits, const float *mu_q, const float *mu_k,
                          const float *table, int Gy, int Gx, float scale, int B, int H, int N, int d,
                          void *out, const int64_t out_strides[3], const void *workspace,
                          size_t workspace_bytes, unsigned flags, void *stream);

/*
 * binattn_prepare_kv followed by binattn_attend (all of Alg. 1 after phi);
 * arguments as above.
 */
int binattn_forward(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                    const float *mu_k, const void *v, const int64_t v_strides[3],
                    const void *bias, int bias_dtype, const int64_t bias_strides[3],
                    float scale, int B, int H, int N, int d, void *out,
                    const int64_t out_strides[3], void *workspace, size_t workspace_bytes,
                    unsigned flags, void *stream);

/*
 * binattn_forward for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as binattn_forward, without the workspace: the operand images,
 * delta_v and the V absmax partials live in a buffer of BINATTN_STATIC_SCRATCH_BYTES that is
 * part of the library's device code (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing.
 *  - A shape with binattn_workspace_bytes(B, H, N, d) > BINATTN_STATIC_SCRATCH_BYTES returns
 *    BINATTN_ERR_TOO_LARGE and launches nothing (the five benchmark workloads fit).
 *  - Every call on a GPU uses that GPU's one buffer and overwrites all of it that it reads, so
 *    nothing needs clearing between calls; calls that overlap in time on one GPU (different
 *    streams, or several host threads) race on it and must be ordered by the caller.
 *  - The first call on a device looks the buffer's address up (no allocation, but a runtime
 *    query): make it outside a stream capture.
 */
#define BINATTN_STATIC_SCRATCH_BYTES (64u << 20)
int binattn_forward_static(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                           const float *mu_k, const void *v, const int64_t v_strides[3], const void *bias,
                           int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                           int d, void *out, const int64_t out_strides[3], unsigned flags, void *stream);

/* binattn_prepare_kv followed by binattn_attend_axial. */
int binattn_forward_axial(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                          const float *mu_k, const void *v, const int64_t v_strides[3],
                          const float *bias_y, const float *bias_x, int Gy, int Gx, float scale, int B,
                          int H, int N, int d, void *out, const int64_t out_strides[3], void *workspace,
                          size_t workspace_bytes, unsigned flags, void *stream);

/* binattn_prepare_kv followed by binattn_attend_relpos. */
int binattn_forward_relpos(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                           const float *mu_k, const void *v, const int64_t v_strides[3],
                           const float *table, int Gy, int Gx, float scale, int B, int H, int N, int d,
                           void *out, const int64_t out_strides[3], void *workspace,
                           size_t workspace_bytes, unsigned flags, void *stream);

/*
 * All of Alg. 1 in ONE launch for short sequences (N <= 256): phi (Eq. 5: sign bits and
 * abs-means of Q and K), psi (Eq. 7: V codes and delta_v) and the fused loop, one workgroup
 * per (batch, head) with every intermediate kept on chip.  This is the form for the low
 * resolutions where Sec. 5.1 finds the separate quantisation passes to cost as much as the
 * attention itself.  No workspace.
 *   q, k, v    : bf16 [B, H, N, d] with element strides q_strides / k_strides / v_strides.
 *   bias, bias_dtype, bias_strides, scale, out, out_strides, flags : as binattn_attend.
 *   mu_q_out,
 *   mu_k_out   : optional (may be NULL) float32 [B, H]: the abs-means that were used.
 * Results equal binattn_pack_qk + binattn_forward up to the summation order of the
 * abs-means.  N > 256 returns BINATTN_ERR_SHAPE.  A call with more than 256 (batch, head)
 * pairs runs 4-wave workgroups, two per compute unit, each taking a head's two 128-row
 * blocks in turn (BINATTN_FLAG_WIDE8 keeps one 8-wave workgroup per head; same results up
 * to the summation order of the abs-means).
 */
int binattn_forward_fused(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                          const int64_t k_strides[3], const int64_t v_strides[3], const void *bias,
                          int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                          int d, void *out, const int64_t out_strides[3], float *mu_q_out,
                          float *mu_k_out, unsigned flags, void *stream);

/*
 * The whole of Alg. 1 from the bf16 tensors, for any N: phi (Eq. 5), psi (Eq. 7) and the fused
 * loop behind one call.  N <= 256 is binattn_forward_fused (one launch, workspace unused and
 * may be NULL).  Longer sequences take three launches: one pass over Q, K, V that packs the
 * query signs, writes the keys' +-1 operand rows directly (no key sign words in memory),
 * and reduces the V absmax and the |q|, |k| sums per 256 tokens; the V quantisation, which
 * also adds those partial sums in a fixed order (the abs-means are the same bits on every
 * run, unlike binattn_pack_qk's atomics for N > 2048); and binattn_attend.
 *   arguments as binattn_forward_fused, plus the workspace of binattn_workspace_bytes.
 */
int binattn_attention(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                      const int64_t k_strides[3], const int64_t v_strides[3], const void *bias, int bias_dtype,
                      const int64_t bias_strides[3], float scale, int B, int H, int N, int d, void *out,
                      const int64_t out_strides[3], float *mu_q_out, float *mu_k_out, void *workspace,
                      size_t workspace_bytes, unsigned flags, void *stream);

/*
 * binattn_forward_fused with the relative-position table of binattn_attend_relpos as bias
 * (table, Gy, Gx as there, with Gx <= 32 and Gy <= 32; Gy * Gx = N <= 256): for a 16 x 16 token grid the whole layer is
 * one launch and no [N, N] bias exists anywhere.
 */
int binattn_forward_fused_relpos(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                                 const int64_t k_strides[3], const int64_t v_strides[3], const float *table,
                                 int Gy, int Gx, float scale, int B, int H, int N, int d, void *out,
                                 const int64_t out_strides[3], float *mu_q_out, float *mu_k_out,
                                 unsigned flags, void *stream);

/*
 * binattn_attention with the relative-position table of binattn_attend_relpos as bias (the
 * bias trained in Sec. 5.6), for any N = Gy * Gx within that call's grid limits: one launch
 * where binattn_forward_fused_relpos applies, else the three launches of binattn_attention.
 * No [N, N] bias exists anywhere.  Arguments as binattn_forward_fused_relpos plus the
 * workspace of binattn_workspace_bytes (unused and may be NULL in the one-launch case).
 */
int binattn_attention_relpos(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                             const int64_t k_strides[3], const int64_t v_strides[3], const float *table, int Gy,
                             int Gx, float scale, int B, int H, int N, int d, void *out,
                             const int64_t out_strides[3], float *mu_q_out, float *mu_k_out, void *workspace,
                             size_t workspace_bytes, unsigned flags, void *stream);

/*
 * Integer logits I_ij = s_i . t_j of Sec. 4.1 for query rows
 * [row_begin, row_end) of every head: int32 [B, H, row_end - row_begin, N]
 * contiguous.  BINATTN_LOGITS_MFMA_FP4 runs the same tile routine as the fused
 * kernel and needs the workspace of binattn_workspace_bytes (it overwrites the
 * key part); the other variants ignore the workspace arguments.
 */
int binattn_logits_debug(const uint32_t *q_bits, const uint32_t *k_bits, int B, int H, int N,
                         int d, int row_begin, int row_end, int32_t *logits, int variant,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * psi alone (Eq. 7), exported in canonical layout for checking:
 *   vq    : out, int8 [B, H, N, d] contiguous, code = rne(v / delta) in [-127, 127]
 *   delta : out, float32 [B, H, d], delta = absmax over tokens / 127 (1 if the
 *           channel is all zero); both divisions are IEEE fp32.
 * Runs the same quantisation kernels as binattn_forward into `workspace` and
 * then copies the codes out of the library's internal layout.
 */
int binattn_quant_v_debug(const void *v, const int64_t v_strides[3], int B, int H, int N, int d,
                          int8_t *vq, float *delta, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * Measurement aid, not part of the attention path: runs `blocks` workgroups of 256 lanes,
 * each lane issuing 8 * iters vector-ALU instructions in eight independent chains, and writes
 * one float per lane to `out` (blocks * 256 floats).  op = A | (B << 8) with A, B from
 * BINATTN_PROBE_*: even chains issue kind A, odd chains kind B (B = A: one kind; B may
 * otherwise be FMA, CVT_PK_U8, EXP2 or OR).  Timing the launch gives the chip's issue rate
 * for that instruction or mix: the roofline of the fused kernel counts vector-ALU issue
 * slots per (query, key) pair, and this is how the slots of v_exp_f32 (two) and of the others
 * (one) were measured, and which kinds issue side by side.  iters, blocks >= 1.
 */
enum {
    BINATTN_PROBE_FMA = 0, BINATTN_PROBE_EXP2 = 1, BINATTN_PROBE_ADD = 2, BINATTN_PROBE_MAX3 = 3,
    BINATTN_PROBE_CVT_PK_U8 = 4, BINATTN_PROBE_CVT_F32_I32 = 5, BINATTN_PROBE_OR = 6, BINATTN_PROBE_MUL = 7,
    BINATTN_PROBE_LSHL = 8, BINATTN_PROBE_AND = 9, BINATTN_PROBE_XOR = 10, BINATTN_PROBE_MIN3_I32 = 11,
    BINATTN_PROBE_LSHL_ADD = 12, BINATTN_PROBE_MOV = 13, BINATTN_PROBE_ADD_U32 = 14, BINATTN_PROBE_PERM = 15,
    /* the softmax's own per-pair instruction mix on register data, 16 values per lane and step
       (then iters counts steps); op = BINATTN_PROBE_SOFTMAX | (KiB of LDS per workgroup << 8)
       pins the number of workgroups (of four waves) a compute unit can hold */
    BINATTN_PROBE_SOFTMAX = 64
};
int binattn_probe_valu(int op, int iters, int blocks, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BINATTN_H */

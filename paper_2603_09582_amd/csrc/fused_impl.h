// The fused loop of Alg. 1 for one (batch, head, 128-query block) per
// workgroup: QK logits on the matrix cores, scale + bias (Eq. 6), online
// softmax, unsigned 8-bit P, int8 P.V with int32 accumulation, fp32 carry.
//
// One wave owns 32 query rows; a lane owns ONE query row and half of the keys
// of every block (g = lane / 32 selects keys [64 g, 64 g + 64) of the block).
// The vector ALU is the binding unit of this kernel, so the design removes
// vector instructions wherever another unit can do the work.  Per key block of
// BV = 128 keys:
//   0. the next block's operand image is copied global -> LDS asynchronously
//      (no staging registers, no LDS store instructions)
//   1. T = I + b / alpha: the bias is unpacked, divided by the logit multiplier
//      alpha = scale * mu_q * mu_k and handed to the FP4 MFMA as its accumulator
//      input; the MFMA adds the exact integer logit I = s_i . t_j in fp32.
//      (S of Eq. 6 is alpha * T; alpha > 0 after folding its sign into the Q
//      operand, so maxima can be taken on T.)
//   2. block max of T (one cross-lane exchange with lane ^ 32), running max m
//   3. p = 255 * exp(S - m) = exp2(T * alpha*log2(e) + c) with one FMA and one
//      v_exp_f32; row sum in fp32; p rounded to a byte by v_cvt_pk_u8_f32
//      (Eq. 7, scale 1/255, relative to the running maximum as in Alg. 1)
//   4. P.V: the int8 MFMA is signed x signed, so the operand is P - 128 and the
//      accumulator starts from 128 * (column sums of the V block), precomputed
//      by the V quantisation kernel: exact in int32.  The seed also carries the
//      bit pattern of 1.5 * 2^23, so the finished int32 accumulator, read as
//      fp32 bits, IS the float 1.5 * 2^23 + result: no int->float conversion.
//   5. O = exp(m_old - m_new) * O + block result (Alg. 1's rescale line, read as
//      a multiplication) is one FMA per output register; the 1.5 * 2^23 offsets
//      accumulate as 1.5 * 2^23 * rho with rho = sum of the rescale products,
//      tracked per row and subtracted every eighth block and at the end.
// Final: (O - 1.5*2^23*rho) / (sum of 255 * P_hat) * delta_v (Alg. 1 last line;
// the factor 255 is already inside the row sum).
#pragma once

#include "attn_tiles.h"
#include "quant_v.h"

namespace binattn {

// 16-byte loads from addresses that are only element-aligned (gfx950 under HSA
// supports unaligned vector loads; the compiler still emits one dwordx4 load).
typedef u4v u4v_a2 __attribute__((aligned(2)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef f4v f4v_a4 __attribute__((aligned(4)));

constexpr float LOG2E_F = 1.44269504088896340736f;
constexpr float LOG2_255_F = 7.99435343685885793770f;

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

// two fp32 -> two bf16 in one dword, round to nearest even (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    const f2v v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// NB = batch entries per workgroup.  NB = 2 (only with BIAS_BF16_LDS and a bias shared
// over the batch) puts two batch entries of the same (head, row block) into one
// 8-wave workgroup: waves 0-3 work on entry 2 bp, waves 4-7 on entry 2 bp + 1, and
// both read the SAME bias tile from LDS, so the bias - the dominant HBM stream of
// long sequences - is fetched once per pair and can be double-buffered.
//
// With NB = 1 the grid is persistent: a workgroup walks work items v, v + G, v + 2G, ...
// (G = grid size) and treats all their key blocks as ONE stream, so the asynchronous
// copies for the first block of the next item are already in flight during the last
// block of the current one; only the very first block of a workgroup waits for memory.
// That pays for short sequences (few blocks per item).  NB = 2 is only used for long
// sequences, where the item switch is rare and its bookkeeping at the start of every
// block (all waves of a workgroup pass it together, right after the barrier, so it is
// not hidden behind another wave's arithmetic) costs more than it saves: there a
// workgroup computes one item.
//
// ONEHEAD (8 waves) is the single-launch form for at most two key blocks: one workgroup
// owns a whole (batch, head).  It reads the bf16 Q, K, V itself, makes the sign bits, both
// abs-means, the V codes and both operand images directly in LDS (phi and psi of Alg. 1
// fused into their consumer), then runs the same block loop on its two 128-row blocks
// (waves 0-3 / 4-7).  Nothing but the bias and the inputs is read from memory and only the
// output is written.
//
// WIDE_ROWS2 (8 waves) serves head dimensions whose operand images leave no LDS room for two
// 4-wave workgroups with bias tiles (d > 96): the two halves of the workgroup are the row
// blocks 2 rp, 2 rp + 1 of ONE (batch, head); they share the operand images (one copy stream
// for 256 rows) and keep private bias tiles; the grid is persistent as with NB = 1.
//
// ONEHEAD4 (4 waves) is the single-launch form for launches with more heads than compute units:
// the same prologue with 256 threads, then the head's two 128-row blocks one after the other
// as two items of the persistent stream (the images stay where they are).  Two such workgroups
// share a compute unit, so one head's loads and preparation overlap the other's block loop.
enum { WIDE_NONE = 0, WIDE_ONEHEAD = 1, WIDE_ROWS2 = 2, WIDE_ONEHEAD4 = 3 };
template <int DK, int MODE, int NB, int WIDE = WIDE_NONE>
__global__ __launch_bounds__(FUSED_THREADS * NB, 2) void fused_kernel(const FusedParams p) {
    using L = Image<DK>;
    constexpr bool ONEHEAD4 = WIDE == WIDE_ONEHEAD4;
    constexpr bool ONEHEAD = WIDE == WIDE_ONEHEAD || ONEHEAD4, ROWS2 = WIDE == WIDE_ROWS2;
    static_assert(WIDE == WIDE_NONE || ONEHEAD4 || NB == 2, "the wide forms use 8 waves");
    static_assert(!ONEHEAD4 || NB == 1, "the 4-wave single-launch form");
    constexpr bool PAIR = NB == 2 && WIDE == WIDE_NONE;  // two batch entries sharing bias tiles
    constexpr int NWI = ROWS2 ? 8 : 4;                   // waves that copy one operand image
    constexpr int NIMG = PAIR ? 2 : 1;          // operand images per buffer
    constexpr bool PERSIST = NB == 1 || ROWS2;
    constexpr int DKP = 32 * DK;
    constexpr int DK2 = L::DK2;
    constexpr bool LDS_BIAS = MODE == BIAS_BF16_LDS;
    constexpr bool BIAS_DB = LDS_BIAS && PAIR;  // bias tiles double-buffered and shared
    // V operand rows of this many channel blocks are fetched from LDS before the
    // exponential phase (the rest just before their MFMAs): hides the LDS latency
    // where the register budget allows it.
    constexpr int PRE = DK <= 2 ? DK : 1;
    // key blocks between two removals of the accumulator's float-bit offset (a power of two)
    constexpr int REBASE = 8;
    __shared__ __attribute__((aligned(1024))) char bufA[NIMG * L::BYTES];
    __shared__ __attribute__((aligned(1024))) char bufB[NIMG * L::BYTES];
    // BIAS_BF16_LDS: staging of the 32 x 128 bias tiles, 8 KiB per 32-row group.
    // NB = 1: one region per wave, private to it.  NB = 2: two buffers shared by the pair.
    __shared__ __attribute__((aligned(1024))) char biasA[LDS_BIAS ? (NB == 2 && WIDE != WIDE_NONE ? 8 : 4) * 8192 : 1024];
    __shared__ __attribute__((aligned(1024))) char biasB[BIAS_DB ? 4 * 8192 : 1024];
    // BIAS_AXIAL: the head's two relative-position tables, already divided by alpha.
    //   axu: four copies of the REVERSED x table, copy j shifted by j entries, so that every
    //        lane finds its 16-entry window (ascending with the key index) 16-byte aligned.
    //        Neighbouring queries use copies 3, 2, 1, 0 at one offset, then the next lower
    //        offset: a copy pitch of 16 entries beyond a multiple of 64 puts the 16-byte reads
    //        of 16 consecutive lanes on 16 different bank groups.
    //   axw: the y table (one entry per lane and 16-key tile)
    constexpr bool AXIAL = MODE == BIAS_AXIAL;
    constexpr int AXL = 2 * AXIAL_MAX_G + 16;  // pitch of a copy, in entries
    __shared__ __attribute__((aligned(16))) float axu[AXIAL ? 4 * AXL : 4];
    __shared__ float axw[AXIAL ? AXL : 4];
    // BIAS_TABLE: the head's (2 Gy - 1) x (2 Gx - 1) table divided by alpha, every row reversed
    // in x (a lane's 16-entry window then ascends with the key index) at a pitch of TBP
    // entries.  Windows start at any entry, so they are read entry by entry; the 32 lanes of a
    // row group read 32 consecutive entries per access (or two runs 16 banks apart when the
    // group spans two grid rows).
    constexpr bool TABLE = MODE == BIAS_TABLE;
    constexpr int TBP = 2 * TABLE_MAX_G + 16;
    __shared__ float tab2[TABLE ? (2 * TABLE_MAX_G - 1) * TBP : 4];
    // BIAS_TABLE_BLK: the same bias for grids whose table does not fit LDS.  A 128-key block
    // covers 128 / Gx grid rows (or part of one) and so do the item's 128 queries, so a block
    // needs only the table rows iy - jy in [iy_lo - jy_hi, iy_hi - jy_lo]: at most 15 rows of
    // 2 Gx - 1 entries.  They are staged per block, divided by alpha and reversed in x, at a
    // pitch of 4 Gx entries (a power of two, at most 1024 entries in all), double-buffered: the
    // entries for the next block of the stream are loaded at the start of a block and written
    // to the other buffer at its end.  Lane windows are read as in BIAS_TABLE.
    constexpr bool TBLK = MODE == BIAS_TABLE_BLK;
    constexpr int TBLK_N = 1024;
    constexpr int TBLK_PER = TBLK_N / FUSED_THREADS;   // entries a thread stages (NB = 1 only)
    static_assert(!TBLK || (NB == 1 && WIDE == WIDE_NONE), "per-block table rows: 4-wave workgroups");
    __shared__ float tblk[TBLK ? 2 * TBLK_N : 4];
    // BIAS_LUT (no bias): the logit takes only the d + 1 values alpha * I, I = d, d - 2, ..., -d, and
    // the running maximum is one of them, so 255 * exp(S - m) is one of d + 1 numbers that depend
    // on the head alone: lut[k] = 255 * exp(-2 alpha k) for m - I = 2 k.  Entries d + 1 ... 2 d + 1
    // are 0: keys past the end of the sequence are given the "logit" I = -3 d - 2, below every
    // real one and at most 2 d + 1 table steps under any running maximum.  The exponential and
    // its argument disappear from the per-pair work; what remains is one address addition and
    // one LDS read.
    constexpr bool LUT = MODE == BIAS_LUT;
    constexpr int LUTN = 264;
    __shared__ float lut[LUT ? LUTN : 4];
    // delta_v of the current item (two copies: consecutive items alternate)
    __shared__ __attribute__((aligned(16))) float sdelta[2][NIMG][DKP];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3);  // 32-row group
    const int bsel = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);        // half of the workgroup
    const int isel = PAIR ? bsel : 0;                // which resident image / delta copy
    const int wreg = (NB == 2 && WIDE != WIDE_NONE) ? 4 * bsel + wave : wave;  // this wave's private bias region / copy share
    const int m = lane & 31, g = lane >> 5;
    const int N = p.N, d = p.d, W = (d + 31) / 32;
    const int nbp = p.B / NIMG;
    const int per_xcd = (p.total_wg + 7) >> 3;
    const int vmax = 8 * per_xcd;
    const int bsb = (MODE == BIAS_F32_VEC) ? 4 : 2;  // bytes per bias element

    // Work item v -> (batch, head, row block).  Consecutive ids go to different XCDs, so v
    // is first turned into (xcd, slot); items that share a bias slab (same head and row
    // block, different batch entry) are neighbours on one XCD and share it through that
    // XCD's L2.  The grid size is a multiple of 8, so a workgroup stays on its XCD.
    struct Item {
        int b, h, rb, bh;
        bool valid;
    };
    auto decode = [&](int v) -> Item {
        Item t;
        // (ONEHEAD4: ids v, v + grid size are the two row blocks of one head; grid size = vmax)
        const int j4 = ONEHEAD4 ? (v >= 2 * vmax ? 2 : v >= vmax ? 1 : 0) : 0;
        if (ONEHEAD4) v -= j4 * vmax;
        const int u = (v & 7) * per_xcd + (v >> 3);
        t.valid = v < vmax && u < p.total_wg;
        if (ONEHEAD4) t.valid = t.valid && j4 < p.nrb;
        const int uu = t.valid ? u : 0;
        t.b = ONEHEAD ? uu / p.H : (uu % nbp) * NIMG + isel;
        t.rb = ONEHEAD4 ? j4 : ONEHEAD ? bsel : ROWS2 ? 2 * ((uu / nbp) % p.nrb) + bsel : (uu / nbp) % p.nrb;
        t.h = ONEHEAD ? uu % p.H : uu / (nbp * p.nrb);
        t.bh = t.b * p.H + t.h;
        return t;
    };

    int v = blockIdx.x;
    Item cur = decode(v);
    if (!cur.valid) return;  // uniform over the workgroup

    // ---- per-item state ---------------------------------------------------------
    const char *imgs;  // block images of the item's head
    int q;             // this lane's query row
    float inv_alpha, a2;
    v4i qB[DK2];
    const char *brow = nullptr;  // this lane's bias row (register modes)
    // BIAS_BF16_LDS: the tile is fetched with full-cache-line requests (8 lanes cover the
    // 128 bytes of one row segment) straight into LDS.  Copy instruction (rg, gh) moves rows
    // 8 rg + [0, 8) x keys 64 gh + [0, 64); lane 8 r' + s fetches 16-byte chunk c = s ^ r of
    // row r = r' ^ (rg & 1), so that chunk c of row r lands at 128 (r ^ (rg & 1)) + 16 (c ^ r):
    // the later 16-byte reads of 16 consecutive rows (two row groups) at one chunk index hit
    // 16 different 16-byte bank groups of the 256-byte LDS row.
    // A wave copies RGW of the four 8-row groups of its 32-row tile: all four when the
    // tile is its own (NB = 1), two when the tile is shared with the other batch entry.
    constexpr int RGW = PAIR ? 2 : 4;
    const int rg0 = PAIR ? RGW * bsel : 0;  // first row group of the tile this wave copies
    // The copy address is a wave-uniform base (first row of the group, scalar registers,
    // advanced by scalar arithmetic) plus a 32-bit lane offset that is fixed for an item.
    struct BiasSrc {
        const char *base[RGW];
        unsigned voff[RGW];
    };
    BiasSrc bsrc;
    int dma_c[RGW];  // key chunk this lane fetches, per row group
#pragma unroll
    for (int j = 0; j < RGW; ++j) {
        bsrc.base[j] = nullptr;
        bsrc.voff[j] = 0;
        dma_c[j] = (lane & 7) ^ (lane >> 3) ^ ((rg0 + j) & 1);
    }
    int ax_ub = 0, ax_wb = 0;  // BIAS_AXIAL: this lane's window base in axu (floats), its y-table base
    float m_run, l_run, rho;  // running max (units of T = S / alpha), sum of 255 exp(S - m), rescale sum
    int hb_run = 0x7fffffff;  // BIAS_LUT: running minimum of the bit patterns of 1.5 * 2^23 + (d - I)
    float Of[DK][16];         // output carry, channel 32 cb + 8 (r/4) + 4 g + r % 4

    // registers fetched ahead for the NEXT item
    unsigned pend_q[2 * DK2];
    unsigned pend_q2[ONEHEAD4 ? 2 * DK2 : 1];  // ONEHEAD4: sign words of this lane's row in the second row block
    float pend_muq = 1.0f, pend_muk = 1.0f;
    auto fetch_item_regs = [&](const Item &t) {
        if constexpr (ONEHEAD4) {  // made by the prologue
#pragma unroll
            for (int w = 0; w < 2 * DK2; ++w) pend_q[w] = pend_q2[w];
            return;
        }
        const int qc = min(t.rb * BR + wave * ROWS_PER_WAVE + m, N - 1);
        const uint32_t *qw = p.q_bits + ((int64_t)t.bh * N + qc) * W;
#pragma unroll
        for (int w = 0; w < 2 * DK2; ++w) pend_q[w] = w < W ? qw[w] : 0u;
        pend_muq = p.mu_q ? p.mu_q[t.bh] : 1.0f;
        pend_muk = p.mu_k ? p.mu_k[t.bh] : 1.0f;
    };
    // bias pointers of an item (no memory access)
    auto bias_row_ptr = [&](const Item &t) -> const char * {
        const int qc = min(t.rb * BR + wave * ROWS_PER_WAVE + m, N - 1);
        return static_cast<const char *>(p.bias) +
               ((int64_t)t.b * p.bs.b + (int64_t)t.h * p.bs.h + (int64_t)qc * p.bs.n) * bsb;
    };
    auto bias_dma_src = [&](const Item &t) -> BiasSrc {
        BiasSrc o;
#pragma unroll
        for (int j = 0; j < RGW; ++j) {
            const int rg = rg0 + j;
            const int r = (lane >> 3) ^ (rg & 1);
            const int row0 = min(t.rb * BR + wave * ROWS_PER_WAVE + 8 * rg, N - 1);  // uniform
            const int row = min(row0 + r, N - 1);
            o.base[j] = uniform_ptr(static_cast<const char *>(p.bias) +
                                    ((int64_t)t.b * p.bs.b + (int64_t)t.h * p.bs.h + (int64_t)row0 * p.bs.n) * 2);
            o.voff[j] = (unsigned)(row - row0) * (unsigned)p.bs.n * 2u + 16u * dma_c[j];
        }
        return o;
    };
    auto image_ptr = [&](const Item &t) -> const char * {
        return uniform_ptr(p.img + (int64_t)t.bh * p.nblk * L::BYTES);
    };
    // turn the fetched registers into the item's state
    auto begin_item = [&](const Item &t) {
        imgs = image_ptr(t);
        q = t.rb * BR + wave * ROWS_PER_WAVE + m;
        // Logit multiplier alpha of Eq. 6.  Its sign goes into the Q operand and a vanishing
        // alpha clears the Q operand, so that the loop can assume alpha > 0.
        const float alpha = p.scale * pend_muq * pend_muk;
        const bool a_zero = fabsf(alpha) < 1e-30f;
        const bool a_neg = alpha < 0.0f;
        const float a_abs = a_zero ? 1.0f : fabsf(alpha);
        inv_alpha = 1.0f / a_abs;
        a2 = a_abs * LOG2E_F;  // exponent multiplier in base 2
        // (BIAS_LUT lets the matrix core SUBTRACT the logit from a constant, see the block loop)
        load_q_operand<DK2>(pend_q, d, g, LUT ? !a_neg : a_neg, a_zero, qB);
        if (LUT) {
            // (the previous item's last block is behind every wave; the barrier publishes the table)
            for (int i = threadIdx.x; i < LUTN; i += FUSED_THREADS * NB)
                lut[i] = i <= d ? __builtin_amdgcn_exp2f(fmaf(-2.0f * (float)i, a2, LOG2_255_F)) : 0.0f;
            hb_run = 0x7fffffff;
            __syncthreads();
        }
        if (MODE == BIAS_BF16_VEC || MODE == BIAS_F32_VEC) brow = bias_row_ptr(t);
        if (LDS_BIAS) {
            bsrc = bias_dma_src(t);
        }
        if (AXIAL) {
            // every wave is past the previous item's last block (begin_item follows its closing
            // barrier), so the tables can be overwritten; a barrier publishes the new ones
            const int LX = 2 * p.Gx - 1, LY = 2 * p.Gy - 1;
            const float *ux = p.ax_x + (int64_t)t.h * LX, *wy = p.ax_y + (int64_t)t.h * LY;
            // (all loads of a thread go out before the first LDS write: one memory latency)
            constexpr int NTA = FUSED_THREADS * NB;
            constexpr int NU = (4 * AXL + NTA - 1) / NTA, NW = (AXL + NTA - 1) / NTA;
            float tu[NU], tw[NW];
            int tid = threadIdx.x;  // (opaque: keeps the index arithmetic out of the block loop's registers)
            asm volatile("" : "+v"(tid));
#pragma unroll
            for (int j = 0; j < NU; ++j) {
                const int i = tid + j * NTA;
                const int kk = (i % AXL) + (i / AXL);  // index into the reversed table
                const bool on = i < 4 * AXL && kk < LX;
                tu[j] = ux[on ? LX - 1 - kk : 0];
                if (!on) tu[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const int i = tid + j * NTA;
                tw[j] = wy[i < LY ? i : 0];
                if (i >= LY) tw[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < NU; ++j) {
                const int i = tid + j * NTA;
                if (i < 4 * AXL) axu[i] = tu[j] * inv_alpha;
            }
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const int i = tid + j * NTA;
                if (i < AXL) axw[i] = tw[j] * inv_alpha;
            }
            const int qc = min(q, N - 1);
            const int ix = qc & (p.Gx - 1), iy = qc >> p.gx_shift;
            const int s0 = p.Gx - 1 - ix;  // reversed-table index of key column 0
            ax_ub = (s0 & 3) * AXL + (s0 & ~3);
            ax_wb = iy + p.Gy - 1;
            __syncthreads();
        }
        if (TABLE) {
            // (as above: the previous item's last block is behind every wave)
            const int LX = 2 * p.Gx - 1, LY = 2 * p.Gy - 1;
            const float *tb = p.table + (int64_t)t.h * LY * LX;
            // (all loads of a thread go out before the first LDS write: one memory latency)
            constexpr int NTT = FUSED_THREADS * NB;
            constexpr int TBN = ((2 * TABLE_MAX_G - 1) * TBP + NTT - 1) / NTT;
            // (the thread index is made opaque so that the per-thread table indices are
            // recomputed here instead of being kept in registers across the whole block loop)
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
            float tv[TBN];
#pragma unroll
            for (int j = 0; j < TBN; ++j) {
                const int i = tid + j * NTT;
                const int ry = i / TBP, kk = i % TBP;
                const bool on = i < LY * TBP && kk < LX;
                tv[j] = tb[on ? ry * LX + (LX - 1 - kk) : 0];
                if (!on) tv[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < TBN; ++j) {
                const int i = tid + j * NTT;
                if (i < LY * TBP) tab2[i] = tv[j] * inv_alpha;
            }
            const int qc = min(q, N - 1);
            ax_ub = p.Gx - 1 - (qc & (p.Gx - 1));       // reversed-row index of key column 0
            ax_wb = (qc >> p.gx_shift) + p.Gy - 1;      // table row of key row 0
            __syncthreads();
        }
        if (TBLK) {
            const int qc = min(q, N - 1);
            ax_ub = p.Gx - 1 - (qc & (p.Gx - 1));                               // reversed-row index of key column 0
            ax_wb = (qc >> p.gx_shift) - ((t.rb * BR) >> p.gx_shift);           // grid row inside the item's range
        }
        m_run = -INFINITY;
        l_run = 0.0f;
        rho = 0.0f;
#pragma unroll
        for (int cb = 0; cb < DK; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) Of[cb][r] = 0.0f;
    };

    // ---- bias access ----------------------------------------------------------
    auto dma_bias = [&](const BiasSrc &src, int blk, unsigned region) {  // region: LDS offset of the 8 KiB tile
#pragma unroll
        for (int j = 0; j < RGW; ++j)
#pragma unroll
            for (int gh = 0; gh < 2; ++gh) {
                const int key0 = blk * BV + 64 * gh + 8 * dma_c[j];
                if (key0 < N)  // (a last chunk that straddles N lies inside the row pitch: the host checked)
                    dma16(src.base[j] + (blk * BV + 64 * gh) * 2, src.voff[j],
                          region + ((rg0 + j) * 2 + gh) * 1024);
            }
    };
    auto dma_bias_one = [&](const BiasSrc &src, int blk, unsigned region, int idx) {  // copy idx = 2 j + gh of dma_bias
        const int j = idx >> 1, gh = idx & 1;
        const int key0 = blk * BV + 64 * gh + 8 * dma_c[j];
        if (key0 < N)
            dma16(src.base[j] + (blk * BV + 64 * gh) * 2, src.voff[j], region + ((rg0 + j) * 2 + gh) * 1024);
    };
    u4v braw[8];  // the 64 bf16 bias values of this lane for the current block
    auto load_bias_vec = [&](const char *row, int blk) {  // BIAS_BF16_VEC: registers straight from global memory
        const int k0 = blk * BV + 64 * g;
        const uint16_t *src = reinterpret_cast<const uint16_t *>(row) + k0;
        if (blk * BV + BV <= N) {
#pragma unroll
            for (int i = 0; i < 8; ++i) braw[i] = *reinterpret_cast<const u4v_a2 *>(src + 8 * i);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (k0 + 8 * i + 8 <= N) {
                    braw[i] = *reinterpret_cast<const u4v_a2 *>(src + 8 * i);
                } else {
                    unsigned e[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) e[j] = (k0 + 8 * i + j < N) ? src[8 * i + j] : 0u;
                    braw[i] = u4v{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                                  e[6] | (e[7] << 16)};
                }
            }
        }
    };
    // accumulator input of QK tile t: bias / alpha for keys blk*BV + 64 g + 16 t + [0, 16)
    auto bias_tile = [&](int blk, int t) -> v16f {
        const int k0 = blk * BV + 64 * g + 16 * t;
        v16f bt;
        if (MODE == BIAS_NONE) {
#pragma unroll
            for (int r = 0; r < 16; ++r) bt[r] = 0.0f;
        } else if (MODE == BIAS_BF16_VEC || MODE == BIAS_BF16_LDS) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const u4v w = braw[2 * t + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bt[8 * i + 2 * j] = bf16_lo(w[j]) * inv_alpha;
                    bt[8 * i + 2 * j + 1] = bf16_hi(w[j]) * inv_alpha;
                }
            }
        } else {  // BIAS_F32_VEC: 16-byte loads at float alignment, guarded at the row end
            const float *src = reinterpret_cast<const float *>(brow) + k0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (k0 + 4 * i + 4 <= N) {
                    const f4v w = *reinterpret_cast<const f4v_a4 *>(src + 4 * i);
#pragma unroll
                    for (int j = 0; j < 4; ++j) bt[4 * i + j] = w[j] * inv_alpha;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        bt[4 * i + j] = (k0 + 4 * i + j < N) ? src[4 * i + j] * inv_alpha : 0.0f;
                }
            }
        }
        return bt;
    };

    // ---- epilogue of an item: (O - magic * rho) / (255 l) * delta_v, bf16 store ----
    // A lane holds 4 consecutive channels per (cb, q4) and its partner lane ^ 32 the next 4.
    // One permlane32 swap per dword regroups two such quads so that the lower lane owns 8
    // consecutive channels of quad 2k and the upper lane those of quad 2k + 1: 16-byte stores.
    auto finish_item = [&](const Item &t, const float *dl) {
        const float l_tot = pair_sum(l_run);
        const float inv = 1.0f / l_tot;
        const float off = PV_MAGIC_F * rho;
        uint16_t *orow = p.out + (int64_t)t.b * p.os.b + (int64_t)t.h * p.os.h + (int64_t)min(q, N - 1) * p.os.n;
#pragma unroll
        for (int cb = 0; cb < DK; ++cb)
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                unsigned w[2][2];  // [quad 2k / 2k+1][dword]
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int q4 = 2 * k + e;
                    const float4 d4 = *reinterpret_cast<const float4 *>(dl + 32 * cb + 8 * q4 + 4 * g);
                    w[e][0] = pack_bf16x2((Of[cb][4 * q4 + 0] - off) * inv * d4.x,
                                          (Of[cb][4 * q4 + 1] - off) * inv * d4.y);
                    w[e][1] = pack_bf16x2((Of[cb][4 * q4 + 2] - off) * inv * d4.z,
                                          (Of[cb][4 * q4 + 3] - off) * inv * d4.w);
                }
                // lower lanes: {own quad 2k, partner's quad 2k}; upper: {partner's 2k+1, own 2k+1}
                const auto s0 = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                const int c = 32 * cb + 16 * k + 8 * g;  // first of this lane's 8 channels
                if (q < N && c < d)
                    *reinterpret_cast<u4v *>(orow + c) = u4v{s0[0], s1[0], s0[1], s1[1]};
            }
    };

    // ---- BIAS_TABLE_BLK: the table rows of one (item, key block) ------------------------
    // first row difference iy - jy of the block, and how many
    auto tblk_range = [&](const Item &t, int blk, int *dy_min) -> int {
        const int iy_lo = (t.rb * BR) >> p.gx_shift, iy_hi = min((t.rb * BR + BR - 1) >> p.gx_shift, p.Gy - 1);
        const int jy_lo = (blk * BV) >> p.gx_shift, jy_hi = min((blk * BV + BV - 1) >> p.gx_shift, p.Gy - 1);
        *dy_min = iy_lo - jy_hi;
        return iy_hi - jy_lo - *dy_min + 1;
    };
    float tstage[TBLK ? TBLK_PER : 1];
    auto tblk_load = [&](const Item &t, int blk) {  // global loads only
        int dy_min;
        const int nrows = tblk_range(t, blk, &dy_min);
        const int LX = 2 * p.Gx - 1, LY = 2 * p.Gy - 1, sh = p.gx_shift + 2;
        const float *tb = p.table + (int64_t)t.h * LY * LX;
#pragma unroll
        for (int j = 0; j < TBLK_PER; ++j) {
            const int i = threadIdx.x + j * FUSED_THREADS;
            const int row = i >> sh, kk = i & ((4 << p.gx_shift) - 1);
            const bool on = row < nrows && kk < LX;
            const float x = tb[on ? (int64_t)(dy_min + row + p.Gy - 1) * LX + (LX - 1 - kk) : 0];
            tstage[j] = on ? x : 0.0f;
        }
    };
    auto tblk_store = [&](float *dst, float ia) {
#pragma unroll
        for (int j = 0; j < TBLK_PER; ++j) dst[threadIdx.x + j * FUSED_THREADS] = tstage[j] * ia;
    };
    // 1 / |alpha| of an item from the abs-means fetched for it (as begin_item computes it)
    auto inv_alpha_of = [&](float muq, float muk) {
        const float alpha = p.scale * muq * muk;
        return fabsf(alpha) < 1e-30f ? 1.0f : 1.0f / fabsf(alpha);
    };

    // ---- stream position --------------------------------------------------------
    int it = 0;        // key block inside the current item
    const bool younger = 2 * blockIdx.x >= gridDim.x;
    int parity = 0;    // items alternate between the two delta_v copies
    Item nxt = decode(PERSIST ? v + gridDim.x : vmax);

    // One key/value block of the stream: compute block `it` of item `cur` from the image at
    // `ibuf` (and bias tile at `bbuf`), prefetch the next block of the stream into the LDS
    // offsets `inxt` / `bnxt`.  Returns false after the last block of the last item.
    auto step = [&](const char *ibuf, unsigned inxt, const char *bbuf, unsigned bnxt, int tpar) -> bool {
        const bool last = it + 1 == p.nblk;          // last block of this item
        const bool more = !last || (PERSIST && nxt.valid);  // the stream goes on
        // 0. start the copies for the next block of the stream
        const bool sw = PERSIST && last;  // ... which belongs to the next item
        const char *nimg = sw ? image_ptr(nxt) : imgs + (int64_t)(it + 1) * L::BYTES;
        const int nblkidx = sw ? 0 : it + 1;
        const BiasSrc nsrc = (LDS_BIAS && sw) ? bias_dma_src(nxt) : bsrc;
        if (!ONEHEAD && more) dma_image<DK, NWI>(nimg, inxt + isel * L::BYTES, ROWS2 ? wreg : wave, lane);
        if (!ONEHEAD && it == 0 && (ROWS2 ? wreg : wave) == 0 && lane < DKP / 4)  // delta_v of this item, for its epilogue
            dma16(p.delta + (int64_t)cur.bh * DKP, 16 * lane, lds_offset(&sdelta[parity][isel][0]));
        if (sw && nxt.valid) fetch_item_regs(nxt);
        if (TBLK && more) tblk_load(sw ? nxt : cur, nblkidx);  // lands during this block, stored at its end

        // Two 4-wave workgroups share a CU, and the SIMDs issue the older wave first: the
        // workgroup dispatched first then runs ~25 % faster than the other and leaves the CU
        // half empty at the end.  The second half of the grid (dispatched after every CU has
        // its first workgroup) therefore raises its priority on every other block.  Only a
        // scheduling hint: results do not depend on it.
        if (NB == 1) {
            if (younger && (it & 1)) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        // 1. all LDS reads of the logit phase go out together: bias tile, key rows
        if (LDS_BIAS) {
            // chunk i of this lane's row sits at row + 16 (i ^ (m & 7)) = (row + 16 (m & 7)) ^ 16 i (rows are
            // 128-byte aligned); the lane number is made opaque so that the addresses are formed here
            // instead of being carried through the block loop in eight registers per buffer
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int mm = ln & 31, gg = ln >> 5;
            const unsigned a0 = lds_offset(bbuf) + ((mm >> 3) * 2 + gg) * 1024 +
                                128 * ((mm & 7) ^ ((mm >> 3) & 1)) + 16 * (mm & 7);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                braw[i] = *reinterpret_cast<const __attribute__((address_space(3))) u4v *>((size_t)(a0 ^ (16u * i)));
        }
        v4i ka[KT][DK2];
#pragma unroll
        for (int t = 0; t < KT; ++t) load_k_operand<DK>(ibuf, t, m, g, ka[t]);
        __builtin_amdgcn_sched_barrier(0);  // all of them in flight before the first use
        //    T = I + b / alpha
        v16f T[KT];
        float wt[KT];  // BIAS_AXIAL: the y term of tile t (constant over its 16 keys), else 0
        if (AXIAL) {
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int key0 = it * BV + 64 * g + 16 * t;
                const int jx0 = key0 & (p.Gx - 1), jy = min(key0 >> p.gx_shift, p.Gy - 1);
                const float *win = axu + ax_ub + jx0;
                v16f cin;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const f4v x = *reinterpret_cast<const f4v *>(win + 4 * i);
                    cin[4 * i] = x[0]; cin[4 * i + 1] = x[1]; cin[4 * i + 2] = x[2]; cin[4 * i + 3] = x[3];
                }
                wt[t] = axw[ax_wb - jy];
                T[t] = qk_mfma<DK2>(ka[t], qB, cin);
            }
        } else if (TABLE) {
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int key0 = it * BV + 64 * g + 16 * t;  // 16 keys of one grid row (Gx >= 16)
                const int jx0 = key0 & (p.Gx - 1), jy = min(key0 >> p.gx_shift, p.Gy - 1);
                const float *win = tab2 + (ax_wb - jy) * TBP + ax_ub + jx0;
                v16f cin;
#pragma unroll
                for (int r = 0; r < 16; ++r) cin[r] = win[r];
                wt[t] = 0.0f;
                T[t] = qk_mfma<DK2>(ka[t], qB, cin);
            }
        } else if (TBLK) {
            const float *tcur = tblk + tpar * TBLK_N;
            const int jy_hi = min((it * BV + BV - 1) >> p.gx_shift, p.Gy - 1);
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int key0 = it * BV + 64 * g + 16 * t;  // 16 keys of one grid row (Gx >= 16)
                const int jx0 = key0 & (p.Gx - 1), jy = min(key0 >> p.gx_shift, p.Gy - 1);
                const float *win = tcur + ((ax_wb + jy_hi - jy) << (p.gx_shift + 2)) + ax_ub + jx0;
                v16f cin;
#pragma unroll
                for (int r = 0; r < 16; ++r) cin[r] = win[r];
                wt[t] = 0.0f;
                T[t] = qk_mfma<DK2>(ka[t], qB, cin);
            }
        } else if (LUT) {
            // 1.5 * 2^23 + d - I: an integer in [0, 2 d] on top of the float-bit offset, so the bit
            // pattern read as an integer is PV_MAGIC_BITS + (d - I) and all further logit
            // arithmetic (minimum, table address) is integer arithmetic on it
            const float cm = PV_MAGIC_F + (float)d;
            v16f cin;
#pragma unroll
            for (int r = 0; r < 16; ++r) cin[r] = cm;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                wt[t] = 0.0f;
                T[t] = qk_mfma<DK2>(ka[t], qB, cin);
            }
        } else {
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                wt[t] = 0.0f;
                T[t] = qk_mfma<DK2>(ka[t], qB, bias_tile(it, t));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (MODE == BIAS_BF16_VEC && more)  // braw is free again
            load_bias_vec(sw ? bias_row_ptr(nxt) : brow, nblkidx);
        if (LDS_BIAS && !BIAS_DB && more) {
            wait_lds();                       // this block's tile has been read into registers
            dma_bias(nsrc, nblkidx, bnxt);    // refill the wave's own region
        }
        //    the LDS reads of the P.V phase go out now and land during the exponentials
        v16i acc[DK];
        v4i va[PRE > 0 ? PRE : 1][KT];
#pragma unroll
        for (int cb = 0; cb < PRE; ++cb) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const v4i c4 = *reinterpret_cast<const v4i *>(ibuf + L::CS_OFF + 4 * (32 * cb + 8 * q4 + 4 * g));
                acc[cb][4 * q4] = c4[0]; acc[cb][4 * q4 + 1] = c4[1];
                acc[cb][4 * q4 + 2] = c4[2]; acc[cb][4 * q4 + 3] = c4[3];
            }
#pragma unroll
            for (int t = 0; t < KT; ++t)
                va[cb][t] = *reinterpret_cast<const v4i *>(ibuf + L::V_OFF + (32 * cb + m) * L::VP + 64 * g + 16 * t);
        }

        const bool ragged = it * BV + BV > N;
        if (ragged) {  // ragged last block: keys beyond N never count
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (it * BV + 64 * g + 16 * t + r >= N)
                        T[t][r] = LUT ? PV_MAGIC_F + (float)(4 * d + 2) : -INFINITY;
        }

        float resc;
        float ls0 = 0.0f, ls1 = 0.0f;
        v4i pk[KT];
        if constexpr (LUT) {
            // 2. running maximum of I = running minimum of the bit patterns (a block always holds
            //    a key inside the sequence, so the minimum is a real logit)
            int hb = __float_as_int(T[0][0]);
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) hb = min(hb, __float_as_int(T[t][r]));
            {
                const auto sw2 = __builtin_amdgcn_permlane32_swap((unsigned)hb, (unsigned)hb, false, false);
                hb = min((int)sw2[0], (int)sw2[1]);
            }
            const int hb_new = min(hb_run, hb);
            // e^{m_old - m_new} with m = alpha (d - h): the first block of an item has nothing to carry
            resc = hb_run == 0x7fffffff ? 0.0f : __builtin_amdgcn_exp2f((float)(hb_new - hb_run) * a2);
            hb_run = hb_new;
            // 3. 255 * exp(S - m) = lut[(h - h_min) / 2]: byte address 2 (h - h_min) past the table
            const unsigned abase = lds_offset(lut) - 2u * (unsigned)hb_new;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned w = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const unsigned a = ((unsigned)__float_as_int(T[t][4 * i + j]) << 1) + abase;
                        const float pe = *reinterpret_cast<const __attribute__((address_space(3))) float *>((size_t)a);
                        if (j & 1) ls1 += pe; else ls0 += pe;
                        w = __builtin_amdgcn_cvt_pk_u8_f32(pe, j, w);
                    }
                    pk[t][i] = (int)(w ^ 0x80808080u);
                }
            }
        } else {
        // 2. running maximum (Alg. 1: m_ij = max(m_i,j-1, rowmax S_ij))
        float mx;
        if (AXIAL) {  // per-tile maxima, each shifted by the tile's y term
            mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                float mt = T[t][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mt = fmaxf(mt, T[t][r]);
                mx = fmaxf(mx, mt + wt[t]);
            }
        } else {
            mx = T[0][0];
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, T[t][r]);
        }
        const float m_new = fmaxf(m_run, pair_max(mx));
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;  // whole row masked so far
        resc = __builtin_amdgcn_exp2f((m_run - m_use) * a2);  // e^{m_old - m_new}
        const float cexp = LOG2_255_F - m_use * a2;
        m_run = m_new;

        // 3. p = 255 * exp(S - m), its row sum, and the byte codes
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const float ce = AXIAL ? fmaf(wt[t], a2, cexp) : cexp;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                unsigned w = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(T[t][4 * i + j], a2, ce));
                    if (j & 1) ls1 += pe; else ls0 += pe;
                    w = __builtin_amdgcn_cvt_pk_u8_f32(pe, j, w);
                }
                pk[t][i] = (int)(w ^ 0x80808080u);  // code - 128 as signed bytes
            }
            // The shared bias tile of the next block (BIAS_DB), one copy per tile of exponentials:
            // issued in one burst at the start of the block, beside the image copies, they fill
            // the memory pipeline's queue and hold the wave there (1.5 % of the block time).
            if (BIAS_DB && more && t < 2 * RGW) dma_bias_one(nsrc, nblkidx, bnxt, t);
        }
        }
        l_run = fmaf(l_run, resc, ls0 + ls1);
        rho = fmaf(rho, resc, 1.0f);

        // 4. P~ . V~ : the prefetched channel blocks as interleaved MFMA chains ...
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int cb = 0; cb < PRE; ++cb)
                acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(va[cb][t], pk[t], acc[cb], 0, 0, 0);
        //    ... then the remaining ones
#pragma unroll
        for (int cb = PRE; cb < DK; ++cb) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const v4i c4 = *reinterpret_cast<const v4i *>(ibuf + L::CS_OFF + 4 * (32 * cb + 8 * q4 + 4 * g));
                acc[cb][4 * q4] = c4[0]; acc[cb][4 * q4 + 1] = c4[1];
                acc[cb][4 * q4 + 2] = c4[2]; acc[cb][4 * q4 + 3] = c4[3];
            }
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const v4i a = *reinterpret_cast<const v4i *>(ibuf + L::V_OFF + (32 * cb + m) * L::VP + 64 * g + 16 * t);
                acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, pk[t], acc[cb], 0, 0, 0);
            }
        }
        // 5. O = e^{m_old - m_new} O + block result
#pragma unroll
        for (int cb = 0; cb < DK; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) Of[cb][r] = fmaf(Of[cb][r], resc, __int_as_float(acc[cb][r]));
        if (TBLK && more)
            tblk_store(tblk + (tpar ^ 1) * TBLK_N, sw ? inv_alpha_of(pend_muq, pend_muk) : inv_alpha);
        __builtin_amdgcn_sched_barrier(0);  // keep the wait at the very end of the block
        wait_vmem();      // this wave's copies for the next block have landed
        __syncthreads();  // everyone is done with this block's buffers, the next ones are complete

        if (!last) {
            ++it;
            return true;
        }
        finish_item(cur, &sdelta[parity][isel][0]);
        if (!PERSIST || !nxt.valid) return false;
        cur = nxt;
        v += gridDim.x;
        nxt = decode(v + gridDim.x);
        begin_item(cur);
        it = 0;
        if (!ONEHEAD4) parity ^= 1;  // (the single-launch forms keep one copy of delta_v)
        return true;
    };

    // ---- prologue: first block of the first item --------------------------------
    const char *bA = biasA + wreg * 8192, *bB = BIAS_DB ? biasB + wave * 8192 : bA;
    if constexpr (ONEHEAD) {
        // phi and psi of Alg. 1 for this head, straight into the two LDS images.
        constexpr int NT = FUSED_THREADS * NB;
        __shared__ int sabs[DKP];            // per-channel absmax of V (bit patterns)
        __shared__ __attribute__((aligned(16))) float srlo[DKP], srhi[DKP];  // bracketing reciprocals of delta_v
        __shared__ float ssum[2][NT / 64];   // |q| and |k| partial sums per wave
        const int C16 = d / 8, nblk = p.nblk;
        auto imgp = [&](int blk) -> char * { return blk ? bufB : bufA; };
        const uint16_t *qb_ = p.xq + (int64_t)cur.b * p.xqs.b + (int64_t)cur.h * p.xqs.h;
        const uint16_t *kb_ = p.xk + (int64_t)cur.b * p.xks.b + (int64_t)cur.h * p.xks.h;
        const uint16_t *vb_ = p.xv + (int64_t)cur.b * p.xvs.b + (int64_t)cur.h * p.xvs.h;

        // Every global load of the head goes out before the first one is used, oldest first in
        // the order of use: the bias tile, this lane's query chunks, the V rows, the key chunks.
        if (LDS_BIAS) {
            bsrc = bias_dma_src(cur);
            dma_bias(bsrc, 0, lds_offset(bA));
        }
        if (MODE == BIAS_BF16_VEC) load_bias_vec(bias_row_ptr(cur), 0);
        // this lane's query row: the chunks of the sign words its B operand needs (channels
        // 64 s + 32 g + 8 j); addresses are clamped into the row, unused chunks are skipped below
        const int qrow = cur.rb * BR + wave * ROWS_PER_WAVE + m;
        u4 qx[DK2][4];
        float qsum = 0.0f;
        auto load_q_row = [&](int row) {
#pragma unroll
            for (int sI = 0; sI < DK2; ++sI)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c0 = 32 * (2 * sI + g) + 8 * j;
                    qx[sI][j] = *reinterpret_cast<const u4 *>(qb_ + (int64_t)min(row, N - 1) * p.xqs.n + (c0 < d ? c0 : 0));
                }
        };
        auto q_row_words = [&](int row, unsigned *words) {  // sign words of the loaded row, |q| into qsum
#pragma unroll
            for (int w = 0; w < 2 * DK2; ++w) words[w] = 0u;
#pragma unroll
            for (int sI = 0; sI < DK2; ++sI) {
                unsigned word = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (row < N && 32 * (2 * sI + g) + 8 * j < d) word |= sign_bits8_abs(qx[sI][j], qsum) << (8 * j);
                if (g) words[2 * sI + 1] = word; else words[2 * sI] = word;
            }
        };
        load_q_row(qrow);
        // V rows into registers: a thread owns quads of consecutive tokens of one 8-channel
        // chunk; consecutive lanes take consecutive chunks (whole-row loads)
        // i / C16 for 0 <= i < 2^12 and C16 <= 16 without the integer-division sequence:
        // (i + 0.5) / C16 is at least 1/32 away from every integer, far more than the error
        // of the fp32 product
        const float rc16 = 1.0f / (float)C16;
        auto div_c16 = [&](int i) { return (int)(((float)i + 0.5f) * rc16); };
        const int RT = div_c16(NT);           // thread groups = token quads per pass (>= 32)
        const int vr = div_c16(threadIdx.x), vc = threadIdx.x - vr * C16;
        const bool von = vr < RT;
        // (loads are unconditional from clamped rows and masked where they are used: a load
        // under a condition makes the compiler wait for it on the spot)
        // (token quads per pass: 512 threads cover the 64 quads of two key blocks in two passes
        // for every head dimension, 256 threads in at most four)
        constexpr int KQ = NB == 2 ? 2 : 4;
        u4 vw[KQ][4];
        auto v_row_on = [&](int kq, int t) { return von && 4 * (vr + kq * RT) + t < N && vr + kq * RT < 2 * BV / 4; };
#pragma unroll
        for (int kq = 0; kq < KQ; ++kq)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                vw[kq][t] = *reinterpret_cast<const u4 *>(vb_ + (int64_t)min(4 * (vr + kq * RT) + t, N - 1) * p.xvs.n + 8 * vc);
        // this thread's key chunks (8 channels of one key each), loaded before the first barrier
        constexpr int KPT = (2 * BV * 4 * DK + NT - 1) / NT;  // chunks per thread, at most
        u4 kx[KPT];
#pragma unroll
        for (int kk = 0; kk < KPT; ++kk) {
            const int i = threadIdx.x + kk * NT;
            const int ic = div_c16(i), c8 = i - ic * C16, pos = ic % BV, blk = ic / BV;
            const int key = blk * BV + key_of_position(pos);
            kx[kk] = *reinterpret_cast<const u4 *>(kb_ + (int64_t)min(key, N - 1) * p.xks.n + 8 * c8);
        }
        // clear both images, the absmax cells
        for (int i = threadIdx.x; i < L::BYTES / 16; i += NT) {
            reinterpret_cast<u4 *>(bufA)[i] = u4{0u, 0u, 0u, 0u};
            reinterpret_cast<u4 *>(bufB)[i] = u4{0u, 0u, 0u, 0u};
        }
        if (threadIdx.x < DKP) sabs[threadIdx.x] = 0;
        // the sign words of the query row (the oldest loads: V and K may still be in flight)
        q_row_words(qrow, pend_q);
        // (ONEHEAD4: the lane's row in the second row block takes the same registers; its loads
        // land during the key phase below)
        if constexpr (ONEHEAD4) load_q_row(qrow + BR);
        __syncthreads();
        // keys: sign bits -> FP4 codes of +-1 at the row position the QK tile reads
        float ksum = 0.0f;
#pragma unroll
        for (int kk = 0; kk < KPT; ++kk) {
            const int i = threadIdx.x + kk * NT;
            const int ic = div_c16(i), c8 = i - ic * C16, pos = ic % BV, blk = ic / BV;
            const int key = blk * BV + key_of_position(pos);
            if (blk < nblk && key < N) {
                const unsigned bits = sign_bits8_abs(kx[kk], ksum);
                *reinterpret_cast<unsigned *>(imgp(blk) + L::K_OFF + pos * L::KP +
                                              16 * k_chunk(pos, c8 >> 2, L::KP) + 4 * (c8 & 3)) =
                    fp4_pm1_from_bits8(bits);
            }
        }
        if constexpr (ONEHEAD4) q_row_words(qrow + BR, pend_q2);
        // V: absmax per channel through LDS integer maxima
        if (von) {
            unsigned mb[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int kq = 0; kq < KQ; ++kq)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (!v_row_on(kq, t)) vw[kq][t] = u4{0u, 0u, 0u, 0u};  // rows beyond N: code 0
                    absmax_acc(mb, vw[kq][t]);
                }
            float mf[8];
            absmax_floats(mb, mf);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (mf[i] > 0.0f) atomicMax(&sabs[8 * vc + i], __float_as_int(mf[i]));
        }
        // abs-means: wave sums, then the eight partials
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            qsum += __shfl_down(qsum, off, 64);
            ksum += __shfl_down(ksum, off, 64);
        }
        if (lane == 0) {
            ssum[0][threadIdx.x >> 6] = qsum;
            ssum[1][threadIdx.x >> 6] = ksum;
        }
        __syncthreads();
        if (threadIdx.x < 8 * C16) {
            float dl;
            quant_consts(__int_as_float(sabs[threadIdx.x]), &dl, &srlo[threadIdx.x], &srhi[threadIdx.x]);
            sdelta[0][0][threadIdx.x] = dl;
        }
        float tq = 0.0f, tk = 0.0f;
#pragma unroll
        for (int i = 0; i < NT / 64; ++i) {
            tq += ssum[0][i];
            tk += ssum[1][i];
        }
        const float inv_cnt = 1.0f / ((float)N * (float)d);
        pend_muq = p.use_mu ? tq * inv_cnt : 1.0f;
        pend_muk = p.use_mu ? tk * inv_cnt : 1.0f;
        if (threadIdx.x == 0) {
            if (p.mu_q_out) p.mu_q_out[cur.bh] = tq * inv_cnt;
            if (p.mu_k_out) p.mu_k_out[cur.bh] = tk * inv_cnt;
        }
        __syncthreads();
        // V codes, channel-major, into the images
        if (von) {
            const QuantConsts8 kc = load_quant_consts8(&sdelta[0][0][0], srlo, srhi, vc);
#pragma unroll
            for (int kq = 0; kq < KQ; ++kq) {
                const int quad = vr + kq * RT;
                if (4 * quad < N && quad < 2 * BV / 4) {
                    unsigned packed[8];
                    quant_quad(vw[kq], kc, packed);
                    char *imgq = imgp(quad / (BV / 4));
                    char *dstv = imgq + L::V_OFF + 4 * (quad % (BV / 4));
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        *reinterpret_cast<unsigned *>(dstv + (8 * vc + i) * L::VP) = packed[i];
                }
            }
        }
    } else {
        dma_image<DK, NWI>(image_ptr(cur), lds_offset(bufA) + isel * L::BYTES, ROWS2 ? wreg : wave, lane);
        fetch_item_regs(cur);
    }
    begin_item(cur);
    if (!ONEHEAD) {
        if (MODE == BIAS_BF16_VEC) load_bias_vec(brow, 0);
        if (LDS_BIAS) dma_bias(bsrc, 0, lds_offset(bA));
    }
    if (TBLK) {
        tblk_load(cur, 0);
        tblk_store(tblk, inv_alpha);
    }
    wait_vmem();
    __syncthreads();
    if constexpr (ONEHEAD) {
        // accumulator seeds of the two images: float-bit offset + 128 * (column sums of the V
        // codes), one thread per (block, channel) over the finished tiles
        if ((int)threadIdx.x < p.nblk * DKP) {
            char *imgq = threadIdx.x / DKP ? bufB : bufA;
            const int ch = threadIdx.x % DKP;
            int sum = 0;
#pragma unroll
            for (int j = 0; j < BV / 16; ++j) {
                const u4 x = *reinterpret_cast<const u4 *>(imgq + L::V_OFF + ch * L::VP + 16 * j);
#pragma unroll
                for (int n = 0; n < 4; ++n) sum = __builtin_amdgcn_sdot4((int)x[n], 0x01010101, sum, false);
            }
            reinterpret_cast<int *>(imgq + L::CS_OFF)[ch] = PV_MAGIC_BITS + 128 * sum;
        }
        __syncthreads();
    }

    const char *imgA = bufA + isel * L::BYTES, *imgB = bufB + isel * L::BYTES;
    // The carried offset 1.5 * 2^23 * rho sets the carry's rounding unit: it is taken out once
    // in REBASE blocks (one FMA per output register), so that rho stays below REBASE + 2 and a
    // block result is rounded to at most 8 units of the integer accumulator whatever N is.  (At
    // the loop's back edge: inside the block body the extra branch cost the four-channel-block
    // kernels their registers.)
    auto rebase = [&]() {
#pragma unroll
        for (int cb = 0; cb < DK; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) Of[cb][r] = fmaf(-PV_MAGIC_F, rho, Of[cb][r]);
        rho = 0.0f;
    };
    for (;;) {
        if (!step(imgA, lds_offset(bufB), bA, lds_offset(bB), 0)) break;
        if (!step(imgB, lds_offset(bufA), bB, lds_offset(bA), 1)) break;
        if (it >= REBASE && (it & (REBASE - 2)) == 0) rebase();  // `it`: the block that comes next
    }
}

template <int DK>
int launch_fused_dk(const FusedParams &p, int mode, hipStream_t stream) {
    // NB = 1, persistent grid: as many workgroups as fit on the chip at once (two 4-wave
    // workgroups per CU, 256 CUs), a multiple of 8 so that a workgroup's items stay on one
    // XCD; fewer if there is less work.  NB = 2: one workgroup per item.
    const int needed = ((p.total_wg + 7) / 8) * 8;
    if (p.wide == WIDE_ROWS2) {  // persistent, one 8-wave workgroup per CU
        if constexpr (DK == 4) {
            if (mode != BIAS_BF16_LDS) return BINATTN_ERR_DTYPE;
            const dim3 grid((unsigned)(needed < 256 ? needed : 256)), block(FUSED_THREADS * 2);
            hipLaunchKernelGGL((fused_kernel<DK, BIAS_BF16_LDS, 2, WIDE_ROWS2>), grid, block, 0, stream, p);
            return check_launch();
        }
        return BINATTN_ERR_SHAPE;
    }
    const dim3 grid((unsigned)(p.nb == 2 || needed < 512 ? needed : 512));
    const dim3 block(FUSED_THREADS * p.nb);
    if (p.nb == 2) {
        if constexpr (DK <= 2) {
            if (mode != BIAS_BF16_LDS) return BINATTN_ERR_DTYPE;
            hipLaunchKernelGGL((fused_kernel<DK, BIAS_BF16_LDS, 2>), grid, block, 0, stream, p);
            return check_launch();
        }
        return BINATTN_ERR_SHAPE;
    }
    switch (mode) {
#define CASE(M) case M: hipLaunchKernelGGL((fused_kernel<DK, M, 1>), grid, block, 0, stream, p); break;
        CASE(BIAS_NONE) CASE(BIAS_LUT) CASE(BIAS_BF16_VEC) CASE(BIAS_F32_VEC) CASE(BIAS_AXIAL) CASE(BIAS_TABLE)
        CASE(BIAS_TABLE_BLK)
#undef CASE
        case BIAS_BF16_LDS:
            if constexpr (DK <= 3) {
                hipLaunchKernelGGL((fused_kernel<DK, BIAS_BF16_LDS, 1>), grid, block, 0, stream, p);
                break;
            }
            return BINATTN_ERR_SHAPE;
        default: return BINATTN_ERR_DTYPE;
    }
    return check_launch();
}

template <int DK>
int launch_onehead_dk(const FusedParams &p, int mode, hipStream_t stream) {
    const int needed = ((p.total_wg + 7) / 8) * 8;
    if (p.nb == 1) {  // 4-wave form: the variants onehead4_built() names
        const dim3 grid((unsigned)needed), block(FUSED_THREADS);
#define CASE(M)                                                                                          \
    case M:                                                                                              \
        if constexpr (onehead4_built(DK, M)) {                                                           \
            hipLaunchKernelGGL((fused_kernel<DK, M, 1, WIDE_ONEHEAD4>), grid, block, 0, stream, p);     \
            return check_launch();                                                                       \
        }                                                                                                \
        return BINATTN_ERR_SHAPE;
        switch (mode) {
            CASE(BIAS_NONE) CASE(BIAS_LUT) CASE(BIAS_BF16_VEC) CASE(BIAS_F32_VEC) CASE(BIAS_AXIAL) CASE(BIAS_TABLE)
            CASE(BIAS_BF16_LDS)
            default: return BINATTN_ERR_DTYPE;
        }
#undef CASE
    }
    const dim3 grid((unsigned)needed), block(FUSED_THREADS * 2);
    switch (mode) {
#define CASE(M) case M: hipLaunchKernelGGL((fused_kernel<DK, M, 2, WIDE_ONEHEAD>), grid, block, 0, stream, p); break;
        CASE(BIAS_NONE) CASE(BIAS_LUT) CASE(BIAS_BF16_VEC) CASE(BIAS_F32_VEC) CASE(BIAS_AXIAL) CASE(BIAS_TABLE)
#undef CASE
        case BIAS_BF16_LDS:
            if constexpr (DK <= 3) {
                hipLaunchKernelGGL((fused_kernel<DK, BIAS_BF16_LDS, 2, WIDE_ONEHEAD>), grid, block, 0, stream, p);
                break;
            }
            return BINATTN_ERR_SHAPE;
        default: return BINATTN_ERR_DTYPE;
    }
    return check_launch();
}

}  // namespace binattn

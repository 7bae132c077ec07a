// C ABI of libbinattn: argument validation (before anything is launched) and
// the launch sequences.  See include/binattn.h for the contract.
#include "binattn_internal.h"

#include <mutex>

using namespace binattn;

// Scratch of binattn_forward_static: one array per GPU, held from the moment the library's
// code is loaded on that GPU until the process ends.  In host code this name only stands for
// the symbol; the device address is looked up once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[BINATTN_STATIC_SCRATCH_BYTES];

namespace {

bool shape_ok(int B, int H, int N, int d) {
    if (B < 1 || H < 1 || N < 1 || N > (1 << 24)) return false;
    if (d < 8 || d > 128 || (d % 8) != 0) return false;
    if ((int64_t)B * H >= ((int64_t)1 << 31) / 128) return false;
    return true;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Strides of a bf16 [B,H,N,d] tensor: non-negative, rows at least d apart and
// every stride a multiple of 8 elements (16 bytes).
int check_strides_bhnd(const int64_t st[3], const Shape &s, Strides3 *out) {
    if (!st) return BINATTN_ERR_NULL;
    for (int i = 0; i < 3; ++i)
        if (st[i] < 0 || (st[i] % 8) != 0) return BINATTN_ERR_STRIDE;
    if (s.N > 1 && st[2] < s.d) return BINATTN_ERR_STRIDE;
    out->b = st[0]; out->h = st[1]; out->n = st[2];
    return BINATTN_OK;
}

int check_workspace(const void *ws, size_t bytes, const Workspace &w) {
    if (!ws) return BINATTN_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return BINATTN_ERR_WORKSPACE;
    if (bytes < w.total) return BINATTN_ERR_WORKSPACE;
    return BINATTN_OK;
}

// Arguments common to the binattn_forward* entry points (everything but bias and workspace).
int check_forward_args(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q, const float *mu_k,
                       const void *v, const int64_t v_strides[3], const void *out,
                       const int64_t out_strides[3], int B, int H, int N, int d) {
    if (!q_bits || !k_bits || !v || !out) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    Strides3 tmp;
    int rc;
    if ((rc = check_strides_bhnd(v_strides, s, &tmp)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(out_strides, s, &tmp)) != BINATTN_OK) return rc;
    if (!aligned(v, 16) || !aligned(out, 16) || !aligned(q_bits, 4) || !aligned(k_bits, 4))
        return BINATTN_ERR_ALIGN;
    if ((mu_q && !aligned(mu_q, 4)) || (mu_k && !aligned(mu_k, 4))) return BINATTN_ERR_ALIGN;
    return BINATTN_OK;
}

// A dense bias argument (ignored when absent or switched off by the flag).
int check_dense_bias(const void *bias, int bias_dtype, const int64_t bias_strides[3], int N, unsigned flags) {
    if (bias == nullptr || (flags & BINATTN_FLAG_NO_BIAS)) return BINATTN_OK;
    if (bias_dtype != BINATTN_BIAS_BF16 && bias_dtype != BINATTN_BIAS_F32) return BINATTN_ERR_DTYPE;
    if (!bias_strides) return BINATTN_ERR_NULL;
    for (int i = 0; i < 3; ++i)
        if (bias_strides[i] < 0) return BINATTN_ERR_STRIDE;
    if (N > 1 && bias_strides[2] < N) return BINATTN_ERR_STRIDE;
    if (!aligned(bias, bias_dtype == BINATTN_BIAS_BF16 ? 2 : 4)) return BINATTN_ERR_ALIGN;
    return BINATTN_OK;
}

}  // namespace

extern "C" {

int binattn_version(void) { return 140; }

const char *binattn_strerror(int code) {
    switch (code) {
        case BINATTN_OK: return "ok";
        case BINATTN_ERR_NULL: return "a required pointer is NULL";
        case BINATTN_ERR_SHAPE: return "unsupported shape (need B,H,N >= 1, d a multiple of 8 in [8,128])";
        case BINATTN_ERR_STRIDE: return "bad stride (negative, smaller than the row, or not a multiple of 8 elements)";
        case BINATTN_ERR_ALIGN: return "base pointer not aligned as required";
        case BINATTN_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or too small";
        case BINATTN_ERR_DTYPE: return "unknown bias dtype";
        case BINATTN_ERR_LAUNCH: return "HIP runtime refused the launch";
        case BINATTN_ERR_VARIANT: return "unknown logits variant";
        case BINATTN_ERR_RANGE: return "row range outside [0, N]";
        case BINATTN_ERR_TOO_LARGE: return "the shape needs more scratch than the library's static buffer holds";
        case BINATTN_ERR_DEVICE: return "the HIP runtime could not name the current device or the static buffer";
        default: return "unknown error code";
    }
}

size_t binattn_workspace_bytes(int B, int H, int N, int d) {
    if (!shape_ok(B, H, N, d)) return 0;
    return make_workspace(make_shape(B, H, N, d)).total;
}

int binattn_pack_qk(const void *q, const void *k, int B, int H, int N, int d,
                    const int64_t q_strides[3], const int64_t k_strides[3], uint32_t *q_bits,
                    uint32_t *k_bits, float *mu_q, float *mu_k, void *stream) {
    if (!q || !k || !q_bits || !k_bits || !mu_q || !mu_k) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    Strides3 qs, ks;
    int rc;
    if ((rc = check_strides_bhnd(q_strides, s, &qs)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(k_strides, s, &ks)) != BINATTN_OK) return rc;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(q_bits, 4) || !aligned(k_bits, 4) ||
        !aligned(mu_q, 4) || !aligned(mu_k, 4))
        return BINATTN_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return launch_pack_qk(q, qs, k, ks, s, q_bits, k_bits, mu_q, mu_k, st);
}

int binattn_prepare_kv(const uint32_t *k_bits, const void *v, const int64_t v_strides[3], int B,
                       int H, int N, int d, void *workspace, size_t workspace_bytes, void *stream) {
    if (!k_bits || !v) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    const Workspace w = make_workspace(s);
    Strides3 vs;
    int rc;
    if ((rc = check_strides_bhnd(v_strides, s, &vs)) != BINATTN_OK) return rc;
    if (!aligned(v, 16) || !aligned(k_bits, 4)) return BINATTN_ERR_ALIGN;
    if ((rc = check_workspace(workspace, workspace_bytes, w)) != BINATTN_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    return launch_prepare(v, vs, k_bits, s, ws, w, st);
}

}  // extern "C" (reopened below)

namespace {

// bias generated in the kernel from relative positions on a Gy x Gx token grid: either the
// two tables of the decomposed form (y, x) or the full table (table)
struct AxialBias {
    const float *y, *x;
    int Gy, Gx;
    const float *table = nullptr;
};

// inputs of the single-launch form (binattn_forward_fused)
struct RawInputs {
    const void *q, *k, *v;
    Strides3 qs, ks, vs;
    float *mu_q_out, *mu_k_out;
};

// BIAS_AXIAL arguments: tables present and aligned, Gx a power of two in [16, 256],
// Gy in [1, 256], Gy * Gx = N.
// Full table: present and aligned, same grid limits; the single-launch form (small = true)
// holds the whole table in LDS and stops at 32 x 32.
int check_axial(const AxialBias &ax, int N, bool small = false) {
    const bool full = ax.table != nullptr;
    if (!full && (!ax.y || !ax.x)) return BINATTN_ERR_NULL;
    const int gmax = small ? TABLE_MAX_G : AXIAL_MAX_G;
    if (ax.Gy < 1 || ax.Gy > gmax || ax.Gx < 16 || ax.Gx > gmax ||
        (ax.Gx & (ax.Gx - 1)) != 0 || (int64_t)ax.Gy * ax.Gx != N)
        return BINATTN_ERR_SHAPE;
    if (full ? !aligned(ax.table, 4) : (!aligned(ax.y, 4) || !aligned(ax.x, 4))) return BINATTN_ERR_ALIGN;
    return BINATTN_OK;
}

// raw == nullptr: the attention stage over a prepared workspace (q_bits, mu_q, mu_k, workspace
// used).  raw != nullptr: the single-launch form on the bf16 inputs (those four unused).
int attend_impl(const uint32_t *q_bits, const float *mu_q, const float *mu_k, const void *bias,
                int bias_dtype, const int64_t bias_strides[3], const AxialBias *ax, const RawInputs *raw,
                float scale, int B, int H, int N, int d, void *out, const int64_t out_strides[3],
                const void *workspace, size_t workspace_bytes, unsigned flags, void *stream) {
    if ((!raw && !q_bits) || !out) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    const Workspace w = make_workspace(s);
    Strides3 os;
    int rc;
    if ((rc = check_strides_bhnd(out_strides, s, &os)) != BINATTN_OK) return rc;
    if (!aligned(out, 16) || (!raw && !aligned(q_bits, 4))) return BINATTN_ERR_ALIGN;
    if ((mu_q && !aligned(mu_q, 4)) || (mu_k && !aligned(mu_k, 4))) return BINATTN_ERR_ALIGN;

    const bool no_bias = (flags & BINATTN_FLAG_NO_BIAS) != 0;
    const bool use_bias = bias != nullptr && !no_bias;
    // without a bias BINATTN_FLAG_LUT reads the exponentials from a per-head table
    int mode = (flags & BINATTN_FLAG_LUT) ? BIAS_LUT : BIAS_NONE;
    Strides3 bs = {0, 0, 0};
    int gx_shift = 0;
    bool wide_rows2 = false;
    if (ax != nullptr) {
        if ((rc = check_axial(*ax, N, raw != nullptr && ax->table != nullptr)) != BINATTN_OK) return rc;
        while ((1 << gx_shift) < ax->Gx) ++gx_shift;
        const bool small_grid = ax->Gx <= TABLE_MAX_G && ax->Gy <= TABLE_MAX_G;
        if (!no_bias) mode = !ax->table ? BIAS_AXIAL : small_grid ? BIAS_TABLE : BIAS_TABLE_BLK;
    } else if (use_bias) {
        if (bias_dtype != BINATTN_BIAS_BF16 && bias_dtype != BINATTN_BIAS_F32) return BINATTN_ERR_DTYPE;
        if (!bias_strides) return BINATTN_ERR_NULL;
        for (int i = 0; i < 3; ++i)
            if (bias_strides[i] < 0) return BINATTN_ERR_STRIDE;
        if (N > 1 && bias_strides[2] < N) return BINATTN_ERR_STRIDE;
        bs.b = bias_strides[0]; bs.h = bias_strides[1]; bs.n = bias_strides[2];
        const int esz = bias_dtype == BINATTN_BIAS_BF16 ? 2 : 4;
        if (!aligned(bias, esz)) return BINATTN_ERR_ALIGN;
        if (bias_dtype == BINATTN_BIAS_BF16) {
            // LDS staging needs 16-byte aligned rows made of whole 16-byte chunks, and LDS
            // room for two workgroups per CU (d <= 96); everything else takes register loads.
            const bool rows16 = aligned(bias, 16) && bs.b % 8 == 0 && bs.h % 8 == 0 && bs.n % 8 == 0;
            // (and a row pitch whose 7-fold fits a 32-bit lane offset)
            // (d > 96 and at least two row blocks: 8-wave workgroups over row-block pairs)
            // (N no multiple of 8: the chunk that straddles the row end must lie inside the row pitch)
            const bool lds_ok = rows16 && (N % 8 == 0 || bs.n >= (N + 7) / 8 * 8) && bs.n < (1 << 27);
            wide_rows2 = lds_ok && s.DK == 4 && N > BR && raw == nullptr;
            mode = (lds_ok && (s.DK <= 3 || wide_rows2)) ? BIAS_BF16_LDS : BIAS_BF16_VEC;
        } else {
            mode = BIAS_F32_VEC;
        }
    }
    if (!raw && (rc = check_workspace(workspace, workspace_bytes, w)) != BINATTN_OK) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const char *ws = static_cast<const char *>(workspace);
    FusedParams p;
    p.q_bits = q_bits;
    const bool use_mu = !(flags & BINATTN_FLAG_NO_MU);
    p.mu_q = use_mu ? mu_q : nullptr;
    p.mu_k = use_mu ? mu_k : nullptr;
    p.bias = use_bias ? bias : nullptr;
    p.bs = bs;
    p.scale = scale;
    p.out = static_cast<uint16_t *>(out);
    p.os = os;
    p.img = raw ? nullptr : ws + w.img;
    p.delta = raw ? nullptr : reinterpret_cast<const float *>(ws + w.delta);
    p.B = B; p.H = H; p.N = N; p.d = d;
    p.nblk = s.nblk;
    p.ax_y = ax ? ax->y : nullptr;
    p.ax_x = ax ? ax->x : nullptr;
    p.table = ax ? ax->table : nullptr;
    p.Gy = ax ? ax->Gy : 0;
    p.Gx = ax ? ax->Gx : 0;
    p.gx_shift = gx_shift;
    p.use_mu = use_mu ? 1 : 0;
    if (raw) {
        p.xq = static_cast<const uint16_t *>(raw->q);
        p.xk = static_cast<const uint16_t *>(raw->k);
        p.xv = static_cast<const uint16_t *>(raw->v);
        p.xqs = raw->qs; p.xks = raw->ks; p.xvs = raw->vs;
        p.mu_q_out = raw->mu_q_out; p.mu_k_out = raw->mu_k_out;
        // More heads than compute units: 4-wave workgroups, two per compute unit, each taking
        // the head's two row blocks in turn; otherwise one 8-wave workgroup per head.
        const bool four = B * H > ONEHEAD4_MIN_HEADS && onehead4_built(s.DK, mode) && !(flags & BINATTN_FLAG_WIDE8);
        p.wide = four ? 3 : 1;
        p.nrb = four ? (N + BR - 1) / BR : 1;
        p.nb = four ? 1 : 2;
        p.total_wg = B * H;
        switch (s.DK) {
            case 1: return launch_onehead_dk<1>(p, mode, st);
            case 2: return launch_onehead_dk<2>(p, mode, st);
            case 3: return launch_onehead_dk<3>(p, mode, st);
            case 4: return launch_onehead_dk<4>(p, mode, st);
            default: return BINATTN_ERR_SHAPE;
        }
    }
    p.xq = p.xk = p.xv = nullptr;
    p.xqs = p.xks = p.xvs = Strides3{0, 0, 0};
    p.mu_q_out = p.mu_k_out = nullptr;
    p.wide = 0;
    p.nrb = (N + BR - 1) / BR;
    if (wide_rows2) {
        p.wide = 2;
        p.nb = 2;
        p.nrb = (p.nrb + 1) / 2;
        p.total_wg = p.nrb * H * B;
        return launch_fused_dk<4>(p, mode, st);
    }
    // Long sequences with a batch-shared, LDS-staged bias: pair batch entries in one
    // workgroup so that the bias stream is fetched once per pair.
    p.nb = (mode == BIAS_BF16_LDS && bs.b == 0 && B % 2 == 0 && s.DK <= 2 && s.nblk >= 8) ? 2 : 1;
    p.total_wg = p.nrb * H * (B / p.nb);
    switch (s.DK) {
        case 1: return launch_fused_dk<1>(p, mode, st);
        case 2: return launch_fused_dk<2>(p, mode, st);
        case 3: return launch_fused_dk<3>(p, mode, st);
        case 4: return launch_fused_dk<4>(p, mode, st);
        default: return BINATTN_ERR_SHAPE;
    }
}

}  // namespace

extern "C" {

int binattn_attend(const uint32_t *q_bits, const float *mu_q, const float *mu_k, const void *bias,
                   int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                   int d, void *out, const int64_t out_strides[3], const void *workspace,
                   size_t workspace_bytes, unsigned flags, void *stream) {
    return attend_impl(q_bits, mu_q, mu_k, bias, bias_dtype, bias_strides, nullptr, nullptr, scale, B, H, N, d,
                       out, out_strides, workspace, workspace_bytes, flags, stream);
}

int binattn_attend_axial(const uint32_t *q_bits, const float *mu_q, const float *mu_k,
                         const float *bias_y, const float *bias_x, int Gy, int Gx, float scale, int B,
                         int H, int N, int d, void *out, const int64_t out_strides[3],
                         const void *workspace, size_t workspace_bytes, unsigned flags, void *stream) {
    const AxialBias ax = {bias_y, bias_x, Gy, Gx};
    return attend_impl(q_bits, mu_q, mu_k, nullptr, 0, nullptr, &ax, nullptr, scale, B, H, N, d, out,
                       out_strides, workspace, workspace_bytes, flags, stream);
}

int binattn_attend_relpos(const uint32_t *q_bits, const float *mu_q, const float *mu_k,
                          const float *table, int Gy, int Gx, float scale, int B, int H, int N, int d,
                          void *out, const int64_t out_strides[3], const void *workspace,
                          size_t workspace_bytes, unsigned flags, void *stream) {
    if (!table) return BINATTN_ERR_NULL;
    AxialBias ax = {nullptr, nullptr, Gy, Gx};
    ax.table = table;
    return attend_impl(q_bits, mu_q, mu_k, nullptr, 0, nullptr, &ax, nullptr, scale, B, H, N, d, out,
                       out_strides, workspace, workspace_bytes, flags, stream);
}

int binattn_forward(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                    const float *mu_k, const void *v, const int64_t v_strides[3], const void *bias,
                    int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                    int d, void *out, const int64_t out_strides[3], void *workspace,
                    size_t workspace_bytes, unsigned flags, void *stream) {
    // Validate the second stage's arguments before the first stage launches anything.
    int rc = check_forward_args(q_bits, k_bits, mu_q, mu_k, v, v_strides, out, out_strides, B, H, N, d);
    if (rc != BINATTN_OK) return rc;
    if ((rc = check_dense_bias(bias, bias_dtype, bias_strides, N, flags)) != BINATTN_OK) return rc;
    if ((rc = binattn_prepare_kv(k_bits, v, v_strides, B, H, N, d, workspace, workspace_bytes,
                                 stream)) != BINATTN_OK)
        return rc;
    return binattn_attend(q_bits, mu_q, mu_k, bias, bias_dtype, bias_strides, scale, B, H, N, d, out,
                          out_strides, workspace, workspace_bytes, flags, stream);
}

}  // extern "C" (reopened below)

namespace {
// Device address of `scratch` on the current device, looked up on the first call there.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return BINATTN_ERR_DEVICE;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return BINATTN_ERR_DEVICE;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return BINATTN_OK;
}
}  // namespace

extern "C" {

int binattn_forward_static(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                           const float *mu_k, const void *v, const int64_t v_strides[3], const void *bias,
                           int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                           int d, void *out, const int64_t out_strides[3], unsigned flags, void *stream) {
    int rc = check_forward_args(q_bits, k_bits, mu_q, mu_k, v, v_strides, out, out_strides, B, H, N, d);
    if (rc != BINATTN_OK) return rc;
    if ((rc = check_dense_bias(bias, bias_dtype, bias_strides, N, flags)) != BINATTN_OK) return rc;
    const size_t need = make_workspace(make_shape(B, H, N, d)).total;
    if (need > (size_t)BINATTN_STATIC_SCRATCH_BYTES) return BINATTN_ERR_TOO_LARGE;
    void *ptr = nullptr;
    if ((rc = static_scratch(&ptr)) != BINATTN_OK) return rc;
    return binattn_forward(q_bits, k_bits, mu_q, mu_k, v, v_strides, bias, bias_dtype, bias_strides, scale, B,
                           H, N, d, out, out_strides, ptr, (size_t)BINATTN_STATIC_SCRATCH_BYTES, flags, stream);
}

int binattn_forward_axial(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                          const float *mu_k, const void *v, const int64_t v_strides[3],
                          const float *bias_y, const float *bias_x, int Gy, int Gx, float scale, int B,
                          int H, int N, int d, void *out, const int64_t out_strides[3], void *workspace,
                          size_t workspace_bytes, unsigned flags, void *stream) {
    // Validate the second stage's arguments before the first stage launches anything.
    int rc = check_forward_args(q_bits, k_bits, mu_q, mu_k, v, v_strides, out, out_strides, B, H, N, d);
    if (rc != BINATTN_OK) return rc;
    const AxialBias ax = {bias_y, bias_x, Gy, Gx};
    if ((rc = check_axial(ax, N)) != BINATTN_OK) return rc;
    if ((rc = binattn_prepare_kv(k_bits, v, v_strides, B, H, N, d, workspace, workspace_bytes,
                                 stream)) != BINATTN_OK)
        return rc;
    return binattn_attend_axial(q_bits, mu_q, mu_k, bias_y, bias_x, Gy, Gx, scale, B, H, N, d, out,
                                out_strides, workspace, workspace_bytes, flags, stream);
}

int binattn_forward_relpos(const uint32_t *q_bits, const uint32_t *k_bits, const float *mu_q,
                           const float *mu_k, const void *v, const int64_t v_strides[3],
                           const float *table, int Gy, int Gx, float scale, int B, int H, int N, int d,
                           void *out, const int64_t out_strides[3], void *workspace,
                           size_t workspace_bytes, unsigned flags, void *stream) {
    if (!table) return BINATTN_ERR_NULL;
    // Validate the second stage's arguments before the first stage launches anything.
    int rc = check_forward_args(q_bits, k_bits, mu_q, mu_k, v, v_strides, out, out_strides, B, H, N, d);
    if (rc != BINATTN_OK) return rc;
    AxialBias ax = {nullptr, nullptr, Gy, Gx};
    ax.table = table;
    if ((rc = check_axial(ax, N)) != BINATTN_OK) return rc;
    if ((rc = binattn_prepare_kv(k_bits, v, v_strides, B, H, N, d, workspace, workspace_bytes,
                                 stream)) != BINATTN_OK)
        return rc;
    return binattn_attend_relpos(q_bits, mu_q, mu_k, table, Gy, Gx, scale, B, H, N, d, out, out_strides,
                                 workspace, workspace_bytes, flags, stream);
}

}  // extern "C" (reopened below)

namespace {
// arguments of the single-launch forms: bf16 inputs and optional abs-mean exports
int check_raw(const void *q, const void *k, const void *v, const int64_t q_strides[3],
              const int64_t k_strides[3], const int64_t v_strides[3], int B, int H, int N, int d,
              const void *out, float *mu_q_out, float *mu_k_out, RawInputs *raw) {
    if (!q || !k || !v || !out) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d) || N > 2 * BV) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    int rc;
    if ((rc = check_strides_bhnd(q_strides, s, &raw->qs)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(k_strides, s, &raw->ks)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(v_strides, s, &raw->vs)) != BINATTN_OK) return rc;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16)) return BINATTN_ERR_ALIGN;
    if ((mu_q_out && !aligned(mu_q_out, 4)) || (mu_k_out && !aligned(mu_k_out, 4))) return BINATTN_ERR_ALIGN;
    raw->q = q; raw->k = k; raw->v = v;
    raw->mu_q_out = mu_q_out; raw->mu_k_out = mu_k_out;
    return BINATTN_OK;
}
}  // namespace

extern "C" {

int binattn_forward_fused(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                          const int64_t k_strides[3], const int64_t v_strides[3], const void *bias,
                          int bias_dtype, const int64_t bias_strides[3], float scale, int B, int H, int N,
                          int d, void *out, const int64_t out_strides[3], float *mu_q_out,
                          float *mu_k_out, unsigned flags, void *stream) {
    RawInputs raw;
    const int rc = check_raw(q, k, v, q_strides, k_strides, v_strides, B, H, N, d, out, mu_q_out, mu_k_out, &raw);
    if (rc != BINATTN_OK) return rc;
    return attend_impl(nullptr, nullptr, nullptr, bias, bias_dtype, bias_strides, nullptr, &raw, scale, B, H,
                       N, d, out, out_strides, nullptr, 0, flags, stream);
}

int binattn_attention(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                      const int64_t k_strides[3], const int64_t v_strides[3], const void *bias, int bias_dtype,
                      const int64_t bias_strides[3], float scale, int B, int H, int N, int d, void *out,
                      const int64_t out_strides[3], float *mu_q_out, float *mu_k_out, void *workspace,
                      size_t workspace_bytes, unsigned flags, void *stream) {
    if (N <= 2 * BV)  // at most two key blocks: everything in one launch, nothing in memory
        return binattn_forward_fused(q, k, v, q_strides, k_strides, v_strides, bias, bias_dtype, bias_strides,
                                     scale, B, H, N, d, out, out_strides, mu_q_out, mu_k_out, flags, stream);
    if (!q || !k || !v || !out) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    const Workspace w = make_workspace(s);
    Strides3 qs, ks, vs, os;
    int rc;
    if ((rc = check_strides_bhnd(q_strides, s, &qs)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(k_strides, s, &ks)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(v_strides, s, &vs)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(out_strides, s, &os)) != BINATTN_OK) return rc;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16)) return BINATTN_ERR_ALIGN;
    if ((mu_q_out && !aligned(mu_q_out, 4)) || (mu_k_out && !aligned(mu_k_out, 4))) return BINATTN_ERR_ALIGN;
    if ((rc = check_dense_bias(bias, bias_dtype, bias_strides, N, flags)) != BINATTN_OK) return rc;
    if ((rc = check_workspace(workspace, workspace_bytes, w)) != BINATTN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if ((rc = launch_phi_psi(q, qs, k, ks, v, vs, s, ws, w, mu_q_out, mu_k_out, st)) != BINATTN_OK) return rc;
    const float *mu = reinterpret_cast<const float *>(ws + w.mu);
    return binattn_attend(reinterpret_cast<const uint32_t *>(ws + w.qbits), mu, mu + s.BH, bias, bias_dtype,
                          bias_strides, scale, B, H, N, d, out, out_strides, workspace, workspace_bytes, flags,
                          stream);
}

int binattn_forward_fused_relpos(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                                 const int64_t k_strides[3], const int64_t v_strides[3], const float *table,
                                 int Gy, int Gx, float scale, int B, int H, int N, int d, void *out,
                                 const int64_t out_strides[3], float *mu_q_out, float *mu_k_out,
                                 unsigned flags, void *stream) {
    if (!table) return BINATTN_ERR_NULL;
    RawInputs raw;
    const int rc = check_raw(q, k, v, q_strides, k_strides, v_strides, B, H, N, d, out, mu_q_out, mu_k_out, &raw);
    if (rc != BINATTN_OK) return rc;
    AxialBias ax = {nullptr, nullptr, Gy, Gx};
    ax.table = table;
    return attend_impl(nullptr, nullptr, nullptr, nullptr, 0, nullptr, &ax, &raw, scale, B, H, N, d, out,
                       out_strides, nullptr, 0, flags, stream);
}

int binattn_attention_relpos(const void *q, const void *k, const void *v, const int64_t q_strides[3],
                             const int64_t k_strides[3], const int64_t v_strides[3], const float *table, int Gy,
                             int Gx, float scale, int B, int H, int N, int d, void *out,
                             const int64_t out_strides[3], float *mu_q_out, float *mu_k_out, void *workspace,
                             size_t workspace_bytes, unsigned flags, void *stream) {
    if (!table) return BINATTN_ERR_NULL;
    if (N <= 2 * BV && Gx <= TABLE_MAX_G && Gy <= TABLE_MAX_G)  // the single launch holds the whole table in LDS
        return binattn_forward_fused_relpos(q, k, v, q_strides, k_strides, v_strides, table, Gy, Gx, scale, B, H, N, d,
                                            out, out_strides, mu_q_out, mu_k_out, flags, stream);
    if (!q || !k || !v || !out) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    const Workspace w = make_workspace(s);
    Strides3 qs, ks, vs, os;
    int rc;
    if ((rc = check_strides_bhnd(q_strides, s, &qs)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(k_strides, s, &ks)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(v_strides, s, &vs)) != BINATTN_OK) return rc;
    if ((rc = check_strides_bhnd(out_strides, s, &os)) != BINATTN_OK) return rc;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16)) return BINATTN_ERR_ALIGN;
    if ((mu_q_out && !aligned(mu_q_out, 4)) || (mu_k_out && !aligned(mu_k_out, 4))) return BINATTN_ERR_ALIGN;
    AxialBias ax = {nullptr, nullptr, Gy, Gx};
    ax.table = table;
    if ((rc = check_axial(ax, N, false)) != BINATTN_OK) return rc;
    if ((rc = check_workspace(workspace, workspace_bytes, w)) != BINATTN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    if ((rc = launch_phi_psi(q, qs, k, ks, v, vs, s, ws, w, mu_q_out, mu_k_out, static_cast<hipStream_t>(stream))) !=
        BINATTN_OK)
        return rc;
    const float *mu = reinterpret_cast<const float *>(ws + w.mu);
    return binattn_attend_relpos(reinterpret_cast<const uint32_t *>(ws + w.qbits), mu, mu + s.BH, table, Gy, Gx, scale,
                                 B, H, N, d, out, out_strides, workspace, workspace_bytes, flags, stream);
}

int binattn_logits_debug(const uint32_t *q_bits, const uint32_t *k_bits, int B, int H, int N, int d,
                         int row_begin, int row_end, int32_t *logits, int variant, void *workspace,
                         size_t workspace_bytes, void *stream) {
    if (!q_bits || !k_bits || !logits) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    if (row_begin < 0 || row_end < row_begin || row_end > N) return BINATTN_ERR_RANGE;
    const bool rowsum = (variant & BINATTN_LOGITS_ROWSUM) != 0;
    variant &= ~BINATTN_LOGITS_ROWSUM;
    if (variant != BINATTN_LOGITS_POPCOUNT && variant != BINATTN_LOGITS_MFMA_I8 &&
        variant != BINATTN_LOGITS_MFMA_FP4)
        return BINATTN_ERR_VARIANT;
    if (!aligned(q_bits, 4) || !aligned(k_bits, 4) || !aligned(logits, 4)) return BINATTN_ERR_ALIGN;
    const Shape s = make_shape(B, H, N, d);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (variant == BINATTN_LOGITS_POPCOUNT)
        return launch_logits_popcount(q_bits, k_bits, s, row_begin, row_end, logits, rowsum, st);
    if (variant == BINATTN_LOGITS_MFMA_I8)
        return launch_logits_i8(q_bits, k_bits, s, row_begin, row_end, logits, rowsum, st);
    const Workspace w = make_workspace(s);
    int rc;
    if ((rc = check_workspace(workspace, workspace_bytes, w)) != BINATTN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    if ((rc = launch_expand_k(k_bits, s, ws, w, st)) != BINATTN_OK) return rc;
    return launch_logits_fp4(q_bits, ws, w, s, row_begin, row_end, logits, rowsum, st);
}

int binattn_quant_v_debug(const void *v, const int64_t v_strides[3], int B, int H, int N, int d,
                          int8_t *vq, float *delta, void *workspace, size_t workspace_bytes,
                          void *stream) {
    if (!v || !vq || !delta) return BINATTN_ERR_NULL;
    if (!shape_ok(B, H, N, d)) return BINATTN_ERR_SHAPE;
    const Shape s = make_shape(B, H, N, d);
    const Workspace w = make_workspace(s);
    Strides3 vs;
    int rc;
    if ((rc = check_strides_bhnd(v_strides, s, &vs)) != BINATTN_OK) return rc;
    if (!aligned(v, 16) || !aligned(delta, 4)) return BINATTN_ERR_ALIGN;
    if ((rc = check_workspace(workspace, workspace_bytes, w)) != BINATTN_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    if ((rc = launch_prepare(v, vs, nullptr, s, ws, w, st)) != BINATTN_OK) return rc;
    return launch_export_vq(s, ws, w, vq, delta, st);
}

int binattn_probe_valu(int op, int iters, int blocks, float *out, void *stream) {
    if (!out) return BINATTN_ERR_NULL;
    if (iters < 1 || blocks < 1 || blocks > (1 << 20)) return BINATTN_ERR_SHAPE;
    if (!aligned(out, 4)) return BINATTN_ERR_ALIGN;
    return launch_probe_valu(op, iters, blocks, out, static_cast<hipStream_t>(stream));
}

}  // extern "C"

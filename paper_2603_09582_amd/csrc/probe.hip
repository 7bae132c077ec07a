// Issue-rate probe for the vector-ALU instructions the softmax part of the fused kernel is
// made of.  The kernel's roofline is "lane-instructions per second" of the vector ALU; this
// probe measures how many issue slots each instruction kind really takes on the chip (a
// dependent-free stream, eight independent chains per lane, every lane busy), which is where
// the count of two slots for v_exp_f32 comes from, and - with two kinds mixed half and half -
// which kinds can issue side by side.  Not part of the attention path.
#include "binattn_internal.h"

namespace binattn {

constexpr int PROBE_CHAINS = 8;

// one instruction of kind OP on chain state (x, u); `o` is another chain's integer state
template <int OP>
__device__ __forceinline__ void probe_step(float &x, unsigned &u, float seed, unsigned o) {
    if (OP == BINATTN_PROBE_FMA) x = fmaf(x, 1.0001f, 0.5f);
    if (OP == BINATTN_PROBE_EXP2) x = __builtin_amdgcn_exp2f(x);
    if (OP == BINATTN_PROBE_ADD) x = x + seed;
    if (OP == BINATTN_PROBE_MAX3) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x) : "v"(seed), "v"(o));
    if (OP == BINATTN_PROBE_CVT_PK_U8) u = __builtin_amdgcn_cvt_pk_u8_f32(x, 1, u);
    if (OP == BINATTN_PROBE_CVT_F32_I32) asm volatile("v_cvt_f32_i32 %0, %0" : "+v"(x));
    // (inline assembly where the compiler would fold a chain of the same integer operation)
    if (OP == BINATTN_PROBE_OR) asm volatile("v_or_b32 %0, %1, %0" : "+v"(u) : "v"(o));
    if (OP == BINATTN_PROBE_MUL) x = x * 1.0001f;
    if (OP == BINATTN_PROBE_LSHL) asm volatile("v_lshlrev_b32 %0, 16, %0" : "+v"(u));
    if (OP == BINATTN_PROBE_AND) asm volatile("v_and_b32 %0, 0xffff0000, %0" : "+v"(u));
    if (OP == BINATTN_PROBE_XOR) asm volatile("v_xor_b32 %0, 0x80808080, %0" : "+v"(u));
    if (OP == BINATTN_PROBE_MIN3_I32) asm volatile("v_min3_i32 %0, %0, %1, %1" : "+v"(u) : "v"(o));
    if (OP == BINATTN_PROBE_LSHL_ADD) asm volatile("v_lshl_add_u32 %0, %0, 1, %1" : "+v"(u) : "v"(o));
    if (OP == BINATTN_PROBE_MOV) asm volatile("v_mov_b32 %0, %1" : "+v"(u) : "v"(o));
    if (OP == BINATTN_PROBE_ADD_U32) asm volatile("v_add_u32 %0, %0, %1" : "+v"(u) : "v"(o));
    if (OP == BINATTN_PROBE_PERM) asm volatile("v_perm_b32 %0, %0, %1, %1" : "+v"(u) : "v"(o));
}

// chains 0-3 run kind A, chains 4-7 kind B (A == B: one kind)
template <int A, int B>
__global__ __launch_bounds__(256) void probe_valu_kernel(float *out, int iters, float seed) {
    float x[PROBE_CHAINS];
    unsigned u[PROBE_CHAINS];
#pragma unroll
    for (int i = 0; i < PROBE_CHAINS; ++i) {
        x[i] = seed + threadIdx.x * 1e-3f + i;
        u[i] = threadIdx.x + i;
    }
    const unsigned o = threadIdx.x * 2654435761u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_CHAINS; ++i) {
            // (interleaved: A, B, A, B, ...)
            if (i & 1) probe_step<B>(x[i], u[i], seed, o);
            else probe_step<A>(x[i], u[i], seed, o);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < PROBE_CHAINS; ++i) s += x[i] + (float)u[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The per-pair vector work of the fused kernel's block loop on synthetic register data (bias
// unpack + scale, maximum, exponent FMA + v_exp_f32, row sum, byte codes), 16 values per lane
// and step, with `lds_bytes` of dynamic LDS per workgroup so that the launch can pin the number
// of waves per SIMD: how does the mix scale with occupancy?
__global__ __launch_bounds__(256) void probe_softmax_kernel(float *out, int iters, float seed) {
    extern __shared__ char probe_lds[];
    unsigned w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = 0x3c003c00u + threadIdx.x * 65537u + i * 257u;
    const float ia = seed * 1.01f, a2 = seed * 0.1f;
    float ls0 = 0.0f, ls1 = 0.0f, mrun = -1e30f;
    unsigned chk = 0;
    for (int it = 0; it < iters; ++it) {
        float t[16];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            t[2 * i] = __uint_as_float(w[i] << 16) * ia;
            t[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u) * ia;
        }
        float mx = t[0];
#pragma unroll
        for (int i = 1; i < 16; i += 2) mx = fmaxf(fmaxf(mx, t[i]), t[(i + 1) & 15]);
        mrun = fmaxf(mrun, mx);
        const float ce = 7.99f - mrun * a2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned pk = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(t[4 * i + j], a2, ce));
                if (j & 1) ls1 += pe; else ls0 += pe;
                pk = __builtin_amdgcn_cvt_pk_u8_f32(pe, j, pk);
            }
            chk += pk ^ 0x80808080u;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] += (chk & 0x00010001u) + 0x00010000u;  // new "bias" words
    }
    if (probe_lds[threadIdx.x] == 77) chk += 1;  // (keeps the LDS allocation)
    out[blockIdx.x * blockDim.x + threadIdx.x] = ls0 + ls1 + (float)chk + mrun;
}

template <int A>
static int launch_probe_b(int b, int iters, dim3 grid, float *out, hipStream_t stream) {
    const dim3 block(256);
    switch (b) {
#define CASE(K) case K: hipLaunchKernelGGL((probe_valu_kernel<A, K>), grid, block, 0, stream, out, iters, 1.0f); break;
        CASE(BINATTN_PROBE_FMA) CASE(BINATTN_PROBE_CVT_PK_U8) CASE(BINATTN_PROBE_EXP2) CASE(BINATTN_PROBE_OR)
#undef CASE
        default:
            if (b != A) return BINATTN_ERR_VARIANT;
            hipLaunchKernelGGL((probe_valu_kernel<A, A>), grid, block, 0, stream, out, iters, 1.0f);
    }
    return check_launch();
}

// op = A | (B << 8); B is A itself or one of fma, cvt_pk_u8, exp2, or
int launch_probe_valu(int op, int iters, int blocks, float *out, hipStream_t stream) {
    const int a = op & 0xff, b = (op >> 8) & 0xff;
    const dim3 grid((unsigned)blocks);
    if (a == BINATTN_PROBE_SOFTMAX) {  // bits 8.. : KiB of LDS per workgroup (1 ... 160)
        const int kib = (op >> 8) & 0xff;
        if (kib < 1 || kib > 160) return BINATTN_ERR_VARIANT;
        if (kib > 64 && hipFuncSetAttribute(reinterpret_cast<const void *>(probe_softmax_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, kib * 1024) != hipSuccess)
            return BINATTN_ERR_LAUNCH;
        hipLaunchKernelGGL(probe_softmax_kernel, grid, dim3(256), (size_t)kib * 1024, stream, out, iters, 1.0f);
        return check_launch();
    }
    switch (a) {
#define CASE(K) case K: return launch_probe_b<K>(b, iters, grid, out, stream);
        CASE(0) CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11)
        CASE(12) CASE(13) CASE(14) CASE(15)
#undef CASE
        default: return BINATTN_ERR_VARIANT;
    }
}

}  // namespace binattn

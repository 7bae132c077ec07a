// Issue-rate probe for the vector-ALU instructions the softmax part of the fused kernel is
// made of.  The kernel's roofline is "lane-instructions per second" of the vector ALU; this
// probe measures how many issue slots each instruction kind really takes on the chip (a
// dependent-free stream of one kind, eight independent chains per lane, every lane busy), which
// is where the count of two slots for v_exp_f32 comes from.  Not part of the attention path.
#include "binattn_internal.h"

namespace binattn {

constexpr int PROBE_CHAINS = 8;

template <int OP>
__global__ __launch_bounds__(256) void probe_valu_kernel(float *out, int iters, float seed) {
    float x[PROBE_CHAINS];
    unsigned u[PROBE_CHAINS];
#pragma unroll
    for (int i = 0; i < PROBE_CHAINS; ++i) {
        x[i] = seed + threadIdx.x * 1e-3f + i;
        u[i] = threadIdx.x + i;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_CHAINS; ++i) {
            if (OP == BINATTN_PROBE_FMA) x[i] = fmaf(x[i], 1.0001f, 0.5f);
            if (OP == BINATTN_PROBE_EXP2) x[i] = __builtin_amdgcn_exp2f(x[i]);
            if (OP == BINATTN_PROBE_ADD) x[i] = x[i] + seed;
            if (OP == BINATTN_PROBE_MAX3) x[i] = fmaxf(fmaxf(x[i], x[(i + 1) % PROBE_CHAINS]), seed);
            if (OP == BINATTN_PROBE_CVT_PK_U8) {  // two instructions: the conversion and an OR that keeps the chain in floats
                u[i] = __builtin_amdgcn_cvt_pk_u8_f32(x[i], 1, u[i]);
                x[i] = __uint_as_float(u[i] | 0x3f800000u);
            }
            if (OP == BINATTN_PROBE_CVT_F32_I32) x[i] = (float)(int)__float_as_uint(x[i]);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < PROBE_CHAINS; ++i) s += x[i] + (float)u[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

int launch_probe_valu(int op, int iters, int blocks, float *out, hipStream_t stream) {
    const dim3 grid((unsigned)blocks), block(256);
    switch (op) {
#define CASE(K) case K: hipLaunchKernelGGL(probe_valu_kernel<K>, grid, block, 0, stream, out, iters, 1.0f); break;
        CASE(BINATTN_PROBE_FMA) CASE(BINATTN_PROBE_EXP2) CASE(BINATTN_PROBE_ADD) CASE(BINATTN_PROBE_MAX3)
        CASE(BINATTN_PROBE_CVT_PK_U8) CASE(BINATTN_PROBE_CVT_F32_I32)
#undef CASE
        default: return BINATTN_ERR_VARIANT;
    }
    return check_launch();
}

}  // namespace binattn

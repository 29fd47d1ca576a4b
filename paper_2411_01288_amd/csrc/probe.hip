// Benchmark helper: a register-only bf16 MFMA loop, to measure the matrix rate the part sustains
// at the clock its power limit allows (the ceiling the contraction kernels are compared with,
// next to the nominal 2.5 PFLOP/s).  Not part of the layer.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Every wavefront issues iters * 32 MFMAs (16x16x32, the instruction the contraction kernels use,
// 16 384 FLOP each) on eight independent accumulators; operands never leave registers.  The
// operands are pseudo-random values of the size the layer's activations have: the sustained clock
// depends on how many operand bits toggle (measured: 2.3-2.5 PFLOP/s on all-zero operands,
// 1.9 PFLOP/s on random ones; 1.8 with 32x32x16 MFMAs).  The result is written only if it is NaN,
// which these operands cannot produce: the store keeps the loop alive.
__global__ __launch_bounds__(256) void mfma_probe(int iters, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t h = (uint32_t)(lane * 8 + i) * 2654435761u;
        h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
        a[i] = (__bf16)(((float)(h & 0xffffu) / 65536.f - 0.5f) * 0.1f);
        b[i] = (__bf16)(((float)(h >> 16) / 65536.f - 0.5f) * 0.1f);
    }
    f32x4 c[8] = {};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            c[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[0], 0, 0, 0);
            c[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, a, c[1], 0, 0, 0);
            c[2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, a, c[2], 0, 0, 0);
            c[3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, b, c[3], 0, 0, 0);
            c[4] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[4], 0, 0, 0);
            c[5] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, a, c[5], 0, 0, 0);
            c[6] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, a, c[6], 0, 0, 0);
            c[7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, b, c[7], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
    if (s != s) sink[0] = s;
}

}  // namespace

extern "C" hexa_status hexa_moe_mfma_probe(int32_t workgroups, int32_t iters, float* sink, void* stream,
                                           double* flop) {
    if (!sink || !flop) return HEXA_ERR_NULL;
    if (workgroups <= 0 || iters <= 0) return HEXA_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_probe, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, iters, sink);
    *flop = (double)workgroups * 4.0 * (double)iters * 32.0 * 16384.0;
    return hipGetLastError() == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE;
}

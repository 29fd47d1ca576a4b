// Benchmark helper (include/hexa_moe_bench.h): a register-only MFMA loop, to measure the matrix
// rate the part sustains at the clock its power limit allows (the ceiling the contraction kernels
// are compared with, next to the nominal 2.5 PFLOP/s).  Not part of the layer.
#include "common.h"
#include "../../include/hexa_moe_bench.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every wavefront issues iters * 32 MFMAs of 16 384 FLOP each (VARIANT 2: iters * 16 of 32 768) on
// independent accumulators; operands never leave registers.  The sustained clock depends on how
// many operand bits toggle, so the operands are either pseudo-random values of the size the
// layer's activations have (VARIANT 0: 16x16x32, the instruction the contraction kernels use;
// VARIANT 2: 32x32x16) or all zero (VARIANT 1, 16x16x32).  The result is written only if it is
// NaN, which these operands cannot produce: the store keeps the loop alive.
template <int VARIANT>
__global__ __launch_bounds__(256) void mfma_probe(int iters, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t h = (uint32_t)(lane * 8 + i) * 2654435761u;
        h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
        a[i] = (__bf16)(VARIANT == 1 ? 0.f : ((float)(h & 0xffffu) / 65536.f - 0.5f) * 0.1f);
        b[i] = (__bf16)(VARIANT == 1 ? 0.f : ((float)(h >> 16) / 65536.f - 0.5f) * 0.1f);
    }
    // keep the compiler from folding the all-zero case
    asm volatile("" : "+v"(a), "+v"(b));
    float s = 0.f;
    if constexpr (VARIANT == 2) {
        f32x16 c[4] = {};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[0], 0, 0, 0);
                c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c[1], 0, 0, 0);
                c[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, a, c[2], 0, 0, 0);
                c[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, b, c[3], 0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) s += c[i][q];
    } else {
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
#pragma unroll
        for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
    }
    if (s != s) sink[0] = s;
}

}  // namespace

extern "C" hexa_status hexa_moe_mfma_probe(int32_t variant, int32_t workgroups, int32_t iters, float* sink,
                                           void* stream, double* flop) {
    if (!sink || !flop) return HEXA_ERR_NULL;
    if (workgroups <= 0 || iters <= 0) return HEXA_ERR_SHAPE;
    if (variant < 0 || variant > 2) return HEXA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    if (variant == 0) hipLaunchKernelGGL(mfma_probe<0>, dim3(workgroups), dim3(256), 0, st, iters, sink);
    else if (variant == 1) hipLaunchKernelGGL(mfma_probe<1>, dim3(workgroups), dim3(256), 0, st, iters, sink);
    else hipLaunchKernelGGL(mfma_probe<2>, dim3(workgroups), dim3(256), 0, st, iters, sink);
    // both forms do 16384 * 32 FLOP per loop iteration and accumulator set
    *flop = (double)workgroups * 4.0 * (double)iters * 32.0 * 16384.0;
    return hipGetLastError() == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE;
}

// fp32 path: the same dataflow as the bf16 MFMA path (App. B Table 5 rows 1-10 on the re-index
// vector) with plain FMA tiles.  It exists for the precision-critical fp32 workloads, where
// products must stay in fp32; throughput is not its purpose.
#include "common.h"

namespace {

constexpr int TS = 16;

enum RowsMode { F32_FC1 = 0, F32_FC2 = 1, F32_DGRAD2 = 2, F32_DGRAD1 = 3 };

struct RowsArgs {
    const float* A;        // row operand; rows are perm positions, or tokens when `gather`
    int lda;
    const int32_t* perm;   // used when gather
    int k;                 // top-k (token = perm[p] / k)
    int gather;
    const float* B;        // [E] matrices
    size_t b_expert_stride;
    int sbk, sbn;          // element strides of B along the contraction and the output column
    const float* bias;     // [E][N] or NULL
    const float* pre_in;   // DGRAD2: saved pre-activations [A][N]
    float* out0;           // [A][N]
    float* out1;           // FC1: h
    int K, N, E, mode;
    int act;               // hexa_activation (FC1, DGRAD2)
    const int32_t* offsets;
};

__device__ __forceinline__ float gelu_f(float u) {
    return 0.5f * u * (1.f + tanhf(HEXA_GELU_C * (u + HEXA_GELU_A * u * u * u)));
}
__device__ __forceinline__ float gelu_grad_f(float u) {
    const float th = tanhf(HEXA_GELU_C * (u + HEXA_GELU_A * u * u * u));
    return 0.5f * (1.f + th) +
           0.5f * u * (1.f - th * th) * HEXA_GELU_C * (1.f + 3.f * HEXA_GELU_A * u * u);
}

// F and F' for the three activations (accurate library functions: this is the 1e-5 path)
__device__ __forceinline__ float act_f(float u, int act) {
    if (act == HEXA_ACT_RELU) return u > 0.f ? u : 0.f;
    if (act == HEXA_ACT_SILU) return u / (1.f + expf(-u));
    return gelu_f(u);
}
__device__ __forceinline__ float act_grad_f(float u, int act) {
    if (act == HEXA_ACT_RELU) return u > 0.f ? 1.f : 0.f;
    if (act == HEXA_ACT_SILU) {
        const float sg = 1.f / (1.f + expf(-u));
        return sg * (1.f + u * (1.f - sg));
    }
    return gelu_grad_f(u);
}

// ESMM (Sec. 3.1 item 1; App. B Alg. 2): one 16x16 output tile of one expert segment per workgroup.
__global__ __launch_bounds__(256) void f32_rows_gemm(RowsArgs a) {
    __shared__ float As[TS][TS + 1], Bs[TS][TS + 1];
    const SegTile s = seg_tile_find(a.offsets, a.E, TS, blockIdx.x);
    if (s.e < 0) return;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n0 = blockIdx.y * TS;
    // row operand source row for the row this thread loads (ty)
    long long src_row = -1;
    if (ty < s.rows) {
        const int p = s.row0 + ty;
        src_row = a.gather ? (long long)(a.perm[p] / a.k) : (long long)p;
    }
    const float* Be = a.B + (size_t)s.e * a.b_expert_stride;
    float acc = 0.f;
    for (int k0 = 0; k0 < a.K; k0 += TS) {
        const int ka = k0 + tx;
        As[ty][tx] = (src_row >= 0 && ka < a.K) ? a.A[(size_t)src_row * a.lda + ka] : 0.f;
        const int kb = k0 + ty, nb = n0 + tx;
        Bs[ty][tx] = (kb < a.K && nb < a.N) ? Be[(size_t)kb * a.sbk + (size_t)nb * a.sbn] : 0.f;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < TS; ++q) acc = fmaf(As[ty][q], Bs[q][tx], acc);
        __syncthreads();
    }
    const int n = n0 + tx;
    if (ty >= s.rows || n >= a.N) return;
    const size_t oi = (size_t)(s.row0 + ty) * a.N + n;
    if (a.bias) acc += a.bias[(size_t)s.e * a.N + n];
    if (a.mode == F32_FC1) {
        a.out0[oi] = acc;
        a.out1[oi] = act_f(acc, a.act);
    } else if (a.mode == F32_DGRAD2) {
        a.out0[oi] = acc * act_grad_f(a.pre_in[oi], a.act);
    } else {
        a.out0[oi] = acc;
    }
}

struct WgradArgs {
    const float* A;       // [rows][M]; rows are perm positions, or tokens when gather
    const int32_t* perm;
    int k, gather;
    const float* B;       // [A][N] perm order
    float* out;           // [E][M][N]
    int M, N;
    const int32_t* offsets;
};

// ESTMM (Sec. 3.1 item 3; App. B Alg. 4): out[e] = sum over the expert's rows of A_row^T B_row.
__global__ __launch_bounds__(256) void f32_wgrad(WgradArgs a) {
    __shared__ float As[TS][TS + 1], Bs[TS][TS + 1];
    const int e = blockIdx.z;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
    const int b = a.offsets[e], end = a.offsets[e + 1];
    float acc = 0.f;
    for (int p0 = b; p0 < end; p0 += TS) {
        const int p = p0 + ty;
        float av = 0.f, bv = 0.f;
        if (p < end) {
            const size_t ar = a.gather ? (size_t)(a.perm[p] / a.k) : (size_t)p;
            if (m0 + tx < a.M) av = a.A[ar * a.M + m0 + tx];
            if (n0 + tx < a.N) bv = a.B[(size_t)p * a.N + n0 + tx];
        }
        As[ty][tx] = av;
        Bs[ty][tx] = bv;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < TS; ++q) acc = fmaf(As[q][ty], Bs[q][tx], acc);
        __syncthreads();
    }
    const int m = m0 + ty, n = n0 + tx;
    if (m < a.M && n < a.N) a.out[((size_t)e * a.M + m) * a.N + n] = acc;
}

void rows_launch(const MoeDims& D, const RowsArgs& a, hipStream_t st) {
    static const char* names[] = {"fc1", "fc2", "dgrad2", "dgrad1"};
    ProfScope ps(st, names[a.mode]);
    const int max_tiles = D.A / TS + D.E;
    hipLaunchKernelGGL(f32_rows_gemm, dim3(max_tiles, ceil_div(a.N, TS)), dim3(256), 0, st, a);
}

}  // namespace

hipError_t launch_f32_fwd(const MoeDims& D, const float* x, const float* W1, const float* b1,
                          const float* W2, const float* b2, const hexa_moe_idx& idx,
                          const MoeWorkspace& ws, hipStream_t st) {
    RowsArgs a{};
    a.offsets = idx.offsets; a.perm = idx.perm; a.k = D.k; a.E = D.E; a.act = D.act;
    // fc1: pre = x W1 + b1, h = F(pre)
    a.A = x; a.lda = D.d; a.gather = 1;
    a.B = W1; a.b_expert_stride = (size_t)D.d * D.f; a.sbk = D.f; a.sbn = 1;
    a.bias = b1; a.out0 = (float*)ws.pre; a.out1 = (float*)ws.h; a.K = D.d; a.N = D.f; a.mode = F32_FC1;
    rows_launch(D, a, st);
    // fc2: o = h W2 + b2
    a.A = (const float*)ws.h; a.lda = D.f; a.gather = 0;
    a.B = W2; a.b_expert_stride = (size_t)D.f * D.d; a.sbk = D.d; a.sbn = 1;
    a.bias = b2; a.out0 = (float*)ws.o; a.out1 = nullptr; a.K = D.f; a.N = D.d; a.mode = F32_FC2;
    rows_launch(D, a, st);
    return hipGetLastError();
}

hipError_t launch_f32_bwd(const MoeDims& D, const float* x, const float* W1, const float* W2,
                          const hexa_moe_idx& idx, const MoeWorkspace& ws, float* dW1, float* dW2,
                          hipStream_t st) {
    RowsArgs a{};
    a.offsets = idx.offsets; a.perm = idx.perm; a.k = D.k; a.E = D.E; a.act = D.act; a.gather = 0;
    // dh = do W2^T ; dpre = dh * GELU'(pre)
    a.A = (const float*)ws.dout; a.lda = D.d;
    a.B = W2; a.b_expert_stride = (size_t)D.f * D.d; a.sbk = 1; a.sbn = D.d;
    a.pre_in = (const float*)ws.pre; a.out0 = (float*)ws.dpre; a.K = D.d; a.N = D.f; a.mode = F32_DGRAD2;
    rows_launch(D, a, st);
    // dxp = dpre W1^T
    a.A = (const float*)ws.dpre; a.lda = D.f;
    a.B = W1; a.b_expert_stride = (size_t)D.d * D.f; a.sbk = 1; a.sbn = D.f;
    a.pre_in = nullptr; a.out0 = (float*)ws.dxp; a.K = D.f; a.N = D.d; a.mode = F32_DGRAD1;
    rows_launch(D, a, st);
    // dW2[e] = h^T do ; dW1[e] = x^T dpre
    WgradArgs w{};
    w.offsets = idx.offsets; w.perm = idx.perm; w.k = D.k;
    w.A = (const float*)ws.h; w.gather = 0; w.B = (const float*)ws.dout; w.out = dW2; w.M = D.f; w.N = D.d;
    { ProfScope ps(st, "wgrad2");
    hipLaunchKernelGGL(f32_wgrad, dim3(ceil_div(w.N, TS), ceil_div(w.M, TS), D.E), dim3(256), 0, st, w); }
    w.A = x; w.gather = 1; w.B = (const float*)ws.dpre; w.out = dW1; w.M = D.d; w.N = D.f;
    { ProfScope ps(st, "wgrad1");
    hipLaunchKernelGGL(f32_wgrad, dim3(ceil_div(w.N, TS), ceil_div(w.M, TS), D.E), dim3(256), 0, st, w); }
    return hipGetLastError();
}

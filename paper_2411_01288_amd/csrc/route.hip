// Router front-end: top-k selection over a token's E logits and the gate weights, i.e. the step
// that produces the routing choice {R_j(x)} the expert-specific operators take as input (HEXA-MoE
// Sec. 3.1; App. B Table 5).  The paper treats the router as given; the rule here is the usual one:
// the k largest logits, equal logits to the lower expert id, slots in descending order of logit,
// gates = softmax over the selected logits (or the full softmax evaluated at them).
//
// Two kernels.  E <= 64 and k <= 16 (the usual case): 16 lanes per token, lane g holding the
// E/16 (rounded up) consecutive logits from g*VPL on, so a wavefront takes four tokens per pass and
// several passes, its loads all issued up front; each of the k rounds is an arg-max over
// (logit, -expert id) inside the 16-lane row.  Otherwise one 64-lane wavefront per token, lane l
// holding logits l, l+64, ... (E <= 1024).  Selection uses comparisons only, so the indices are
// bit-exact whatever the float environment.  HBM-bound: T*E*4 bytes in, T*k*8 out (35.7 MB at
// T = 131072, E = 64, k = 2).
#include "common.h"

namespace {

constexpr int kMaxPerLane = 16;   // E <= 64 * 16

__device__ __forceinline__ bool better(float v, int e, float bv, int be) {
    return v > bv || (v == bv && e < be);
}

template <int NPL>   // logits per lane
__global__ __launch_bounds__(256) void route_topk(int T, int E, int k, int mode,
                                                  const float* __restrict__ logits,
                                                  int32_t* __restrict__ topk_idx,
                                                  float* __restrict__ gate) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float* row = logits + (size_t)t * E;
    const float NEG = -__builtin_huge_valf();
    float v[NPL];
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
        const int e = lane + 64 * i;
        const float x = e < E ? row[e] : NEG;
        v[i] = (x == x) ? x : NEG;           // a NaN logit is never preferred
    }
    uint32_t taken = 0;                       // bit i: this lane's i-th logit is selected
    float my_v = NEG;                         // lane j keeps the j-th winner
    int my_e = 0;
    float vmax = 0.f;
    for (int j = 0; j < k; ++j) {
        float bv = NEG;
        int be = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int e = lane + 64 * i;
            if (e < E && !((taken >> i) & 1u) && better(v[i], e, bv, be)) { bv = v[i]; be = e; }
        }
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) {
            const float ov = __shfl_xor(bv, s);
            const int oe = __shfl_xor(be, s);
            if (better(ov, oe, bv, be)) { bv = ov; be = oe; }
        }
        // every lane now holds the same winner (be < E because k <= E)
        if ((be & 63) == lane) taken |= 1u << (be >> 6);
        if (j == lane) { my_v = bv; my_e = be; }   // k <= 64
        if (j == 0) vmax = bv;
    }
    const bool mine = lane < k;
    float w = mine ? expf(my_v - vmax) : 0.f;
    float den;
    if (mode == 0) {
        den = w;
    } else {
        den = 0.f;
#pragma unroll
        for (int i = 0; i < NPL; ++i)
            if (lane + 64 * i < E) den += expf(v[i] - vmax);
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) den += __shfl_xor(den, s);
    if (mine) {
        topk_idx[(size_t)t * k + lane] = my_e;
        gate[(size_t)t * k + lane] = w / den;
    }
}

// E <= 16*VPL, k <= 16: a token per 16-lane row, PASSES tokens per row.
constexpr int kRowPasses = 4;

template <int VPL>
__global__ __launch_bounds__(256) void route_topk_rows(int T, int E, int k, int mode,
                                                       const float* __restrict__ logits,
                                                       int32_t* __restrict__ topk_idx,
                                                       float* __restrict__ gate) {
    const int g = threadIdx.x & 15;                   // lane inside the row
    const int row = threadIdx.x >> 4;                 // 16 rows per workgroup
    const int t0 = (blockIdx.x * 16 + row) * kRowPasses;
    const float NEG = -__builtin_huge_valf();
    const int e0 = g * VPL;
    float v[kRowPasses][VPL];
#pragma unroll
    for (int p = 0; p < kRowPasses; ++p) {
        const int t = t0 + p;
        const float* src = logits + (size_t)(t < T ? t : 0) * E;
        if (VPL == 4 && E == 64) {                    // 16-byte aligned rows: one vector load per lane
            const float4 q = *reinterpret_cast<const float4*>(src + e0);
            v[p][0] = q.x; v[p][1 % VPL] = q.y; v[p][2 % VPL] = q.z; v[p][3 % VPL] = q.w;
        } else {
#pragma unroll
            for (int i = 0; i < VPL; ++i) v[p][i] = e0 + i < E ? src[e0 + i] : NEG;
        }
    }
#pragma unroll
    for (int p = 0; p < kRowPasses; ++p) {
        const int t = t0 + p;
#pragma unroll
        for (int i = 0; i < VPL; ++i) v[p][i] = (v[p][i] == v[p][i]) ? v[p][i] : NEG;   // a NaN logit is never preferred
        uint32_t taken = 0;
        float my_v = NEG, vmax = 0.f;
        int my_e = 0;
        for (int j = 0; j < k; ++j) {
            float bv = NEG;
            int be = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < VPL; ++i)
                if (e0 + i < E && !((taken >> i) & 1u) && better(v[p][i], e0 + i, bv, be)) { bv = v[p][i]; be = e0 + i; }
#pragma unroll
            for (int s = 8; s > 0; s >>= 1) {
                const float ov = __shfl_xor(bv, s);
                const int oe = __shfl_xor(be, s);
                if (better(ov, oe, bv, be)) { bv = ov; be = oe; }
            }
            // every lane of the row holds the same winner (be < E because k <= E)
            if (be / VPL == g) taken |= 1u << (be - e0);
            if (j == g) { my_v = bv; my_e = be; }
            if (j == 0) vmax = bv;
        }
        const bool mine = g < k;
        const float w = mine ? expf(my_v - vmax) : 0.f;
        float den;
        if (mode == 0) {
            den = w;
        } else {
            den = 0.f;
#pragma unroll
            for (int i = 0; i < VPL; ++i)
                if (e0 + i < E) den += expf(v[p][i] - vmax);
        }
#pragma unroll
        for (int s = 8; s > 0; s >>= 1) den += __shfl_xor(den, s);
        if (mine && t < T) {
            topk_idx[(size_t)t * k + g] = my_e;
            gate[(size_t)t * k + g] = w / den;
        }
    }
}

}  // namespace

extern "C" hexa_status hexa_moe_route(const hexa_moe_shape* shape, const float* logits, int32_t gate_mode,
                                      int32_t* topk_idx, float* gate, void* stream) {
    if (!shape || !logits || !topk_idx || !gate) return HEXA_ERR_NULL;
    const int T = shape->T, E = shape->E, k = shape->k;
    if (T <= 0 || E <= 0 || k <= 0 || (long long)T * k > 0x7fffffffLL || E > 64 * kMaxPerLane)
        return HEXA_ERR_SHAPE;
    if (k > E || k > 64 || (gate_mode != HEXA_GATE_SOFTMAX_SELECTED && gate_mode != HEXA_GATE_SOFTMAX_ALL))
        return HEXA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(ceil_div(T, 4)), block(256);
    ProfScope ps(st, "route");
    if (E <= 64 && k <= 16) {
        const dim3 grid_rows(ceil_div(T, 16 * kRowPasses));
        const int vpl = ceil_div(E, 16);
        if (vpl <= 1) hipLaunchKernelGGL(route_topk_rows<1>, grid_rows, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
        else if (vpl <= 2) hipLaunchKernelGGL(route_topk_rows<2>, grid_rows, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
        else hipLaunchKernelGGL(route_topk_rows<4>, grid_rows, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
        return hipGetLastError() == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE;
    }
    const int npl = ceil_div(E, 64);
    if (npl <= 1) hipLaunchKernelGGL(route_topk<1>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    else if (npl <= 2) hipLaunchKernelGGL(route_topk<2>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    else if (npl <= 4) hipLaunchKernelGGL(route_topk<4>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    else hipLaunchKernelGGL(route_topk<kMaxPerLane>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    return hipGetLastError() == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE;
}

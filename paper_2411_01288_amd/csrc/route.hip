// Router front-end: top-k selection over a token's E logits and the gate weights, i.e. the step
// that produces the routing choice {R_j(x)} the expert-specific operators take as input (HEXA-MoE
// Sec. 3.1; App. B Table 5).  The paper treats the router as given; the rule here is the usual one:
// the k largest logits, equal logits to the lower expert id, slots in descending order of logit,
// gates = softmax over the selected logits (or the full softmax evaluated at them).
//
// One 64-lane wavefront per token, lane l holding logits l, l+64, ... (E <= 1024).  Each of the k
// rounds is a wavefront arg-max over (logit, -expert id) by xor-shuffles; selection uses
// comparisons only, so the indices are bit-exact whatever the float environment.  HBM-bound:
// T*E*4 bytes in, T*k*8 out (33.5 MB at T = 131072, E = 64).
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
    const int npl = ceil_div(E, 64);
    if (npl <= 1) hipLaunchKernelGGL(route_topk<1>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    else if (npl <= 2) hipLaunchKernelGGL(route_topk<2>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    else if (npl <= 4) hipLaunchKernelGGL(route_topk<4>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    else hipLaunchKernelGGL(route_topk<kMaxPerLane>, grid, block, 0, st, T, E, k, gate_mode, logits, topk_idx, gate);
    return hipGetLastError() == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE;
}

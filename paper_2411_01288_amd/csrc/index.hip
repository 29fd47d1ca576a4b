// Re-index build (HEXA-MoE Sec. 3.2; App. B Alg. 1), redesigned for CDNA4.
//
// The paper scatters token ids with one global atomicAdd per token, which makes
// the order inside an expert's segment depend on scheduling.  Here the result is
// the unique stable counting sort of the flat assignment ids, built without any
// order-dependent atomic:
//   1. index_count   each wavefront owns a contiguous run of ids and histograms
//                    it in LDS (integer adds commute, so the counts are exact);
//   2. index_scan    one workgroup turns the [chunk][expert] histogram into
//                    counts, offsets and, per chunk and expert, the first output
//                    position (expert-major, chunk-minor exclusive scan);
//   3. index_scatter each wavefront re-reads its run 64 ids at a time; the rank
//                    of an id among equal experts in its row comes from
//                    ballot + popcount of the lower lanes, rows are chained
//                    through a per-wave LDS cursor.
// Segments carry no padding: tiles are cut per segment by the consumers.
#include "common.h"

#include <mutex>

namespace {

constexpr int kWavesPerWg = 4;
constexpr int kMaxChunks = 1024;

struct IndexPlan { int rows_per_wave, nchunks; };

IndexPlan plan_for(int A) {
    IndexPlan p;
    p.rows_per_wave = (A + 64 * kMaxChunks - 1) / (64 * kMaxChunks);
    if (p.rows_per_wave < 1) p.rows_per_wave = 1;
    p.nchunks = (A + 64 * p.rows_per_wave - 1) / (64 * p.rows_per_wave);
    return p;
}

__global__ __launch_bounds__(256) void index_count(const int32_t* __restrict__ idx, int A, int E,
                                                   int R, int nchunks, int32_t* __restrict__ hist) {
    extern __shared__ int32_t lh[];  // [4][E]
    for (int i = threadIdx.x; i < kWavesPerWg * E; i += 256) lh[i] = 0;
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * kWavesPerWg + wave;
    if (chunk < nchunks) {
        const int a0 = chunk * 64 * R;
        for (int r = 0; r < R; ++r) {
            const int a = a0 + r * 64 + lane;
            if (a < A) {
                const int e = idx[a];
                if ((unsigned)e < (unsigned)E) atomicAdd(&lh[wave * E + e], 1);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kWavesPerWg * E; i += 256) {
        const int c = blockIdx.x * kWavesPerWg + i / E;
        if (c < nchunks) hist[(size_t)c * E + i % E] = lh[i];
    }
}

// hist[c][e] (counts) -> hist[c][e] (first output position of chunk c's ids of expert e)
__global__ __launch_bounds__(1024) void index_scan(int32_t* __restrict__ hist, int E, int nchunks,
                                                   int32_t* __restrict__ counts,
                                                   int32_t* __restrict__ offsets) {
    __shared__ int32_t gs[1024];   // [G][E] group sums, then exclusive group bases
    __shared__ int32_t cnt[1024];  // counts, then offsets
    const int G = max(1, 1024 / E);
    const int cpg = ceil_div(nchunks, G);
    const int t = threadIdx.x;
    const int e = t % E, g = t / E;
    const bool active = g < G;
    const int c0 = g * cpg, c1 = min(nchunks, c0 + cpg);
    // (both passes over this thread's chunks go eight loads at a time: one at a time, the kernel is
    // a chain of memory latencies)
    int s = 0;
    if (active) {
        for (int c = c0; c < c1; c += 8) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = c + u < c1 ? hist[(size_t)(c + u) * E + e] : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
    }
    if (active) gs[g * E + e] = s;
    __syncthreads();
    int base = 0;
    if (active) {
        for (int q = 0; q < g; ++q) base += gs[q * E + e];
        if (g == 0) {
            int tot = 0;
            for (int q = 0; q < G; ++q) tot += gs[q * E + e];
            cnt[e] = tot;
            counts[e] = tot;
        }
    }
    __syncthreads();
    int off = 0, mine = 0;
    if (t < E) {
        for (int q = 0; q < t; ++q) off += cnt[q];
        mine = cnt[t];
    }
    __syncthreads();
    if (t < E) {
        cnt[t] = off;
        offsets[t] = off;
        if (t == E - 1) offsets[E] = off + mine;
    }
    __syncthreads();
    if (active) {
        int run = cnt[e] + base;
        for (int c = c0; c < c1; c += 8) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = c + u < c1 ? hist[(size_t)(c + u) * E + e] : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (c + u < c1) hist[(size_t)(c + u) * E + e] = run;
                run += v[u];
            }
        }
    }
}

__global__ __launch_bounds__(256) void index_scatter(const int32_t* __restrict__ idx, int A, int E,
                                                     int R, int nchunks,
                                                     const int32_t* __restrict__ hist,
                                                     const int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ perm,
                                                     int32_t* __restrict__ inv) {
    extern __shared__ int32_t lraw[];  // [4][E] cursors
    volatile int32_t* lb = lraw;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * kWavesPerWg + wave;
    for (int i = threadIdx.x; i < kWavesPerWg * E; i += 256) {
        const int c = blockIdx.x * kWavesPerWg + i / E;
        lraw[i] = c < nchunks ? hist[(size_t)c * E + i % E] : 0;
    }
    __syncthreads();
    if (chunk >= nchunks) return;
    const int n_valid = offsets[E];
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const int a0 = chunk * 64 * R;
    for (int r = 0; r < R; ++r) {
        const int a = a0 + r * 64 + lane;
        int e = -1;
        if (a < A) e = idx[a];
        const bool valid = (a < A) && ((unsigned)e < (unsigned)E);
        uint64_t remaining = __ballot(valid);
        int rank = 0, cnt = 0;
        while (remaining) {  // uniform: one trip per distinct expert in this row
            const int leader = __ffsll((long long)remaining) - 1;
            const int e0 = __shfl(e, leader);
            const uint64_t m = __ballot(valid && e == e0);
            if (valid && e == e0) {
                rank = __popcll(m & lt_mask);
                cnt = __popcll(m);
            }
            remaining &= ~m;
        }
        int b = 0;
        if (valid) b = lb[wave * E + e];
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            const int pos = b + rank;
            perm[pos] = a;
            inv[a] = pos;
            if (rank == cnt - 1) lb[wave * E + e] = b + cnt;
        } else if (a < A) {
            inv[a] = -1;  // dropped: expert id outside [0, E)
        }
        if (a < A && a >= n_valid) perm[a] = -1;  // tail left empty by dropped ids
        __builtin_amdgcn_wave_barrier();
    }
}

// The paper's padded form of the index (App. B Alg. 1; Sec. 3.2), derived from the unpadded one:
// expert e's sub-vector starts at idx_[e] = sum over e' < e of ceil(n_e' / blk) * blk and holds its
// perm entries followed by -1 up to the next multiple of blk; entries past idx_[E] are -1 too.
// Two launches: the padded starts (one workgroup, E <= 1024 threads), then one thread per entry
// of v, which finds its expert by bisection over the padded starts.
__global__ __launch_bounds__(1024) void padded_starts(const int32_t* __restrict__ offsets, int E, int blk,
                                                      int32_t* __restrict__ idx_) {
    __shared__ int s[1024];
    const int e = threadIdx.x;
    const int n = e < E ? offsets[e + 1] - offsets[e] : 0;
    const int padded = ceil_div(n, blk) * blk;
    s[e] = padded;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {     // inclusive scan
        const int v = e >= off ? s[e - off] : 0;
        __syncthreads();
        s[e] += v;
        __syncthreads();
    }
    if (e < E) idx_[e + 1] = s[e];
    if (e == 0) idx_[0] = 0;
}

__global__ __launch_bounds__(256) void padded_fill(const int32_t* __restrict__ offsets,
                                                   const int32_t* __restrict__ perm,
                                                   const int32_t* __restrict__ idx_, int E, long long cap,
                                                   int32_t* __restrict__ v) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= cap) return;
    int out = -1;
    if (i < idx_[E]) {
        int lo = 0, hi = E;                         // largest e with idx_[e] <= i
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (idx_[mid] <= i) lo = mid; else hi = mid;
        }
        const int r = (int)(i - idx_[lo]);
        if (r < offsets[lo + 1] - offsets[lo]) out = perm[offsets[lo] + r];
    }
    v[i] = out;
}

}  // namespace

hipError_t launch_padded_index(const MoeDims& D, const hexa_moe_idx& idx, int blk, long long cap,
                               int32_t* v, int32_t* idx_, hipStream_t st) {
    ProfScope ps(st, "padded_index");
    hipLaunchKernelGGL(padded_starts, dim3(1), dim3(1024), 0, st, idx.offsets, D.E, blk, idx_);
    hipLaunchKernelGGL(padded_fill, dim3((unsigned)((cap + 255) / 256)), dim3(256), 0, st, idx.offsets,
                       idx.perm, idx_, D.E, cap, v);
    return hipGetLastError();
}

size_t index_scratch_bytes(const MoeDims& D) {
    const IndexPlan p = plan_for(D.A);
    return align_up((size_t)p.nchunks * D.E * sizeof(int32_t), 256);
}

hipError_t launch_index(const MoeDims& D, const int32_t* topk_idx, hexa_moe_idx out, void* scratch,
                        hipStream_t st) {
    const IndexPlan p = plan_for(D.A);
    int32_t* hist = (int32_t*)scratch;
    const int nwg = ceil_div(p.nchunks, kWavesPerWg);
    const size_t lds = (size_t)kWavesPerWg * D.E * sizeof(int32_t);
    { ProfScope ps(st, "index_count");
    hipLaunchKernelGGL(index_count, dim3(nwg), dim3(256), lds, st, topk_idx, D.A, D.E,
                       p.rows_per_wave, p.nchunks, hist); }
    { ProfScope ps(st, "index_scan");
    hipLaunchKernelGGL(index_scan, dim3(1), dim3(1024), 0, st, hist, D.E, p.nchunks, out.counts,
                       out.offsets); }
    { ProfScope ps(st, "index_scatter");
    hipLaunchKernelGGL(index_scatter, dim3(nwg), dim3(256), lds, st, topk_idx, D.A, D.E,
                       p.rows_per_wave, p.nchunks, hist, out.offsets, out.perm, out.inv); }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// hexa_moe_index_static: the same three kernels with the chunk histogram in a fixed array of
// device memory that belongs to the library, for callers that cannot allocate (no hipMalloc under
// stream capture, tight serving loops).  Nothing here allocates or frees.
// ---------------------------------------------------------------------------------------------
namespace {

// One copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[HEXA_INDEX_STATIC_SCRATCH_BYTES];

std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up on first use

// The address of this device's copy of the array (the device must be current).
hipError_t static_scratch(void** out) {
    int d = -1;
    hipError_t e = hipGetDevice(&d);
    if (e != hipSuccess) return e;
    if (d < 0 || d >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[d]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[d] = p;
    }
    *out = g_scratch_ptr[d];
    return hipSuccess;
}

}  // namespace

extern "C" hexa_status hexa_moe_index_static(const hexa_moe_shape* shape, const int32_t* topk_idx,
                                             hexa_moe_idx out, void* stream) {
    MoeDims D;
    const hexa_status s = hexa_check_shape(shape, &D);
    if (s != HEXA_OK) return s;
    if (!topk_idx || !out.counts || !out.offsets || !out.perm || !out.inv) return HEXA_ERR_NULL;
    if (index_scratch_bytes(D) > (size_t)HEXA_INDEX_STATIC_SCRATCH_BYTES) return HEXA_ERR_WORKSPACE;
    void* ptr = nullptr;
    if (static_scratch(&ptr) != hipSuccess) return HEXA_ERR_DEVICE;
    // index_count overwrites every histogram entry the later kernels read, so what an earlier
    // call left in the array needs no clearing
    return launch_index(D, topk_idx, out, ptr, (hipStream_t)stream) == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE;
}

// Bandwidth-bound steps around the contractions:
//   combine_y      y_t  = sum_j gate[t,j] * o[inv[t*k+j]]          (top-k sum of App. B Table 5 row 3,
//                                                                    done as a gather in fixed slot order
//                                                                    instead of the paper's atomicAdd)
//   bwd_prologue   do_p = gate_a * dY_t  (a = perm[p]) ; dgate_a = <dY_t, o_p> ; db2 partials
//   combine_dx     dx_t = sum_j dxp[inv[t*k+j]]                     (Table 5 row 10, sum over the k slots)
//   segment_colsum ESS (Sec. 3.1 item 2; App. B Alg. 3): per-expert column sums of a perm-ordered
//                  matrix, in two deterministic stages so a long segment is spread over the chip.
#include "common.h"

namespace {

template <typename T> struct Vec;   // 16-byte vector access of 4 floats or 8 bf16
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, float (&v)[4]) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    __device__ static void store(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, float (&v)[8]) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static void store(bf16_t* p, const float (&v)[8]) {
        uint4 q;
        q.x = pack_bf2(v[0], v[1]); q.y = pack_bf2(v[2], v[3]);
        q.z = pack_bf2(v[4], v[5]); q.w = pack_bf2(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = q;
    }
};

template <> struct Vec<f16_t> {
    static constexpr int N = 8;
    __device__ static void load(const f16_t* p, float (&v)[8]) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) unpack2<true>(w[i], v[2 * i], v[2 * i + 1]);
    }
    __device__ static void store(f16_t* p, const float (&v)[8]) {
        uint4 q;
        q.x = pack_h2(v[0], v[1]); q.y = pack_h2(v[2], v[3]);
        q.z = pack_h2(v[4], v[5]); q.w = pack_h2(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = q;
    }
};

// One thread per VN consecutive columns of one token.  d % VN == 0.
template <typename T>
__global__ __launch_bounds__(256) void combine_rows(int T_, int d, int k,
                                                    const T* __restrict__ src,
                                                    const int32_t* __restrict__ inv,
                                                    const float* __restrict__ gate,  // NULL: plain sum
                                                    T* __restrict__ dst) {
    constexpr int VN = Vec<T>::N;
    const int per_row = d / VN;
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (gid >= (long long)T_ * per_row) return;
    const int t = (int)(gid / per_row);
    const int c = (int)(gid % per_row) * VN;
    float acc[VN];
#pragma unroll
    for (int i = 0; i < VN; ++i) acc[i] = 0.f;
    for (int j = 0; j < k; ++j) {
        const int p = inv[(size_t)t * k + j];
        if (p < 0) continue;  // dropped assignment
        const float g = gate ? gate[(size_t)t * k + j] : 1.f;
        float v[VN];
        Vec<T>::load(src + (size_t)p * d + c, v);
#pragma unroll
        for (int q = 0; q < VN; ++q) acc[q] += g * v[q];
    }
    Vec<T>::store(dst + (size_t)t * d + c, acc);
}

// Tail columns when d is not a multiple of the vector width (fp32 path with odd sizes).
template <typename T>
__global__ __launch_bounds__(256) void combine_rows_scalar(int T_, int d, int k,
                                                           const T* __restrict__ src,
                                                           const int32_t* __restrict__ inv,
                                                           const float* __restrict__ gate,
                                                           T* __restrict__ dst) {
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (gid >= (long long)T_ * d) return;
    const int t = (int)(gid / d), c = (int)(gid % d);
    float acc = 0.f;
    for (int j = 0; j < k; ++j) {
        const int p = inv[(size_t)t * k + j];
        if (p < 0) continue;
        const float g = gate ? gate[(size_t)t * k + j] : 1.f;
        acc += g * Elem<T>::ld(src + (size_t)p * d + c);
    }
    Elem<T>::st(dst + (size_t)t * d + c, acc);
}

// One wavefront per perm row p.
template <typename T>
__global__ __launch_bounds__(256) void bwd_prologue(int A, int d, int k, const T* __restrict__ dY,
                                                    const T* __restrict__ o,
                                                    const int32_t* __restrict__ perm,
                                                    const int32_t* __restrict__ offsets, int E,
                                                    const float* __restrict__ gate,
                                                    T* __restrict__ dout, float* __restrict__ dgate) {
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= A) return;
    const int n_valid = offsets[E];
    if (p >= n_valid) {  // rows past the last segment exist only when ids were dropped
        for (int c = lane; c < d; c += 64) Elem<T>::st(dout + (size_t)p * d + c, 0.f);
        return;
    }
    const int a = perm[p];
    const int t = a / k;
    const float g = gate[a];
    const T* src = dY + (size_t)t * d;
    const T* orow = o + (size_t)p * d;
    T* dst = dout + (size_t)p * d;
    float dot = 0.f;
    constexpr int VN = Vec<T>::N;
    if (d % VN == 0) {
        for (int c = lane * VN; c < d; c += 64 * VN) {
            float v[VN], w[VN], ov[VN];
            Vec<T>::load(src + c, v);
            Vec<T>::load(orow + c, ov);
#pragma unroll
            for (int q = 0; q < VN; ++q) dot += v[q] * ov[q];
#pragma unroll
            for (int q = 0; q < VN; ++q) w[q] = g * v[q];
            Vec<T>::store(dst + c, w);
        }
    } else {
        for (int c = lane; c < d; c += 64) {
            const float v = Elem<T>::ld(src + c);
            dot += v * Elem<T>::ld(orow + c);
            Elem<T>::st(dst + c, g * v);
        }
    }
    if (dgate) {
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) dot += __shfl_xor(dot, s);
        if (lane == 0) dgate[a] = dot;
    }
}

__global__ void fill_zero_f32(float* p, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// Stage 1: one workgroup per (128-row segment tile, 256-column block): each thread owns one column
// pair-free scalar column and walks the rows in order -> partial[tile][col].
constexpr int kColsumRows = 128;

template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1(const T* __restrict__ src, int ncols, int E,
                                                     const int32_t* __restrict__ offsets,
                                                     float* __restrict__ partial) {
    const SegTile s = seg_tile_find(offsets, E, kColsumRows, blockIdx.x);
    if (s.e < 0) return;
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= ncols) return;
    float acc = 0.f;
    const T* p = src + (size_t)s.row0 * ncols + c;
    for (int r = 0; r < s.rows; ++r) acc += Elem<T>::ld(p + (size_t)r * ncols);
    partial[(size_t)blockIdx.x * ncols + c] = acc;
}

// Stage 2: out[e][c] = sum of the expert's partial rows (exact 0 for an empty expert).  The expert's
// tiles (tile height bm, `parts` partial rows per tile) hold rows first*parts .. (first+nt)*parts - 1
// of `partial`.  A workgroup is 256 columns x up to 16 slices (a lane owns four columns, 64 apart):
// slice s adds up a contiguous share of the rows in order, and the slice sums are added in slice
// order, so the result does not depend on scheduling; one thread per column walking all rows alone
// was a chain of up to 800 dependent memory latencies for a large expert.
constexpr int kFinishSlices = 16;   // at most (the launch picks 64 * slices threads)
__global__ __launch_bounds__(64 * kFinishSlices) void colsum_finish(const float* __restrict__ partial, int ncols,
                                                     int E, int bm, int parts,
                                                     const int32_t* __restrict__ offsets,
                                                     float* __restrict__ out) {
    __shared__ float part[kFinishSlices][256];
    const int e = blockIdx.x;
    const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int c0 = blockIdx.y * 256 + lane;
    int first = 0;
    for (int q = 0; q < e; ++q) first += ceil_div(offsets[q + 1] - offsets[q], bm);
    const int nrows = ceil_div(offsets[e + 1] - offsets[e], bm) * parts;
    // as many slices as give each at least eight rows (a function of the expert's row count only)
    const int nsl = min((int)blockDim.x / 64, max(1, nrows / 8));
    const int per = ceil_div(nrows, nsl);
    const int r0 = min(nrows, slice * per), r1 = min(nrows, r0 + per);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const float* src = partial + (size_t)first * parts * ncols;
    for (int i = r0; i < r1; i += 4) {
        float v[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                v[u][q] = (i + u < r1 && c0 + 64 * q < ncols) ? src[(size_t)(i + u) * ncols + c0 + 64 * q] : 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] += v[u][q];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) part[slice][lane + 64 * q] = acc[q];
    __syncthreads();
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (threadIdx.x < 256 && c < ncols) {
        float sum = part[0][threadIdx.x];
        for (int q = 1; q < nsl; ++q) sum += part[q][threadIdx.x];
        out[(size_t)e * ncols + c] = sum;
    }
}

// Slices per workgroup of colsum_finish: many when an expert has many partial rows on average (small
// tiles, few experts), few when it has few: wide workgroups with mostly idle wavefronts cost more
// than they save there.
inline int finish_slices(size_t partial_rows, int E) {
    return partial_rows / (size_t)E >= 64 ? kFinishSlices : 4;
}

// Backward prologue and the fc2 bias gradient in one pass (ESS, Sec. 3.1 item 2; Table 5 row 4):
// one workgroup per segment tile of tile_rows <= 128 rows; a thread owns VN consecutive columns (256*VN columns per
// sweep) and walks the tile's rows in order, so the column sums of do = gate * dY (unrounded) stay
// in registers and go to partial[tile][col] for colsum_finish.  Per row it also writes
// dout_p = round(do) and accumulates <dY_t, o_p> (wave sums meet in LDS, added in wave
// order).  Workgroups past the last tile zero the rows past the last segment (they exist only
// when expert ids were dropped).  d % VN == 0.
template <typename T>
__global__ __launch_bounds__(256) void bwd_prologue_tiles(int A, int d, int k, const T* __restrict__ dY,
                                                          const T* __restrict__ o,
                                                          const int32_t* __restrict__ perm,
                                                          const int32_t* __restrict__ offsets, int E,
                                                          const float* __restrict__ gate,
                                                          T* __restrict__ dout, float* __restrict__ dgate,
                                                          float* __restrict__ partial, int tile_rows) {
    constexpr int VN = Vec<T>::N;
    __shared__ float sdot[kColsumRows][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SegTile s = seg_tile_find(offsets, E, tile_rows, blockIdx.x);
    if (s.e < 0) {
        const int ntiles = seg_tiles_total(offsets, E, tile_rows);
        const long long r0 = (long long)offsets[E] + (long long)(blockIdx.x - ntiles) * tile_rows;
        float z[VN];
#pragma unroll
        for (int q = 0; q < VN; ++q) z[q] = 0.f;
        for (long long r = r0; r < r0 + tile_rows && r < A; ++r)
            for (int c = tid * VN; c < d; c += 256 * VN) Vec<T>::store(dout + (size_t)r * d + c, z);
        return;
    }
    for (int c0 = 0; c0 < d; c0 += 256 * VN) {
        const int c = c0 + tid * VN;
        const bool act = c < d;
        float cs[VN];
#pragma unroll
        for (int q = 0; q < VN; ++q) cs[q] = 0.f;
        for (int r = 0; r < s.rows; ++r) {
            const int p = s.row0 + r;
            const int a = perm[p];
            const int t = a / k;
            const float g = gate[a];
            float dot = 0.f;
            if (act) {
                float v[VN], ov[VN], w[VN];
                Vec<T>::load(dY + (size_t)t * d + c, v);
                Vec<T>::load(o + (size_t)p * d + c, ov);
#pragma unroll
                for (int q = 0; q < VN; ++q) {
                    dot += v[q] * ov[q];
                    w[q] = g * v[q];
                    cs[q] += w[q];
                }
                Vec<T>::store(dout + (size_t)p * d + c, w);
            }
            if (dgate) {
#pragma unroll
                for (int sh = 32; sh > 0; sh >>= 1) dot += __shfl_xor(dot, sh);
                if (lane == 0) sdot[r][wave] = (c0 == 0 ? 0.f : sdot[r][wave]) + dot;
            }
        }
        if (act) {
            float* dst = partial + (size_t)blockIdx.x * d + c;
#pragma unroll
            for (int q = 0; q < VN; q += 4)
                *reinterpret_cast<float4*>(dst + q) = make_float4(cs[q], cs[q + 1], cs[q + 2], cs[q + 3]);
        }
    }
    if (dgate) {
        __syncthreads();
        if (tid < s.rows)
            dgate[perm[s.row0 + tid]] = ((sdot[tid][0] + sdot[tid][1]) + sdot[tid][2]) + sdot[tid][3];
    }
}

template <typename T>
hipError_t combine_impl(int T_, int d, int k, const T* src, const int32_t* inv,
                        const float* gate, T* dst, hipStream_t st) {
    ProfScope ps(st, gate ? "combine_y" : "combine_dx");
    constexpr int VN = Vec<T>::N;
    if (d % VN == 0) {
        const long long n = (long long)T_ * (d / VN);
        hipLaunchKernelGGL(combine_rows<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, T_,
                           d, k, src, inv, gate, dst);
    } else {
        const long long n = (long long)T_ * d;
        hipLaunchKernelGGL(combine_rows_scalar<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                           st, T_, d, k, src, inv, gate, dst);
    }
    return hipGetLastError();
}

}  // namespace

// Rows per workgroup of the fused backward prologue: 128 when that still gives ~2048 workgroups,
// fewer (down to 8) on small problems, where a workgroup's serial walk over its rows would
// otherwise be the whole run time.
int bwd_prologue_tile_rows(const MoeDims& D) {
    int r = kColsumRows;
    while (r > 8 && D.A / r < 2048) r >>= 1;
    return r;
}
// Rows of the column-sum staging buffer that the prologue and the two-stage column sums need.
size_t colsum_partial_rows(const MoeDims& D) {
    return (size_t)(D.A / bwd_prologue_tile_rows(D) + D.E + 1);
}

template <typename T>
hipError_t launch_combine_y(const MoeDims& D, const T* o, const int32_t* inv, const float* gate,
                            T* y, hipStream_t st) {
    return combine_impl<T>(D.T, D.d, D.k, o, inv, gate, y, st);
}

template <typename T>
hipError_t launch_combine_dx(const MoeDims& D, const T* dxp, const int32_t* inv, T* dx,
                             hipStream_t st) {
    return combine_impl<T>(D.T, D.d, D.k, dxp, inv, nullptr, dx, st);
}

template <typename T>
hipError_t launch_bwd_prologue(const MoeDims& D, const T* dY, const T* o,
                               const int32_t* perm, const int32_t* offsets, const float* gate,
                               T* dout, float* dgate, float* partial, float* db2, hipStream_t st) {
    if (dgate) {  // dropped assignments keep a defined (zero) gate gradient
        ProfScope ps(st, "dgate_zero");
        const size_t n = (size_t)D.A;
        hipLaunchKernelGGL(fill_zero_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dgate, n);
    }
    if (D.d % Vec<T>::N == 0) {
        const int R = bwd_prologue_tile_rows(D);
        {
            ProfScope ps(st, "bwd_prologue");
            hipLaunchKernelGGL(bwd_prologue_tiles<T>, dim3(D.A / R + D.E + 1), dim3(256), 0, st, D.A, D.d,
                               D.k, dY, o, perm, offsets, D.E, gate, dout, dgate, partial, R);
        }
        ProfScope ps(st, "colsum_db2");
        hipLaunchKernelGGL(colsum_finish, dim3(D.E, ceil_div(D.d, 256)), dim3(64 * finish_slices((size_t)D.A / R + D.E, D.E)), 0, st, partial, D.d,
                           D.E, R, 1, offsets, db2);
        return hipGetLastError();
    }
    {
        ProfScope ps(st, "bwd_prologue");
        hipLaunchKernelGGL(bwd_prologue<T>, dim3(ceil_div(D.A, 4)), dim3(256), 0, st, D.A, D.d, D.k, dY,
                           o, perm, offsets, D.E, gate, dout, dgate);
    }
    return launch_segment_colsum<T>(D, dout, D.d, offsets, partial, db2, st);
}

template <typename T>
hipError_t launch_segment_colsum(const MoeDims& D, const T* src, int ncols, const int32_t* offsets,
                                 float* partial, float* out, hipStream_t st) {
    const int max_tiles = D.A / kColsumRows + D.E;
    const int cb = ceil_div(ncols, 256);
    ProfScope ps(st, ncols == D.d ? "colsum_db2" : "colsum_db1");
    hipLaunchKernelGGL(colsum_stage1<T>, dim3(max_tiles, cb), dim3(256), 0, st, src, ncols, D.E,
                       offsets, partial);
    hipLaunchKernelGGL(colsum_finish, dim3(D.E, ceil_div(ncols, 256)), dim3(64 * finish_slices((size_t)D.A / kColsumRows + D.E, D.E)), 0, st, partial, ncols, D.E,
                       kColsumRows, 1, offsets, out);
    return hipGetLastError();
}

hipError_t launch_tile_colsum_finish(const MoeDims& D, const float* partial, int ncols,
                                     const int32_t* offsets, float* out, hipStream_t st) {
    ProfScope ps(st, "colsum_db1");
    hipLaunchKernelGGL(colsum_finish, dim3(D.E, ceil_div(ncols, 256)), dim3(64 * finish_slices(((size_t)D.A / gemm_row_tile() + D.E) * gemm_colpart_rows_per_tile(), D.E)), 0, st, partial, ncols,
                       D.E, gemm_row_tile(), gemm_colpart_rows_per_tile(), offsets, out);
    return hipGetLastError();
}

#define INSTANTIATE(T)                                                                              \
    template hipError_t launch_combine_y<T>(const MoeDims&, const T*, const int32_t*,              \
                                            const float*, T*, hipStream_t);                        \
    template hipError_t launch_combine_dx<T>(const MoeDims&, const T*, const int32_t*, T*,         \
                                             hipStream_t);                                         \
    template hipError_t launch_bwd_prologue<T>(const MoeDims&, const T*,                           \
                                               const T*, const int32_t*, const int32_t*,           \
                                               const float*, T*, float*, float*, float*,           \
                                               hipStream_t);                                       \
    template hipError_t launch_segment_colsum<T>(const MoeDims&, const T*, int, const int32_t*,    \
                                                 float*, float*, hipStream_t);
INSTANTIATE(float)
INSTANTIATE(bf16_t)
INSTANTIATE(f16_t)

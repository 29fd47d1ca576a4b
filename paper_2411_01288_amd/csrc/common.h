// Shared device helpers and the internal launcher interface of libhexa_moe.
// gfx950 (CDNA4) only: 64-wide wavefronts, bf16 / fp16 MFMA, 160 KB LDS per CU.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/hexa_moe.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round-to-nearest-even; gfx950 lowers this cast to v_cvt_pk_bf16_f32
__device__ __forceinline__ bf16_t f2bf(float f) {
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// two floats -> two bf16 (round to nearest even) in one word: a single v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

typedef _Float16 f16_t;   // IEEE binary16

// two floats -> two fp16 (round to nearest even) in one word
__device__ __forceinline__ uint32_t pack_h2(float lo, float hi) {
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}
// one word of two 16-bit values -> two floats
template <bool F16>
__device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    if constexpr (F16) {
        typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
        const f16x2_t h = __builtin_bit_cast(f16x2_t, w);
        lo = (float)h[0]; hi = (float)h[1];
    } else {
        lo = __uint_as_float(w << 16); hi = __uint_as_float(w & 0xffff0000u);
    }
}
template <bool F16>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    if constexpr (F16) return pack_h2(lo, hi);
    else return pack_bf2(lo, hi);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    __device__ static float ld(const float* p) { return *p; }
    __device__ static void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    __device__ static float ld(const bf16_t* p) { return bf2f(*p); }
    __device__ static void st(bf16_t* p, float v) { *p = f2bf(v); }
};
template <> struct Elem<f16_t> {
    __device__ static float ld(const f16_t* p) { return (float)*p; }
    __device__ static void st(f16_t* p, float v) { *p = (f16_t)v; }
};

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// GELU, tanh form (the activation F between the two MLPs; App. B Table 5 rows 2, 7).
#define HEXA_GELU_C 0.7978845608028654f
#define HEXA_GELU_A 0.044715f

// A segment tile: `rows` (<= BM) consecutive rows of perm order that all belong
// to expert `e`, starting at perm position `row0`.
struct SegTile { int e, row0, rows; };

// Number of BM-row tiles over all expert segments (each segment tiled on its own,
// so no tile straddles two experts and none is padded to a capacity).
__device__ __forceinline__ int seg_tiles_total(const int32_t* __restrict__ offsets, int E, int BM) {
    int total = 0;
    for (int e = 0; e < E; ++e) total += ceil_div(offsets[e + 1] - offsets[e], BM);
    return total;
}

// Map tile number `tile` (0-based over all segments, expert-major) to its segment tile.
// Returns e = -1 when `tile` is past the last one.
__device__ __forceinline__ SegTile seg_tile_find(const int32_t* __restrict__ offsets, int E, int BM,
                                                 int tile) {
    SegTile s{-1, 0, 0};
    int acc = 0;
    for (int e = 0; e < E; ++e) {
        const int b = offsets[e], n = offsets[e + 1] - b;
        const int nt = ceil_div(n, BM);
        if (tile < acc + nt) {
            const int r0 = (tile - acc) * BM;
            s.e = e; s.row0 = b + r0; s.rows = min(BM, n - r0);
            return s;
        }
        acc += nt;
    }
    return s;
}

// ---- optional per-kernel timing (off unless hexa_moe_profile_enable(1); bench_support.hip) ----
// A ProfScope brackets one kernel launch with two HIP events on the launch stream.
void prof_begin(hipStream_t st, const char* label);
void prof_end(hipStream_t st, const char* label);
struct ProfScope {
    hipStream_t st;
    const char* label;
    ProfScope(hipStream_t s, const char* l) : st(s), label(l) { prof_begin(s, l); }
    ~ProfScope() { prof_end(st, label); }
};

// ---- internal launchers (one per translation unit), all asynchronous on `st` ----
struct MoeDims { int T, d, f, E, k, A, act; };

// Host-side validation of a shape (sizes, dtype, activation, the size rules of the 16-bit path);
// fills D on HEXA_OK.  Touches no device.
hexa_status hexa_check_shape(const hexa_moe_shape* s, MoeDims* D);

constexpr int kMaxDevices = 64;   // per-device state of the library is kept in arrays of this length

// Sets the launch attributes of every contraction kernel (160 KB of dynamic LDS) on the current
// device.  Called once per device by the entry points, outside any stream capture.
hipError_t gemm_bf16_device_init();

// saved + staging regions inside the caller's workspace (device pointers)
struct MoeWorkspace {
    void* pre;      // [A,f] elem   fp32: pre-activations; bf16: GELU'(pre), perm order (saved by fwd)
    void* h;        // [A,f] elem   activations, perm order            (saved by fwd)
    void* o;        // [A,d] elem   per-assignment expert outputs      (saved by fwd)
    void* dout;     // [A,d] elem   gate * dY gathered to perm order   (bwd staging)
    void* dpre;     // [A,f] elem                                       (bwd staging)
    void* dxp;      // [A,d] elem   per-assignment input gradients     (bwd staging)
    uint32_t* rowoff; // [A + 64 E]  byte offsets in x of the token rows, in the order WGRAD1 fetches them (16-bit path; bwd staging)
    float* colpart; // [rows, max(d,f)] f32 partial column sums          (bwd staging)
    float* kpart;   // split-K partial weight-gradient tiles           (bwd staging)
    size_t kpart_slots;
    int32_t* worklist; // row tiles and token-contraction items of the bf16 kernels (saved by fwd, read by bwd)
    size_t total_bytes;
};

int gemm_row_tile();                 // rows of a bf16 row-GEMM tile
int gemm_colpart_rows_per_tile();    // DGRAD2 writes this many column-sum partial rows per row tile
int wgrad_chunk_len(const MoeDims& D);          // tokens per split-K chunk (host policy)
size_t wgrad_max_slots(const MoeDims& D);
size_t gemm_worklist_ints(const MoeDims& D);
int bwd_prologue_tile_rows(const MoeDims& D);   // rows per workgroup of the fused backward prologue
size_t colsum_partial_rows(const MoeDims& D);   // rows of MoeWorkspace::colpart the column sums need    // int32 entries of MoeWorkspace::worklist

hipError_t launch_index(const MoeDims& D, const int32_t* topk_idx, hexa_moe_idx out, void* scratch,
                        hipStream_t st);
size_t index_scratch_bytes(const MoeDims& D);
hipError_t launch_padded_index(const MoeDims& D, const hexa_moe_idx& idx, int blk, long long cap,
                               int32_t* v, int32_t* idx_, hipStream_t st);

template <typename T>
hipError_t launch_combine_y(const MoeDims& D, const T* o, const int32_t* inv, const float* gate,
                            T* y, hipStream_t st);
// dout_p = gate_a dY_t, dgate_a = <dY_t, o_p>, for a = perm[p], and
// db2[e] = sum over the expert's rows of gate_a dY_t (ESS; `partial` is column-sum staging)
template <typename T>
hipError_t launch_bwd_prologue(const MoeDims& D, const T* dY, const T* o,
                               const int32_t* perm, const int32_t* offsets, const float* gate,
                               T* dout, float* dgate, float* partial, float* db2, hipStream_t st);
template <typename T>
hipError_t launch_combine_dx(const MoeDims& D, const T* dxp, const int32_t* inv, T* dx,
                             hipStream_t st);
// ESS: out[e][c] = sum over the expert's rows of src[p][c]; src is [A, ncols] in perm order
template <typename T>
hipError_t launch_segment_colsum(const MoeDims& D, const T* src, int ncols, const int32_t* offsets,
                                 float* partial, float* out, hipStream_t st);

// second stage for column sums the bf16 DGRAD2 kernel left per (row tile, wave row):
// out[e][c] = sum of the partial rows of the expert's tiles, in tile order
hipError_t launch_tile_colsum_finish(const MoeDims& D, const float* partial, int ncols,
                                     const int32_t* offsets, float* out, hipStream_t st);

// fp32 reference-precision path (plain FMA tiles)
hipError_t launch_f32_fwd(const MoeDims& D, const float* x, const float* W1, const float* b1,
                          const float* W2, const float* b2, const hexa_moe_idx& idx,
                          const MoeWorkspace& ws, hipStream_t st);
hipError_t launch_f32_bwd(const MoeDims& D, const float* x, const float* W1, const float* W2,
                          const hexa_moe_idx& idx, const MoeWorkspace& ws, float* dW1, float* dW2,
                          hipStream_t st);

// 16-bit MFMA path: pointers are raw 16-bit storage, bf16 or (f16 = true) IEEE fp16
hipError_t launch_bf16_fwd(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* b1,
                           const bf16_t* W2, const bf16_t* b2, const hexa_moe_idx& idx,
                           const MoeWorkspace& ws, hipStream_t st, bool f16);
hipError_t launch_bf16_bwd(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* W2,
                           const hexa_moe_idx& idx, const MoeWorkspace& ws, float* dW1, float* dW2,
                           hipStream_t st, bool f16);

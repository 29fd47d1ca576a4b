// bf16 MFMA contractions of the expert-specific MoE layer (HEXA-MoE Sec. 3.1; App. B Table 5).
//
// Six contractions share one kernel template:
//   row GEMMs  (ESMM, App. B Alg. 2): rows are one expert segment of the re-index vector
//       FC1     pre = x[perm/k] W1[e] + b1[e],  h = GELU(pre)        K = d, N = f
//       FC2     o   = h W2[e] + b2[e]                                K = f, N = d
//       DGRAD2  dpre = (do W2[e]^T) * GELU'(pre)                     K = d, N = f
//       DGRAD1  dxp = dpre W1[e]^T                                   K = f, N = d
//   token contractions (ESTMM, App. B Alg. 4): the sum runs over one expert's rows
//       WGRAD2  dW2[e] = h^T do                                      M = f, N = d
//       WGRAD1  dW1[e] = xg^T dpre                                   M = d, N = f
//
// What is kept from the paper: rows of a tile all belong to one expert, so a tile needs one
// expert's weights; rows are addressed through the re-index vector, so nothing is padded to a
// capacity and nothing is dropped.  What is not: the 16x16x16 warp tiles, the per-expert serial
// loop of Alg. 4 and the padded (-1) re-index vector.  Here a workgroup owns a 256x256 (or
// 128-wide) tile, each 64-lane wavefront a grid of 32x32x16 bf16 MFMA blocks, operands are
// staged through LDS as [row][64 k] with a 16-byte XOR swizzle (conflict-free 128-bit reads),
// operands whose contraction index is the slow one in memory (weights in the forward GEMMs,
// both operands of the token contractions) are transposed in registers on the way to LDS,
// segments are tiled individually (ragged tails are masked, not padded), long segments of the
// token contractions are split into chunks whose partial tiles are reduced in a fixed order,
// and workgroup ids are remapped so that the 32 CUs of one XCD work on neighbouring tiles.
#include <type_traits>

#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;           // contraction elements per LDS stage (one 128-byte row)
constexpr int kXcds = 8;         // workgroup i is dispatched to XCD i % 8
constexpr int kGroupM = 8;       // row tiles per L2-sharing group

enum Op { OP_FC1 = 0, OP_FC2, OP_DGRAD2, OP_DGRAD1, OP_WGRAD2, OP_WGRAD1 };

struct GemmArgs {
    const bf16_t* A;      // row GEMM: [rows][K] (rows = tokens when gather, else perm positions)
                          // token contraction: [A][M] perm order
    const bf16_t* B;      // row GEMM: weights [E][..]; token contraction: [A][N] perm order
    const int32_t* perm;  // FC1 gather
    const int32_t* offsets;
    const bf16_t* bias;   // [E][N] or NULL
    const bf16_t* pre_in; // DGRAD2
    void* out0;
    void* out1;
    float* kpart;         // split-K slots [slot][M][N]
    int topk, E, K, N, M;
    int chunk_len;        // token contraction: max tokens per work item
};

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// r = 1 / (1 + exp(2 s)),  s = sqrt(2/pi) (u + 0.044715 u^3):  tanh(s) = 1 - 2 r
__device__ __forceinline__ float gelu_r(float u) {
    const float u2 = u * u;
    const float s2 = u * (2.f * HEXA_GELU_C + 2.f * HEXA_GELU_C * HEXA_GELU_A * u2);  // 2 s
    return fast_rcp(1.f + fast_exp2(s2 * 1.4426950408889634f));
}
__device__ __forceinline__ float gelu_fast(float u) { return u - u * gelu_r(u); }
__device__ __forceinline__ float gelu_grad_fast(float u) {
    const float r = gelu_r(u);
    const float sig = 1.f - r;  // (1 + tanh) / 2
    const float q = HEXA_GELU_C * (1.f + 3.f * HEXA_GELU_A * u * u);
    return sig * (1.f + 2.f * u * r * q);
}

__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
    return (uint32_t)(row * 128 + ((chunk ^ (row & 7)) << 4));
}

// ---------------------------------------------------------------------------------------------
// Operand loaders: global -> registers (issued one stage ahead) -> LDS [R rows][64 k], swizzled.
// ---------------------------------------------------------------------------------------------

// Contraction index contiguous in memory: thread owns 16-byte chunks (row q>>3, chunk q&7).
template <int R, int NT>
struct LoaderKC {
    static constexpr int NLD = R * 8 / NT;   // 16-byte loads per thread and stage
    static constexpr int NST = NLD;          // staging registers (uint4)
    static constexpr int NOFF = NLD;         // row offsets kept per thread

    // rowoff: element offset of each owned row's start (already clamped to a valid row)
    __device__ static __forceinline__ void gload(u32x4 (&st)[NST], const long long (&rowoff)[NOFF],
                                                 const bf16_t* __restrict__ base, int k0, int tid) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = (tid + NT * i) & 7;
            st[i] = *reinterpret_cast<const u32x4*>(base + rowoff[i] + k0 + c * 8);
        }
    }
    __device__ static __forceinline__ void sstore(const u32x4 (&st)[NST], uint8_t* lds, int tid) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int q = tid + NT * i;
            *reinterpret_cast<u32x4*>(lds + lds_off(q >> 3, q & 7)) = st[i];
        }
    }
};

// Contraction index strided in memory (row-contiguous): thread owns KR k-rows x 8 columns,
// transposes them in registers and writes 8 LDS rows.  KR = 8 (full block) or 4 (half block,
// used when there are fewer 8x8 blocks than threads).
template <int R, int NT>
struct LoaderKS {
    static constexpr int NBLK = R;  // (R/8) * 8 blocks of 8x8
    static constexpr bool HALF = NBLK < NT;
    static constexpr int KR = HALF ? 4 : 8;
    static constexpr int NB = HALF ? 1 : NBLK / NT;
    static_assert(HALF ? (NBLK * 2 == NT) : (NBLK % NT == 0), "unsupported loader shape");
    static constexpr int NST = NB * KR;
    static constexpr int NOFF = 1;

    // base: element (k = 0 of this stage, column 0 of the tile); ld in elements;
    // kvalid: k-rows of this stage that exist (others read as zero); cvalid: valid columns.
    __device__ static __forceinline__ void gload(u32x4 (&st)[NST], const bf16_t* __restrict__ base,
                                                 long long ld, int kvalid, int cvalid, int tid) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int q = tid + NT * b;
            const int kblk = q & 7;
            const int rblk = HALF ? ((q >> 3) % (R / 8)) : (q >> 3);
            const int hh = HALF ? (q / R) : 0;
            const int col = (rblk * 8 < cvalid) ? rblk * 8 : 0;  // clamp: masked at the store
#pragma unroll
            for (int kk = 0; kk < KR; ++kk) {
                const int krow = kblk * 8 + hh * 4 + kk;
                const bool ok = krow < kvalid;
                const int kr = ok ? krow : 0;
                u32x4 v = *reinterpret_cast<const u32x4*>(base + (long long)kr * ld + col);
                if (!ok) v = u32x4{0, 0, 0, 0};
                st[b * KR + kk] = v;
            }
        }
    }
    __device__ static __forceinline__ void sstore(const u32x4 (&st)[NST], uint8_t* lds, int tid) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int q = tid + NT * b;
            const int kblk = q & 7;
            const int rblk = HALF ? ((q >> 3) % (R / 8)) : (q >> 3);
            const int hh = HALF ? (q / R) : 0;
            uint32_t w[KR][4];
#pragma unroll
            for (int kk = 0; kk < KR; ++kk) {
                w[kk][0] = st[b * KR + kk].x; w[kk][1] = st[b * KR + kk].y;
                w[kk][2] = st[b * KR + kk].z; w[kk][3] = st[b * KR + kk].w;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
                const int row = rblk * 8 + j;
                if constexpr (HALF) {
                    u32x2 o;
                    o.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel);
                    o.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel);
                    *reinterpret_cast<u32x2*>(lds + lds_off(row, kblk) + hh * 8) = o;
                } else {
                    u32x4 o;
                    o.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel);
                    o.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel);
                    o.z = __builtin_amdgcn_perm(w[5][j >> 1], w[4][j >> 1], sel);
                    o.w = __builtin_amdgcn_perm(w[7][j >> 1], w[6][j >> 1], sel);
                    *reinterpret_cast<u32x4*>(lds + lds_off(row, kblk)) = o;
                }
            }
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Work decomposition
// ---------------------------------------------------------------------------------------------

// XCD-aware id: the G logical items are cut into 8 contiguous ranges, one per XCD.
__device__ __forceinline__ int xcd_remap(int wg, int G) {
    const int per = ceil_div(G, kXcds);
    const int xcd = wg % kXcds, loc = wg / kXcds;
    if (loc >= per) return -1;
    const int pid = xcd * per + loc;
    return pid < G ? pid : -1;
}

// Inside one set of tm x tn tiles: groups of kGroupM row tiles, row tile fastest inside a group.
__device__ __forceinline__ void grouped_tile(int local, int tm, int tn, int& tile_m, int& tile_n) {
    const int per_group = kGroupM * tn;
    const int group = local / per_group;
    const int first = group * kGroupM;
    const int gsz = min(kGroupM, tm - first);
    const int in = local - group * per_group;
    tile_m = first + in % gsz;
    tile_n = in / gsz;
}

struct TokenItem { int e, kbeg, kend, tile_m, tile_n, nchunks, slot; };

// Token-contraction items: expert-major, chunk, then tiles.  slot = index into the split-K
// partial buffer (only used when the expert has more than one chunk).
__device__ __forceinline__ TokenItem token_item_find(const int32_t* __restrict__ offsets, int E,
                                                     int L, int tm, int tn, int pid) {
    TokenItem it{-1, 0, 0, 0, 0, 0, 0};
    int acc = 0, slot = 0;
    const int tmn = tm * tn;
    for (int e = 0; e < E; ++e) {
        const int b = offsets[e], n = offsets[e + 1] - b;
        const int nch = ceil_div(n, L);
        const int items = nch * tmn;
        if (pid < acc + items) {
            const int local = pid - acc;
            const int c = local / tmn;
            it.e = e; it.nchunks = nch; it.slot = slot + c;
            it.kbeg = b + c * L; it.kend = min(b + n, it.kbeg + L);
            grouped_tile(local - c * tmn, tm, tn, it.tile_m, it.tile_n);
            return it;
        }
        acc += items;
        if (nch > 1) slot += nch;
    }
    return it;
}

__device__ __forceinline__ int token_items_total(const int32_t* __restrict__ offsets, int E, int L,
                                                 int tmn) {
    int total = 0;
    for (int e = 0; e < E; ++e) total += ceil_div(offsets[e + 1] - offsets[e], L) * tmn;
    return total;
}

// ---------------------------------------------------------------------------------------------
// The kernel
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int OP>
__global__ __launch_bounds__(WM * WN * 64, 1) void gemm_bf16(GemmArgs g) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr bool TOKENS = (OP == OP_WGRAD2 || OP == OP_WGRAD1);
    constexpr bool B_KS = TOKENS || OP == OP_FC1 || OP == OP_FC2;
    constexpr int STAGE = (BM + BN) * 128;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of 32x32");

    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, hi = lane >> 5;

    // ---- which work item ------------------------------------------------------------------
    int e, m0, n0, mvalid, nk;
    int kbeg = 0, kend = 0;           // token contraction: perm rows of this item
    float* tok_out = nullptr;         // token contraction: where the tile goes
    if constexpr (!TOKENS) {
        const int tm_total = seg_tiles_total(g.offsets, g.E, BM);
        const int tn = ceil_div(g.N, BN);
        const int pid = xcd_remap(blockIdx.x, tm_total * tn);
        if (pid < 0) return;
        int tile_m, tile_n;
        grouped_tile(pid, tm_total, tn, tile_m, tile_n);
        const SegTile s = seg_tile_find(g.offsets, g.E, BM, tile_m);
        e = s.e; m0 = s.row0; mvalid = s.rows; n0 = tile_n * BN;
        nk = g.K / BK;
    } else {
        const int tm = ceil_div(g.M, BM), tn = ceil_div(g.N, BN);
        const int G = token_items_total(g.offsets, g.E, g.chunk_len, tm * tn);
        const int pid = xcd_remap(blockIdx.x, G);
        if (pid < 0) return;
        const TokenItem it = token_item_find(g.offsets, g.E, g.chunk_len, tm, tn, pid);
        e = it.e; m0 = it.tile_m * BM; n0 = it.tile_n * BN; mvalid = min(BM, g.M - m0);
        kbeg = it.kbeg; kend = it.kend;
        nk = ceil_div(kend - kbeg, BK);
        tok_out = (it.nchunks > 1) ? g.kpart + (size_t)it.slot * g.M * g.N
                                   : reinterpret_cast<float*>(g.out0) + (size_t)e * g.M * g.N;
    }
    const int nvalid = min(BN, g.N - n0);

    // ---- loaders ----------------------------------------------------------------------------
    using LA = typename std::conditional<TOKENS, LoaderKS<BM, NT>, LoaderKC<BM, NT>>::type;
    using LB = typename std::conditional<B_KS, LoaderKS<BN, NT>, LoaderKC<BN, NT>>::type;
    u32x4 sta[LA::NST], stb[LB::NST];
    long long offa[LA::NOFF], offb[LB::NOFF];
    const bf16_t* a_base;
    const bf16_t* b_base;
    long long a_ld = 0, b_ld = 0;
    if constexpr (!TOKENS) {
        a_base = g.A;
#pragma unroll
        for (int i = 0; i < LA::NLD; ++i) {
            int r = (tid + NT * i) >> 3;
            if (r >= mvalid) r = 0;  // rows past the segment: read a valid row, never stored
            long long src = m0 + r;
            if constexpr (OP == OP_FC1) src = g.perm[m0 + r] / g.topk;
            offa[i] = src * g.K;
        }
        if constexpr (B_KS) {  // W[e][K][N]
            b_base = g.B + (size_t)e * g.K * g.N + n0;
            b_ld = g.N;
        } else {               // W[e][N][K]
            b_base = g.B + (size_t)e * g.N * g.K;
#pragma unroll
            for (int i = 0; i < LB::NLD; ++i) {
                int r = (tid + NT * i) >> 3;
                if (r >= nvalid) r = 0;
                offb[i] = (long long)(n0 + r) * g.K;
            }
        }
    } else {
        a_base = g.A + (size_t)kbeg * g.M + m0; a_ld = g.M;
        b_base = g.B + (size_t)kbeg * g.N + n0; b_ld = g.N;
    }

#define LOAD_STAGE(kt_)                                                                          \
    do {                                                                                         \
        const int kt__ = (kt_);                                                                  \
        if constexpr (!TOKENS) {                                                                 \
            LA::gload(sta, offa, a_base, kt__ * BK, tid);                                        \
            if constexpr (B_KS)                                                                  \
                LB::gload(stb, b_base + (size_t)kt__ * BK * b_ld, b_ld, BK, nvalid, tid);        \
            else                                                                                 \
                LB::gload(stb, offb, b_base, kt__ * BK, tid);                                    \
        } else {                                                                                 \
            const int kv__ = min(BK, kend - kbeg - kt__ * BK);                                   \
            LA::gload(sta, a_base + (size_t)kt__ * BK * a_ld, a_ld, kv__, mvalid, tid);          \
            LB::gload(stb, b_base + (size_t)kt__ * BK * b_ld, b_ld, kv__, nvalid, tid);          \
        }                                                                                        \
    } while (0)
#define STORE_STAGE(buf_)                                                                        \
    do {                                                                                         \
        LA::sstore(sta, smem + (buf_) * STAGE, tid);                                             \
        LB::sstore(stb, smem + (buf_) * STAGE + BM * 128, tid);                                  \
    } while (0)
    (void)offa; (void)offb; (void)a_ld;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // per-lane fragment addresses: row (wave tile row + l32), chunk (2 s + hi) ^ (l32 & 7)
    const uint32_t a_row_off = (uint32_t)((wm * TM + l32) * 128);
    const uint32_t b_row_off = (uint32_t)(BM * 128 + (wn * TN + l32) * 128);
    uint32_t coff[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) coff[s] = (uint32_t)(((2 * s + hi) ^ (l32 & 7)) << 4);

    if (nk > 0) {
        LOAD_STAGE(0);
        STORE_STAGE(0);
        if (nk > 1) LOAD_STAGE(1);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const uint8_t* sbase = smem + cur * STAGE;
        if (kt + 1 < nk) STORE_STAGE(cur ^ 1);   // registers hold stage kt+1
        if (kt + 2 < nk) LOAD_STAGE(kt + 2);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 af[FM], bfr[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(sbase + a_row_off + i * 32 * 128 + coff[s]);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(sbase + b_row_off + j * 32 * 128 + coff[s]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

#undef LOAD_STAGE
#undef STORE_STAGE

    // ---- epilogue: lane holds column l32 of each 32x32 block, rows 8 q + 4 hi + (r & 3) ------
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int col = wn * TN + j * 32 + l32;
        const bool cok = col < nvalid;
        const int n = n0 + col;
        float bias = 0.f;
        if constexpr (OP == OP_FC1 || OP == OP_FC2)
            if (cok) bias = bf2f(g.bias[(size_t)e * g.N + n]);
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * TM + i * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (!cok || row >= mvalid) continue;
                const float v = acc[i][j][r] + bias;
                if constexpr (TOKENS) {
                    tok_out[(size_t)(m0 + row) * g.N + n] = v;
                } else {
                    const size_t oi = (size_t)(m0 + row) * g.N + n;
                    if constexpr (OP == OP_FC1) {
                        reinterpret_cast<bf16_t*>(g.out0)[oi] = f2bf(v);
                        reinterpret_cast<bf16_t*>(g.out1)[oi] = f2bf(gelu_fast(v));
                    } else if constexpr (OP == OP_DGRAD2) {
                        reinterpret_cast<bf16_t*>(g.out0)[oi] = f2bf(v * gelu_grad_fast(bf2f(g.pre_in[oi])));
                    } else {
                        reinterpret_cast<float*>(g.out0)[oi] = v;
                    }
                }
            }
        }
    }
}

// Second stage of the split token contraction, plus exact zeros for experts without tokens.
// out[e] = sum_c kpart[slot_e + c] in chunk order when the expert was split; untouched when it
// had exactly one chunk (the GEMM wrote it directly).
__global__ __launch_bounds__(256) void wgrad_finish(const int32_t* __restrict__ offsets, int E, int L,
                                                    size_t mn, const float* __restrict__ kpart,
                                                    float* __restrict__ out) {
    const int e = blockIdx.y;
    const int n = offsets[e + 1] - offsets[e];
    const int nch = ceil_div(n, L);
    if (nch == 1) return;
    int slot = 0;
    for (int q = 0; q < e; ++q) {
        const int c = ceil_div(offsets[q + 1] - offsets[q], L);
        if (c > 1) slot += c;
    }
    float4* dst = reinterpret_cast<float4*>(out + (size_t)e * mn);
    const size_t n4 = mn / 4;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c = 0; c < nch; ++c) {
            const float4 v = reinterpret_cast<const float4*>(kpart + (size_t)(slot + c) * mn)[i];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        dst[i] = s;
    }
}

constexpr int kNumCUs = 256;

template <int BM, int BN, int WM, int WN, int OP>
void launch_rows(const MoeDims& D, const GemmArgs& g, hipStream_t st) {
    auto kern = gemm_bf16<BM, BN, WM, WN, OP>;
    constexpr int lds = 2 * (BM + BN) * 128;
    static bool attr_done = false;
    if (!attr_done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_done = true;
    }
    const int tm_max = D.A / BM + D.E;
    const int gmax = tm_max * ceil_div(g.N, BN);
    const int grid = kXcds * ceil_div(gmax, kXcds);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds, st, g);
}

template <int BM, int BN, int WM, int WN, int OP>
void launch_tokens(const MoeDims& D, const GemmArgs& g, hipStream_t st) {
    auto kern = gemm_bf16<BM, BN, WM, WN, OP>;
    constexpr int lds = 2 * (BM + BN) * 128;
    static bool attr_done = false;
    if (!attr_done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_done = true;
    }
    const int tmn = ceil_div(g.M, BM) * ceil_div(g.N, BN);
    const int chunks_max = D.A / g.chunk_len + D.E;
    const int grid = kXcds * ceil_div(chunks_max * tmn, kXcds);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds, st, g);
    const size_t mn = (size_t)g.M * g.N;
    const int gx = (int)((mn / 4 + 255) / 256 < 1024 ? (mn / 4 + 255) / 256 : 1024);
    hipLaunchKernelGGL(wgrad_finish, dim3(gx, D.E), dim3(256), 0, st, g.offsets, D.E, g.chunk_len, mn,
                       g.kpart, reinterpret_cast<float*>(g.out0));
}

constexpr int TBM = 256, TBN = 256, TWM = 2, TWN = 2;

}  // namespace

// Tokens per split-K chunk of the token contractions: long enough that most experts are one
// chunk (no partial traffic), short enough that ~4 items per CU exist under skewed routing.
int wgrad_chunk_len(const MoeDims& D) {
    const long long tmn = (long long)ceil_div(D.d, TBM) * ceil_div(D.f, TBN);
    long long L = (long long)D.A * tmn / (4 * kNumCUs);
    L = (L + 63) / 64 * 64;
    if (L < 1024) L = 1024;
    return (int)L;
}

// Upper bound on split-K slots: only experts with more than one chunk use slots, and
// sum over those of ceil(n_e / L) <= 2 A / L.
size_t wgrad_max_slots(const MoeDims& D) {
    return 2 * (size_t)(D.A / wgrad_chunk_len(D)) + 2;
}

hipError_t launch_bf16_fwd(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* b1,
                           const bf16_t* W2, const bf16_t* b2, const hexa_moe_idx& idx,
                           const MoeWorkspace& ws, hipStream_t st) {
    GemmArgs g{};
    g.offsets = idx.offsets; g.perm = idx.perm; g.topk = D.k; g.E = D.E;
    g.A = x; g.B = W1; g.bias = b1; g.out0 = ws.pre; g.out1 = ws.h; g.K = D.d; g.N = D.f;
    launch_rows<TBM, TBN, TWM, TWN, OP_FC1>(D, g, st);
    g.A = (const bf16_t*)ws.h; g.B = W2; g.bias = b2; g.out0 = ws.o; g.out1 = nullptr; g.K = D.f; g.N = D.d;
    launch_rows<TBM, TBN, TWM, TWN, OP_FC2>(D, g, st);
    return hipGetLastError();
}

hipError_t launch_bf16_bwd(const MoeDims& D, const bf16_t* xg, const bf16_t* W1, const bf16_t* W2,
                           const hexa_moe_idx& idx, const MoeWorkspace& ws, float* dW1, float* dW2,
                           hipStream_t st) {
    GemmArgs g{};
    g.offsets = idx.offsets; g.perm = idx.perm; g.topk = D.k; g.E = D.E;
    g.kpart = ws.kpart; g.chunk_len = wgrad_chunk_len(D);
    // dpre = (do W2^T) * GELU'(pre)
    g.A = (const bf16_t*)ws.dout; g.B = W2; g.pre_in = (const bf16_t*)ws.pre; g.out0 = ws.dpre;
    g.K = D.d; g.N = D.f;
    launch_rows<TBM, TBN, TWM, TWN, OP_DGRAD2>(D, g, st);
    // dW2[e] = h^T do
    g.A = (const bf16_t*)ws.h; g.B = (const bf16_t*)ws.dout; g.out0 = dW2; g.M = D.f; g.N = D.d;
    launch_tokens<TBM, TBN, TWM, TWN, OP_WGRAD2>(D, g, st);
    // dxp = dpre W1^T
    g.A = (const bf16_t*)ws.dpre; g.B = W1; g.out0 = ws.dxp; g.K = D.f; g.N = D.d;
    launch_rows<TBM, TBN, TWM, TWN, OP_DGRAD1>(D, g, st);
    // dW1[e] = xg^T dpre
    g.A = xg; g.B = (const bf16_t*)ws.dpre; g.out0 = dW1; g.M = D.d; g.N = D.f;
    launch_tokens<TBM, TBN, TWM, TWN, OP_WGRAD1>(D, g, st);
    return hipGetLastError();
}

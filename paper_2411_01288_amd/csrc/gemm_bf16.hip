// bf16 MFMA contractions of the expert-specific MoE layer (HEXA-MoE Sec. 3.1; App. B Table 5).
//
// Six contractions share one tile routine (forward: one grid each; backward: the input-gradient
// and weight-gradient contractions of a linear layer share a grid):
//   row GEMMs  (ESMM, App. B Alg. 2): rows are one expert segment of the re-index vector
//       FC1     pre = x[perm/k] W1[e] + b1[e],  h = F(pre), g = F'(pre) saved        K = d, N = f
//       FC2     o   = h W2[e] + b2[e]   (stored as bf16)                 K = f, N = d
//       DGRAD2  dpre = (do W2[e]^T) * g                              K = d, N = f
//       DGRAD1  dxp = dpre W1[e]^T      (stored as bf16)                 K = f, N = d
//   token contractions (ESTMM, App. B Alg. 4): the sum runs over one expert's rows
//       WGRAD2  dW2[e] = h^T do                                      M = f, N = d
//       WGRAD1  dW1[e] = x[perm/k]^T dpre  (token rows gathered)      M = d, N = f
//
// What is kept from the paper: rows of a tile all belong to one expert, so a tile needs one
// expert's weights; rows are addressed through the re-index vector, so nothing is padded to a
// capacity and nothing is dropped.  What is not: the 16x16x16 warp tiles, the per-expert serial
// loop of Alg. 4 and the padded (-1) re-index vector.  Here a workgroup owns a 256x256 tile,
// each 64-lane wavefront a grid of 16x16x32 bf16 MFMA blocks, operands go from
// global memory straight into LDS (no registers in between) as [row][64 k] with a 16-byte XOR
// swizzle (conflict-free 128-bit reads); operands whose contraction index is the slow one in
// memory (weights in the forward GEMMs, both operands of the token contractions) keep their
// memory layout in LDS and are transposed by the LDS read instruction; segments are tiled
// individually (ragged tails are masked, not padded), long segments of the token contractions
// are split into chunks whose partial tiles are reduced in a fixed order, and workgroup ids are
// remapped so that the 32 CUs of one XCD work on neighbouring tiles.
#include <type_traits>

#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;            // contraction elements per block of the K loop (one 128-byte line per row)
constexpr int NSLOT = 5;          // LDS ring: five slots, each holds one operand's share of a block
constexpr int kXcds = 8;         // workgroup i is dispatched to XCD i % 8
constexpr int kGroupM = 4;       // row tiles per L2-sharing group
constexpr int kSplitBelow = 128; // row GEMMs with fewer groups cut their last ngroups % 8 groups across the XCDs

enum Op { OP_FC1 = 0, OP_FC2, OP_DGRAD2, OP_DGRAD1, OP_WGRAD2, OP_WGRAD1 };

struct GemmArgs {
    const bf16_t* A;      // row GEMM: [rows][K] (rows = tokens when gather, else perm positions)
                          // token contraction: [A][M] perm order
    const bf16_t* B;      // row GEMM: weights [E][..]; token contraction: [A][N] perm order
    const int32_t* perm;  // FC1 gather
    const uint32_t* rowoff;  // WGRAD1 gather: byte offsets of the token rows, see build_rowoff
    const int32_t* offsets;
    const bf16_t* bias;   // [E][N] or NULL
    const bf16_t* pre_in; // DGRAD2: the saved GELU'(pre)
    void* out0;
    void* out1;
    float* kpart;         // split-K slots [slot][M][N]
    float* colpart;       // DGRAD2: per (row tile, wave row) column sums of dpre [2*tiles][N]
    int topk, E, K, N, M;
    int a_rows;           // FC1: rows of the gathered operand (tokens T)
    int chunk_len;        // token contraction: max tokens per work item
    const int32_t* worklist;  // see build_worklists
    int rt_cap;           // row-tile capacity of the work list
};

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// s = 1 / (1 + exp(-2 t)),  t = sqrt(2/pi) (u + 0.044715 u^3):  tanh(t) = 2 s - 1, GELU(u) = u s.
// exp(-2 t) = 2^(u (k1 + k3 u^2)) with -log2(e) folded into the two constants.
// h = GELU(u) = u s and g = GELU'(u) = s + u s (1 - s) 2C (1 + 3 A u^2) from one s: eight
// full-rate operations and two transcendental ones
// (App. B Table 5 rows 2 and 7 need both; the forward epilogue has u in registers, so it saves g
// for the backward pass instead of u itself: same bytes, and the backward epilogue is one multiply).
__device__ __forceinline__ void gelu_both(float u, float& h, float& g) {
    constexpr float k1 = -2.f * HEXA_GELU_C * 1.4426950408889634f;
    constexpr float k3 = k1 * HEXA_GELU_A;
    const float u2 = u * u;
    const float s = fast_rcp(1.f + fast_exp2(u * (k1 + k3 * u2)));
    h = u * s;
    const float q = 2.f * HEXA_GELU_C + 6.f * HEXA_GELU_C * HEXA_GELU_A * u2;
    g = s + (h - h * s) * q;
}

// The same pair for the other activations: ReLU (derivative 0 at 0) and SiLU u s(u), s = 1/(1+e^-u),
// with derivative s (1 + u (1 - s)).
template <int ACT>
__device__ __forceinline__ void act_both(float u, float& h, float& g) {
    if constexpr (ACT == HEXA_ACT_RELU) {
        h = u > 0.f ? u : 0.f;
        g = u > 0.f ? 1.f : 0.f;
    } else if constexpr (ACT == HEXA_ACT_SILU) {
        const float sg = fast_rcp(1.f + fast_exp2(-1.4426950408889634f * u));
        h = u * sg;
        g = sg * (1.f + u * (1.f - sg));
    } else {
        gelu_both(u, h, g);
    }
}

// LDS image of a K-contiguous operand: row r = BK*2 = 128 bytes = CPRK chunks of 16 bytes (8 bf16
// along k); chunk c of row r sits at position c ^ key(r).  gfx950's LDS serves 128-bit reads 16 lanes
// (256 bytes, 64 banks) per clock; a 16x16x32 fragment read has 16 consecutive lanes on 16
// consecutive rows with one chunk index.  Two consecutive 128-byte rows fill the 256 bytes of bank
// space, so rows r, r+2, ..., r+14 must sit on eight different chunk positions:
// key(r) = (r >> 1) & 7.
constexpr int CPRK = BK * 2 / 16;                 // chunks per row
constexpr int ROWB = BK * 2;                      // bytes per row
static_assert(BK == 64, "the K loop and the swizzle are written for 64-element blocks");
__device__ __forceinline__ uint32_t lds_swz(int row) { return (uint32_t)((row >> 1) & 7); }

// ---------------------------------------------------------------------------------------------
// Operand staging: global -> LDS without passing through registers.
//
// gfx950 can write a 16-byte-per-lane buffer load straight into LDS ("buffer_load_dwordx4 ... lds"):
// the 64 lanes of one instruction fill 1024 consecutive LDS bytes in lane order, each lane
// fetching from its own global address.  LDS stores from registers run at ~64 B/clk/CU on this
// part, half of what a 256x256 tile needs at the MFMA rate, and cost 128 VGPRs per stage; the
// direct path costs neither.  Because the LDS position of a lane is fixed, the bank swizzle is
// applied on the global side: a lane fetches the chunk that belongs at its position.
//
// Reads past the byte range of the buffer resource return zero, which masks ragged row tails and
// the K tail of the token contractions for free.
// ---------------------------------------------------------------------------------------------
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef i32x4 rsrc_t;   // raw buffer resource: base[47:0], stride 0, byte range, gfx9 data format word
typedef __attribute__((address_space(3))) void* lds_void_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    // all four words are wave-uniform; say so, the staging instruction wants them in SGPRs
    const uint64_t b = (uint64_t)base;
    return rsrc_t{__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)b),
                  __builtin_amdgcn_readfirstlane((int32_t)((uint32_t)(b >> 32) & 0xffffu)),
                  __builtin_amdgcn_readfirstlane((int32_t)bytes), 0x00020000};
}
// one instruction: lane l's 16 bytes at (voff + soff) land at lds + 16*l; lds is wave-uniform.
// Written as inline assembly on purpose: the compiler then neither tracks these loads in vmcnt nor
// assumes that every later LDS read may alias them (which made it wait for the whole stage in
// front of each fragment read).  The kernel counts its own requests and waits explicitly (one
// "s_waitcnt vmcnt(n)" in front of the barrier that publishes a block, n = the requests that may
// still be in flight); the only other vector-memory loads inside the K loop are the row-offset
// loads of the gathered token contraction, inline assembly too and counted with them.  M0 carries
// the LDS address (one wait state before the load reads it).
__device__ __forceinline__ void dtl16(rsrc_t r, uint8_t* lds, uint32_t voff, uint32_t soff) {
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
        (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)lds);
    soff = __builtin_amdgcn_readfirstlane(soff);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(r), "s"(soff)
                 : "memory", "m0");
}

// The same in two parts for the K loop, where the instructions of a staging request are spread over
// two issue slots: the LDS address (an integer byte address, wave-uniform) goes into M0 in one slot,
// the load follows in the next one (an MFMA in between provides the wait state).  Nothing else in the
// K loop uses M0.
__device__ __forceinline__ void dtl_m0(uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0" : : "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory", "m0");
}
__device__ __forceinline__ void dtl_load(rsrc_t r, uint32_t voff, uint32_t soff) {
    asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds"
                 :
                 : "v"(voff), "s"(r), "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "memory");
}

// K-contiguous operand (R rows x BK k, ROWB bytes per row in memory order along k).
// Instruction q (= wave + NW*i) fills RPQ = 1024/ROWB rows: lane l -> row RPQ*q + l/CPRK,
// position l%CPRK.
template <int R, int NW, bool GATHER>
struct StageKC {
    static constexpr int RPQ = 1024 / ROWB;      // rows per instruction
    static constexpr int NI = R / RPQ / NW;      // instructions per wave and stage
    static_assert(R % (RPQ * NW) == 0 && (RPQ * NW) % 16 == 0, "unsupported staging shape");
    // byte offset of (row, chunk) from the resource base: one per instruction when the rows are
    // gathered; otherwise instruction i is RPQ*NW*i rows further down, which goes into the scalar
    // offset
    struct Lane { uint32_t voff[GATHER ? NI : 1]; };
    // chunk this lane must fetch: its position XOR the swizzle key of its row (the key has period
    // 16 rows and RPQ*NW is a multiple of 16, so it is the same for every instruction of a wave)
    __device__ static __forceinline__ int lane_chunk(int wave, int lane) {
        return (lane % CPRK) ^ (int)lds_swz(RPQ * wave + lane / CPRK);
    }
    __device__ static __forceinline__ int lane_row(int wave, int lane, int i) {
        return RPQ * (wave + NW * i) + lane / CPRK;
    }
    // instruction i of this wave: set-up (LDS address of its 1 KB piece of the slot at lds_slot) and load
    __device__ static __forceinline__ void prep(uint32_t lds_slot, int wave, int i) {
        dtl_m0(lds_slot + (uint32_t)(wave + NW * i) * 1024u);
    }
    __device__ static __forceinline__ void load(rsrc_t r, uint32_t soff, uint32_t row_bytes, const Lane& ln, int i) {
        if constexpr (GATHER) dtl_load(r, ln.voff[i], soff);
        else dtl_load(r, ln.voff[0], soff + (uint32_t)(RPQ * NW * i) * row_bytes);
    }
};

// K-strided operand (BK k-rows x R columns, a k-row is R*2 contiguous bytes in memory).
// LDS image: k-row k at k*R*2, 16-byte chunk c (8 columns) at position c ^ ks_key(k).
// It is read with ds_read_b64_tr_b16, which hands each lane four k-values of one column; a
// 32-lane half of such a read touches k-rows {8a + j, 8(a+1) + j : j < 4}, 32 bytes (16 columns) of
// each, and the key puts those eight pieces on the eight 32-byte slots of the bank space.
// Instruction q fills k-rows RPI*q .. RPI*q + RPI-1 (RPI = 512 / R rows of R*2 bytes).
__device__ __forceinline__ int ks_key(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

template <int R, int NW>
struct StageKS {
    static constexpr int RB = R * 2;            // bytes per k-row
    static constexpr int CPR = RB / 16;         // chunks per k-row
    static constexpr int RPI = 1024 / RB;       // k-rows per instruction
    static constexpr int NI = BK / RPI / NW;    // instructions per wave and block
    static_assert(RPI >= 1 && (BK / RPI) % NW == 0 && RPI * NW == 8 && CPR >= 16, "unsupported staging shape");
    // instruction i of a wave covers k-rows RPI*wave + kin + 8 i: (k & 3) is the same for all i and
    // ((k >> 3) & 1) = i & 1, so a lane needs two offsets (even and odd i)
    struct Lane { uint32_t voff[2]; };
    // (row_bytes = 0 when the k-rows are gathered: the row part of the offset then comes from a table)
    __device__ static __forceinline__ Lane lane_init(int wave, int lane, uint32_t row_bytes, int col0) {
        const int kin = lane / CPR;                          // k-row inside the instruction
        const int k = (RPI * wave + kin);                    // k-row of instruction i = 0  (< 8)
        Lane ln;
#pragma unroll
        for (int odd = 0; odd < 2; ++odd) {
            const int c = (lane % CPR) ^ ks_key(k + 8 * odd);
            ln.voff[odd] = (uint32_t)k * row_bytes + (uint32_t)(col0 + 8 * c) * 2u;
        }
        return ln;
    }
    // gathered k-rows: instruction i fetches the rows whose byte offsets are roff[i] (per lane)
    __device__ static __forceinline__ void load_gathered(rsrc_t r, const uint32_t (&roff)[NI], const Lane& ln, int i) {
        dtl_load(r, roff[i] + ln.voff[i & 1], 0u);
    }
    __device__ static __forceinline__ void prep(uint32_t lds_slot, int wave, int i) {
        dtl_m0(lds_slot + (uint32_t)(wave + NW * i) * 1024u);
    }
    __device__ static __forceinline__ void load(rsrc_t r, uint32_t soff, uint32_t ld_bytes, const Lane& ln, int i) {
        dtl_load(r, ln.voff[i & 1], soff + (uint32_t)(RPI * NW * i) * ld_bytes);
    }
};

// ---------------------------------------------------------------------------------------------
// Work decomposition
// ---------------------------------------------------------------------------------------------

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

// Work lists, built once per forward call from the segment offsets (the backward pass reads the same
// lists: they are part of what the forward pass leaves in the workspace), so that a
// workgroup finds its tile with two scalar loads instead of a walk over all experts (which cost a
// 256x256 tile of a d = 2048 contraction about a tenth of its time, with the CU idle meanwhile).
//   wl[0] = number of row tiles, wl[1] = number of token-contraction items,
//   wl[2], wl[3] = 1 when the fused backward grid of the second / first linear layer starts with
//                  its token contraction (see gemm_bf16_pair), else 0
//   wl[4 + 4 t ...]            row tile t:  expert, first perm row, rows (1..bm), unused
//   wl[4 + 4 rt_cap + 4 i ...] item i:      expert, first perm row, end perm row, split-K slot
// Row tiles are numbered expert-major (tiles never straddle experts; experts without rows have
// none).  Items are numbered expert-major then chunk: item i covers at most L rows of one expert;
// slot >= 0 numbers the partial tile buffer of an expert that was cut into several chunks, -1
// means the expert is one chunk and its tile goes straight to the output.
__global__ __launch_bounds__(1024) void build_worklists(const int32_t* __restrict__ offsets, int E,
                                                        int bm, int L, int32_t* __restrict__ wl,
                                                        int rt_cap, int d, int f) {
    __shared__ int s_t[1024], s_c[1024], s_s[1024];
    const int e = threadIdx.x;
    int b = 0, n = 0, nt = 0, nc = 0, ns = 0;
    if (e < E) {
        b = offsets[e]; n = offsets[e + 1] - b;
        nt = ceil_div(n, bm); nc = ceil_div(n, L); ns = nc > 1 ? nc : 0;
    }
    s_t[e] = nt; s_c[e] = nc; s_s[e] = ns;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {      // inclusive scans
        int vt = 0, vc = 0, vs = 0;
        if (e >= off) { vt = s_t[e - off]; vc = s_c[e - off]; vs = s_s[e - off]; }
        __syncthreads();
        s_t[e] += vt; s_c[e] += vc; s_s[e] += vs;
        __syncthreads();
    }
    if (e >= E) return;
    int t0 = s_t[e] - nt, c0 = s_c[e] - nc, slot0 = s_s[e] - ns;
    for (int i = 0; i < nt; ++i) {
        int32_t* q = wl + 4 + 4 * (t0 + i);
        q[0] = e; q[1] = b + i * bm; q[2] = min(bm, n - i * bm); q[3] = 0;
    }
    int32_t* items = wl + 4 + 4 * rt_cap;
    for (int c = 0; c < nc; ++c) {
        int32_t* q = items + 4 * (c0 + c);
        q[0] = e; q[1] = b + c * L; q[2] = min(b + n, b + c * L + L); q[3] = nc > 1 ? slot0 + c : -1;
    }
    if (e == E - 1) {
        // the longest token-contraction item, in rows; a fused backward grid starts with the token
        // contraction when that item runs at least eight times as long as a tile of the row GEMM it
        // shares the grid with (K = d for the second layer's, K = f for the first layer's)
        int longest = 0;
        for (int q = 0; q < E; ++q) longest = max(longest, min(L, offsets[q + 1] - offsets[q]));
        wl[0] = s_t[e]; wl[1] = s_c[e];
        wl[2] = longest >= 8 * d ? 1 : 0;
        wl[3] = longest >= 8 * f ? 1 : 0;
    }
}

// Row-offset table of the gathered token contraction (WGRAD1 reads x[perm[p] / k] for perm
// position p; ESTMM, App. B Alg. 4, takes its tokens through the re-index vector the same way).
// Expert e's part starts at entry offsets[e] + 64 e and is cut into blocks of 64 rows (the K-blocks
// of the contraction; a chunk starts on a block boundary); inside a block, entry 8 j + i belongs
// to row 8 i + j, the transposed order in which a lane of the staging instructions needs them.
// An entry is the byte offset of the token's row in x; entries past the segment's end hold `pad`,
// an offset behind the last row of x, which the buffer range check turns into zeros.
__global__ __launch_bounds__(256) void build_rowoff(const int32_t* __restrict__ offsets,
                                                    const int32_t* __restrict__ perm, int E, int k,
                                                    uint32_t row_bytes, uint32_t pad, int total,
                                                    uint32_t* __restrict__ out) {
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= total) return;
    int lo = 0, hi = E - 1;                       // the last expert whose part starts at or before g
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (offsets[mid] + 64 * mid <= g) lo = mid; else hi = mid - 1;
    }
    const int b = offsets[lo], n = offsets[lo + 1] - b;
    const int local = g - (b + 64 * lo);
    const int s = local & 63;
    const int r = (local & ~63) + 8 * (s & 7) + (s >> 3);
    out[g] = r < n ? (uint32_t)(perm[b + r] / k) * row_bytes : pad;
}

// ---------------------------------------------------------------------------------------------
// The kernel
// ---------------------------------------------------------------------------------------------
// One work-item slot `item` (slot i is dispatched to XCD i % 8) of contraction OP.
template <int BM, int BN, int WM, int WN, int OP, int ACT = HEXA_ACT_GELU_TANH, bool F16 = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int item) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 16, FN = TN / 16;   // 16x16 MFMA blocks per wave tile
    constexpr bool TOKENS = (OP == OP_WGRAD2 || OP == OP_WGRAD1);
    constexpr bool B_KS = TOKENS || OP == OP_FC1 || OP == OP_FC2;
    constexpr bool A_GK = (OP == OP_WGRAD1);   // operand A's k-rows (tokens) are gathered rows of x
    constexpr int SLOT = (BM > BN ? BM : BN) * ROWB;   // bytes of one ring slot (one operand, one block)
    constexpr int SPS = BK / 32;              // k-substeps (one MFMA k = 32 each) per block
    static_assert(TM % 16 == 0 && TN % 16 == 0, "wave tile must be a multiple of 16x16");

    extern __shared__ __align__(1024) uint8_t smem[];   // the slot ring; reused by the epilogue

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l16 = lane & 15, grp = lane >> 4;   // MFMA lane coordinates

    // ---- which work item ------------------------------------------------------------------
    int e, m0, n0, mvalid, nk;
    int row_tile = 0;                 // row GEMMs: number of this row tile over all segments
    int kbeg = 0, kend = 0;           // token contraction: perm rows of this item
    float* tok_out = nullptr;         // token contraction: where the tile goes
    if constexpr (!TOKENS) {
        const int tm_total = g.worklist[0];
        const int tn = ceil_div(g.N, BN);
        int tile_m, tile_n;
        {   // groups of kGroupM row tiles x all column tiles are dealt round-robin to the XCDs, so
            // the 8 XCDs work on neighbouring row tiles (mostly one expert) at any time; the last
            // ngroups % 8 groups are cut in eight instead, every XCD taking an eighth of each, so
            // that no XCD is a whole group behind the others at the end
            const int per_group = kGroupM * tn;
            const int ngroups = ceil_div(tm_total, kGroupM);
            const int xcd = item % kXcds, loc = item / kXcds;
            // rounds of eight whole groups; with many groups the last, partial round is dealt whole
            // as well (an XCD's CUs finish their tiles one tile-time apart either way, and whole
            // groups keep their L2 locality), with few the balance matters more
            const int whole = ngroups >= kSplitBelow ? ceil_div(ngroups, kXcds) : ngroups / kXcds;
            int group, within, share;
            if (loc < whole * per_group) {
                group = (loc / per_group) * kXcds + xcd;
                if (group >= ngroups) return;
                within = loc % per_group;
                share = per_group;
            } else {
                const int per8 = ceil_div(per_group, kXcds);
                const int l2 = loc - whole * per_group;
                group = whole * kXcds + l2 / per8;
                if (group >= ngroups) return;
                const int gtiles = min(kGroupM, tm_total - group * kGroupM) * tn;
                share = ceil_div(gtiles, kXcds);          // this XCD's tiles of the group
                if (l2 % per8 >= share) return;
                within = xcd * share + l2 % per8;
            }
            const int first = group * kGroupM;
            const int gsz = min(kGroupM, tm_total - first);
            if (within >= gsz * tn) return;
            tile_m = first + within % gsz;
            tile_n = within / gsz;
        }
        const i32x4 rt = *reinterpret_cast<const i32x4*>(g.worklist + 4 + 4 * tile_m);
        e = rt.x; m0 = rt.y; mvalid = rt.z; n0 = tile_n * BN; row_tile = tile_m;
        nk = g.K / BK;
    } else {
        // every (expert, chunk) item is a set of tm*tn tiles over the same tokens; each XCD takes
        // an eighth of every item's tiles (neighbouring ones), so the XCDs stay balanced however
        // uneven the experts are, and the whole chip streams the same token rows at a time
        const int tm = ceil_div(g.M, BM), tn = ceil_div(g.N, BN);
        const int tmn = tm * tn;
        const int per = ceil_div(tmn, kXcds);
        const int xcd = item % kXcds, loc = item / kXcds;
        const int tile = xcd * per + loc % per;
        if (tile >= tmn) return;
        if (loc / per >= g.worklist[1]) return;
        const i32x4 it = *reinterpret_cast<const i32x4*>(g.worklist + 4 + 4 * g.rt_cap + 4 * (loc / per));
        int tile_m, tile_n;
        grouped_tile(tile, tm, tn, tile_m, tile_n);
        e = it.x; m0 = tile_m * BM; n0 = tile_n * BN; mvalid = min(BM, g.M - m0);
        kbeg = it.y; kend = it.z;
        nk = ceil_div(kend - kbeg, BK);
        tok_out = (it.w >= 0) ? g.kpart + (size_t)it.w * g.M * g.N
                              : reinterpret_cast<float*>(g.out0) + (size_t)e * g.M * g.N;
    }
    const int nvalid = min(BN, g.N - n0);

    // ---- staging set-up -----------------------------------------------------------------------
    constexpr int NW = WM * WN;
    using SA = typename std::conditional<TOKENS, StageKS<BM, NW>, StageKC<BM, NW, OP == OP_FC1>>::type;
    using SB = typename std::conditional<B_KS, StageKS<BN, NW>, StageKC<BN, NW, false>>::type;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    typename SA::Lane lna;
    typename SB::Lane lnb;
    rsrc_t ra, rb;
    uint32_t a_step, b_step;      // bytes one K-step advances each operand
    uint32_t a_ld = 0, b_ld = 0;  // row pitch in bytes of the K-strided operands
    if constexpr (!TOKENS) {
        // FC1 gathers token rows of x through the re-index vector; the other row GEMMs read
        // perm-ordered rows, and rows past the segment fall outside the resource (zeros)
        if constexpr (OP == OP_FC1) ra = make_rsrc(g.A, (uint32_t)g.a_rows * (uint32_t)g.K * 2u);
        else ra = make_rsrc(g.A + (size_t)m0 * g.K, (uint32_t)mvalid * (uint32_t)g.K * 2u);
        a_step = BK * 2;
        const uint32_t ca = (uint32_t)SA::lane_chunk(uwave, lane) * 16u;
        if constexpr (OP == OP_FC1) {
#pragma unroll
            for (int i = 0; i < SA::NI; ++i) {
                const int r = SA::lane_row(uwave, lane, i);
                lna.voff[i] = (uint32_t)(g.perm[m0 + (r < mvalid ? r : 0)] / g.topk) * (uint32_t)g.K * 2u + ca;
            }
        } else {
            lna.voff[0] = (uint32_t)SA::lane_row(uwave, lane, 0) * (uint32_t)g.K * 2u + ca;
        }
        if constexpr (B_KS) {  // W[e][K][N]
            b_ld = (uint32_t)g.N * 2u;
            rb = make_rsrc(g.B + (size_t)e * g.K * g.N, (uint32_t)g.K * b_ld);
            b_step = BK * b_ld;
            lnb = SB::lane_init(uwave, lane, b_ld, n0);
        } else {               // W[e][N][K]: rows past N fall outside the resource
            rb = make_rsrc(g.B + ((size_t)e * g.N + n0) * g.K, (uint32_t)nvalid * (uint32_t)g.K * 2u);
            b_step = BK * 2;
            const uint32_t cb = (uint32_t)SB::lane_chunk(uwave, lane) * 16u;
            lnb.voff[0] = (uint32_t)SB::lane_row(uwave, lane, 0) * (uint32_t)g.K * 2u + cb;
        }
    } else {
        // both operands are [tokens][features] in perm order; tokens past this item's range fall
        // outside the resources
        // (WGRAD1: operand A is x itself, [tokens][M]; the row of perm position p comes from the
        // offset table, whose entries past a segment's end point behind the last row of x)
        a_ld = (uint32_t)g.M * 2u; b_ld = (uint32_t)g.N * 2u;
        if constexpr (A_GK) ra = make_rsrc(g.A, (uint32_t)g.a_rows * a_ld);
        else ra = make_rsrc(g.A + (size_t)kbeg * g.M, (uint32_t)(kend - kbeg) * a_ld);
        rb = make_rsrc(g.B + (size_t)kbeg * g.N, (uint32_t)(kend - kbeg) * b_ld);
        a_step = BK * a_ld; b_step = BK * b_ld;
        if constexpr (TOKENS) {
            lna = SA::lane_init(uwave, lane, A_GK ? 0u : a_ld, m0);
            lnb = SB::lane_init(uwave, lane, b_ld, n0);
        }
    }
    // staging instruction i_ of operand A / B for block kt_ into the ring slot at LDS byte address
    // slot_: set-up part (M0) and load part
    const uint32_t smem0 = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)smem;
    const uint32_t a_row = TOKENS ? a_ld : (uint32_t)g.K * 2u, b_row = B_KS ? b_ld : (uint32_t)g.K * 2u;
#define PREP_A(slot_, i_) SA::prep((slot_), uwave, i_)
#define PREP_B(slot_, i_) SB::prep((slot_), uwave, i_)
#define LOAD_A(kt_, i_)                                                                          \
    do {                                                                                         \
        if constexpr (A_GK) SA::load_gathered(ra, rcur, lna, i_);                                \
        else SA::load(ra, (kt_) * a_step, a_row, lna, i_);                                       \
    } while (0)
#define LOAD_B(kt_, i_) SB::load(rb, (kt_) * b_step, b_row, lnb, i_)

    // The bias values this lane adds in the epilogue (block j: columns j*16 + 4*grp + 0..3 of the
    // wave tile), fetched before the K loop: loaded in the epilogue they would be re-read after every
    // band's stores (which may alias them as far as the compiler knows), each time with the full
    // memory latency and nothing to hide it behind.  These plain loads are older than every staging
    // request, so the staging waits, which count from the youngest request back, cover them.
    u32x2 biasv[FN];
    if constexpr (OP == OP_FC1 || OP == OP_FC2) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int gc = min(n0 + wn * TN + j * 16 + 4 * grp, g.N - 4);   // masked columns read a valid bias
            biasv[j] = *reinterpret_cast<const u32x2*>(g.bias + (size_t)e * g.N + gc);
        }
    }

    // ---- per-lane fragment addresses -----------------------------------------------------------
    // A 16x16x32 MFMA operand fragment: lane (l16, grp) holds k = 8*grp + 0..7 of row (or column) l16
    // of its 16-wide block.
    // K-contiguous image: one 128-bit read of row (block row + l16), chunk (4*sub + grp) ^ key(l16)
    // (wave-tile and block rows are multiples of 16, so key(row) = key(l16)).
    // K-strided image: two transposing 64-bit reads per fragment.  In a group of 16 lanes, lane s
    // addresses k-row (s >> 2) and columns 4*(s & 3).., and receives column s of the block's 16,
    // k-rows 0..3; group grp reads k-rows 32*sub + 8*grp + 4*half + 0..3 (see StageKS).
    constexpr int A_RB = BM * 2, B_RB = BN * 2;  // LDS k-row pitch of the K-strided images
    // KC: aoff[sub] = byte offset of this lane's chunk in block row 0.
    // KS: one lane constant a_l0: k-row part | within-chunk byte | (chunk of block 0 ^ key) << 4.
    // Block q's chunk index differs from block 0's in bits 1..3 only (2q), the bits the key works
    // on, so its offset is a_l0 ^ (q << 5); the k-row of (substep, half) is an immediate.
    uint32_t aoff[SPS], boff[SPS];
    uint32_t a_l0 = 0, b_l0 = 0;
    {
        const int krel = l16 >> 2, pair = (l16 & 3) >> 1, half8 = (l16 & 1) * 8;
        const int key = ks_key(8 * grp + krel);  // the key of every k-row this lane reads
        static_assert(A_RB % 512 == 0 && B_RB % 512 == 0 && TM % 128 == 0 && TN % 128 == 0, "bit fields of the K-strided fragment offset");
        if constexpr (TOKENS) {
            a_l0 = (uint32_t)((8 * grp + krel) * A_RB + half8 + ((((wm * TM) / 8 + pair) ^ key) << 4));
        } else {
#pragma unroll
            for (int sb = 0; sb < SPS; ++sb)
                aoff[sb] = (uint32_t)((wm * TM + l16) * ROWB) + (uint32_t)(((4 * sb + grp) ^ lds_swz(l16)) << 4);
        }
        if constexpr (B_KS) {
            b_l0 = (uint32_t)((8 * grp + krel) * B_RB + half8 + ((((wn * TN) / 8 + pair) ^ key) << 4));
        } else {
#pragma unroll
            for (int sb = 0; sb < SPS; ++sb)
                boff[sb] = (uint32_t)((wn * TN + l16) * ROWB) + (uint32_t)(((4 * sb + grp) ^ lds_swz(l16)) << 4);
        }
    }

    // two fragment sets: one is multiplied while the other one is being read (a read never targets
    // registers an MFMA in flight may still be reading)
    bf16x8 fa0[FM], fb0[FN], fa1[FM], fb1[FN];
#define FENCE() __builtin_amdgcn_sched_barrier(0)
#define TR_READ(p_) __builtin_bit_cast(s16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p_)))
#define TR_JOIN(lo_, p_) __builtin_bit_cast(bf16x8, __builtin_shufflevector((lo_), TR_READ(p_), 0, 1, 2, 3, 4, 5, 6, 7))
    // The MFMAs of a substep run B-fragment-major (MFMA m = A fragment m % FM x B fragment m / FM),
    // so the next substep needs B fragment 0 and every A fragment first: its LDS reads are numbered
    // B0, A0 .. A(FM-1), B1 .. B(FN-1); a K-strided fragment takes two reads (k-rows +0..3 and
    // +4..7), a K-contiguous one takes one.
    constexpr int RA = TOKENS ? 2 : 1, RBn = B_KS ? 2 : 1;
    constexpr int NRD = FM * RA + FN * RBn;
    s16x4 trt;   // first half of the K-strided fragment being read
#define READ_A(fa, ab_, s_, q_, h_)                                                              \
    do {                                                                                         \
        if constexpr (TOKENS) {                                                                  \
            const uint8_t* p_ = (ab_) + (a_l0 ^ (uint32_t)((q_) << 5)) + (32 * (s_) + 4 * (h_)) * A_RB; \
            if ((h_) == 0) trt = TR_READ(p_);                                                    \
            else fa[q_] = TR_JOIN(trt, p_);                                                      \
        } else {                                                                                 \
            fa[q_] = *reinterpret_cast<const bf16x8*>((ab_) + aoff[s_] + (q_) * 16 * ROWB);       \
        }                                                                                        \
    } while (0)
#define READ_B(fb, bb_, s_, q_, h_)                                                              \
    do {                                                                                         \
        if constexpr (B_KS) {                                                                    \
            const uint8_t* p_ = (bb_) + (b_l0 ^ (uint32_t)((q_) << 5)) + (32 * (s_) + 4 * (h_)) * B_RB; \
            if ((h_) == 0) trt = TR_READ(p_);                                                    \
            else fb[q_] = TR_JOIN(trt, p_);                                                      \
        } else {                                                                                 \
            fb[q_] = *reinterpret_cast<const bf16x8*>((bb_) + boff[s_] + (q_) * 16 * ROWB);       \
        }                                                                                        \
    } while (0)
    // read number r_ of k-substep s_ from the slots at ab_ (A image) and bb_ (B image)
#define READ_ONE(fa, fb, ab_, bb_, s_, r_)                                                       \
    do {                                                                                         \
        if ((r_) < RBn) READ_B(fb, bb_, s_, 0, (r_));                                            \
        else if ((r_) < RBn + FM * RA) READ_A(fa, ab_, s_, ((r_) - RBn) / RA, ((r_) - RBn) % RA); \
        else if ((r_) < NRD) READ_B(fb, bb_, s_, 1 + ((r_) - RBn - FM * RA) / RBn, ((r_) - RBn - FM * RA) % RBn); \
    } while (0)

    constexpr int NM = FM * FN;   // MFMAs per k-substep and wave
    // Read r goes into memory slot (RSPAN * r) / NRD: the reads end a quarter substep before the
    // substep does, because the wave waits for all of them at the block barrier and at the loop head
    // (where the compiler merges its counters), and an LDS read issued just before would be waited
    // for in full.
    constexpr int RSPAN = NM * 3 / 4;
    static_assert(FM == 8 && FN == 8 && NRD <= RSPAN, "the issue slots are laid out for an 8 x 8 block grid");
    static_assert(SPS == 2, "the schedule below is written for two k-substeps per block");
    constexpr int NIA = SA::NI, NIB = SB::NI;    // staging instructions per wave, operand and block
    static_assert(NIA == 8 && NIB == 8, "one staging request per eight MFMAs");
    // A 16-cycle MFMA leaves the wave three more issue cycles, so no memory slot may hold more than
    // three instructions: fragment reads are spread evenly over the first three quarters, staging request o sits in the slots
    // 8 o + 1 (M0 set-up) and 8 o + 3 (load; the MFMA in between is the wait state M0 needs).
    // Operand A's requests go into substep 0, operand B's follow the block barrier in substep 1:
    // every wave has waited for its own fragment reads of the slot that is refilled (lgkmcnt) before
    // that barrier.
#define STAGE_AT(m_, PREP_, LOAD_, slot_, kt_)                                                   \
    do {                                                                                         \
        if ((m_) % 8 == 1) PREP_(slot_, (m_) / 8);                                               \
        if ((m_) % 8 == 3) LOAD_(kt_, (m_) / 8);                                                 \
    } while (0)
    // The MFMA gets the B fragment as its first and the A fragment as its second operand (both
    // have the same lane layout), so each 16x16 block comes out transposed: a lane then holds ONE
    // block row (l16) and the 4 consecutive block columns 4*grp + 0..3, which the epilogue stores
    // as 8- or 16-byte vectors.  (16x16x32 rather than 32x32x16: the same FLOP per cycle, but the
    // accumulator traffic per FLOP is half, and under the part's power limit the clock settles
    // higher.)
    // One k-substep: NM MFMAs on fragment set (fa, fb); after MFMA m, memory slot m is issued
    // (at most one fragment read for the next substep or one half of a staging request), so the
    // LDS and vector-memory queues are fed a little at a time while the matrix pipe stays busy:
    // one wavefront per SIMD has nobody else to hide a burst behind.
#define SUBSTEP(fa, fb, READ_, EXTRA_)                                                           \
    do {                                                                                         \
        _Pragma("unroll") for (int m = 0; m < NM; ++m) {                                         \
            if constexpr (F16)                                                                   \
                asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0"                            \
                             : "+a"(acc[m % FM][m / FM]) : "v"(fb[m / FM]), "v"(fa[m % FM]));    \
            else                                                                                 \
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"                           \
                             : "+a"(acc[m % FM][m / FM]) : "v"(fb[m / FM]), "v"(fa[m % FM]));    \
            FENCE();                                                                             \
            _Pragma("unroll") for (int r = 0; r < NRD; ++r)                                      \
                if ((RSPAN * r) / NRD == m) { READ_; }                                           \
            EXTRA_;                                                                              \
            FENCE();                                                                             \
        }                                                                                        \
    } while (0)
    static_assert(NIA + NIB <= 63, "vmcnt is a 6-bit counter");

    // The K loop runs in blocks of BK = 64 (two k-substeps): a row of a K-contiguous operand is
    // then one whole 128-byte line per block, and the texture-address path, which pays per line
    // touched, moves twice the bytes it would with 32-k stages.  One block of one operand (32 KB)
    // is a ring slot; the five slots of the 160 KB LDS hold, in request order,
    //     A(j) B(j) | A(j+1) B(j+1) A(j+2)       block j being multiplied | requested ahead
    // i.e. half-block h (A(j): h = 2j, B(j): h = 2j+1) lives in slot h % 5.
    // During block j: substep 0 requests A(j+2) into the slot B(j-1) left; before substep 1 the
    // wave waits until only that request is outstanding (so A(j+1), B(j+1) are complete) and the
    // barrier publishes them; every fragment read of block j has completed by then, so substep 1
    // requests B(j+2) into A(j)'s slot while it reads the first fragments of block j+1.  Past the
    // last block the requests re-fetch the last block into slots nobody reads, which keeps the
    // loop body free of branches.
    // nk >= 1: K is at least one block in the row GEMMs, and a token-contraction item holds at least
    // one row.  The K loop is bottom-tested for that reason: with a zero-trip path the accumulators
    // of the two paths meet behind the loop, and the register allocator shuffles them there.
    const int klast = nk - 1;
    // WGRAD1: the byte offsets in x of the eight token rows this lane fetches per K-block (instruction
    // i of a wave covers the block's rows 8 i + 2 wave + lane / 32; the table stores a block's 64
    // offsets transposed, so those eight are 32 consecutive bytes).  rcur holds the offsets of the
    // block requested next (block j + 2 during block j); those of the block after it are loaded at
    // the head of block j and taken over at the wait in its middle, which covers them because they
    // are older than operand A's requests of that block.  The loads are inline assembly like the
    // staging requests (own counting of vmcnt).  Their results are tied to the wait statement, so
    // nothing can read them in front of it, and they do not live across the loop's back edge, where
    // the compiler would copy them (before they have arrived).
    uint32_t rcur[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    const uint32_t* rbase = nullptr;   // this item's first table entry (wave-uniform)
    const uint32_t rl_off = (uint32_t)(8 * (2 * uwave + (lane >> 5))) * 4u;   // this lane's eight entries of a block
    auto roff_request = [&](int kt, u32x4& lo, u32x4& hi) __attribute__((always_inline)) {
        const uint32_t* p_ = rbase + (size_t)64 * kt;   // scalar base + lane offset: no vector arithmetic per block
        asm volatile("global_load_dwordx4 %0, %2, %3\n\tglobal_load_dwordx4 %1, %2, %3 offset:16"
                     : "=&v"(lo), "=&v"(hi) : "v"(rl_off), "s"(p_) : "memory");
    };
#define ROFF_TAKE(lo_, hi_)                                                                       \
    do {                                                                                          \
        rcur[0] = (lo_)[0]; rcur[1] = (lo_)[1]; rcur[2] = (lo_)[2]; rcur[3] = (lo_)[3];           \
        rcur[4] = (hi_)[0]; rcur[5] = (hi_)[1]; rcur[6] = (hi_)[2]; rcur[7] = (hi_)[3];           \
    } while (0)
    {
        const uint32_t k1 = (uint32_t)min(1, klast);
        u32x4 r0_lo, r0_hi, r1_lo, r1_hi, r2_lo, r2_hi;
        if constexpr (A_GK) {
            rbase = g.rowoff + (size_t)kbeg + (size_t)64 * e;
            roff_request(0, r0_lo, r0_hi);
            roff_request((int)k1, r1_lo, r1_hi);
            roff_request(min(2, klast), r2_lo, r2_hi);
            asm volatile("s_waitcnt vmcnt(0)"
                         : "+v"(r0_lo), "+v"(r0_hi), "+v"(r1_lo), "+v"(r1_hi), "+v"(r2_lo), "+v"(r2_hi) : : "memory");
            ROFF_TAKE(r0_lo, r0_hi);
        }
        _Pragma("unroll") for (int o = 0; o < NIA; ++o) { PREP_A(smem0 + 0 * SLOT, o); asm volatile("s_nop 0"); LOAD_A(0u, o); }
        _Pragma("unroll") for (int o = 0; o < NIB; ++o) { PREP_B(smem0 + 1 * SLOT, o); asm volatile("s_nop 0"); LOAD_B(0u, o); }
        if constexpr (A_GK) ROFF_TAKE(r1_lo, r1_hi);
        _Pragma("unroll") for (int o = 0; o < NIA; ++o) { PREP_A(smem0 + 2 * SLOT, o); asm volatile("s_nop 0"); LOAD_A(k1, o); }
        _Pragma("unroll") for (int o = 0; o < NIB; ++o) { PREP_B(smem0 + 3 * SLOT, o); asm volatile("s_nop 0"); LOAD_B(k1, o); }
        if constexpr (A_GK) ROFF_TAKE(r2_lo, r2_hi);
    }
    // The accumulators are cleared here, between the first requests and the wait for them: claimed
    // in their accumulation registers by the empty statements (which keep their place among the
    // other volatile statements), the 256 writes run while the first block is on its way instead of
    // after it has arrived.
    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jj = 0; jj < FN; ++jj) {
            acc[i][jj] = f32x4{0.f, 0.f, 0.f, 0.f};
            asm volatile("" : "+a"(acc[i][jj]));
        }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NIA + NIB) : "memory");
    __syncthreads();
    int sa = 0, sb = 1;                           // slots of A(j), B(j)
    int j = 0;
    if constexpr (!TOKENS) {
        // A wave whose 128 rows all lie past the segment's end (the lower half of a tail tile with
        // at most 128 rows) has nothing to multiply: it keeps its share of the staging requests and
        // the barriers, and skips the fragment reads, the MFMAs and the epilogue.  The time of the
        // tile is the other waves'; what is saved is energy, which is what this part runs short of.
        if (__builtin_amdgcn_readfirstlane(mvalid - wm * TM) <= 0) {
            do {
                const int sa1 = sa + 2 >= NSLOT ? sa + 2 - NSLOT : sa + 2;
                const int sb1 = sb + 2 >= NSLOT ? sb + 2 - NSLOT : sb + 2;
                const int sa2 = sa + 4 >= NSLOT ? sa + 4 - NSLOT : sa + 4;
                const uint32_t a2 = smem0 + (uint32_t)(sa2 * SLOT), b2 = smem0 + (uint32_t)(sa * SLOT);
                const uint32_t kreq = (uint32_t)min(j + 2, klast);
                _Pragma("unroll") for (int o = 0; o < NIA; ++o) { PREP_A(a2, o); asm volatile("s_nop 0"); LOAD_A(kreq, o); }
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NIA) : "memory");
                __syncthreads();
                _Pragma("unroll") for (int o = 0; o < NIB; ++o) { PREP_B(b2, o); asm volatile("s_nop 0"); LOAD_B(kreq, o); }
                sa = sa1; sb = sb1;
            } while (++j < nk);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();   // the barrier in front of the other waves' epilogue
            if constexpr (OP == OP_DGRAD2) {   // this wave's column-sum partials: no rows, zeros
                const int col = wn * TN + 2 * lane;
                if (col < nvalid)
                    *reinterpret_cast<float2*>(g.colpart + (size_t)(row_tile * WM + wm) * (size_t)g.N + n0 + col) =
                        make_float2(0.f, 0.f);
            }
            return;
        }
    }
    _Pragma("unroll") for (int r = 0; r < NRD; ++r) READ_ONE(fa0, fb0, smem, smem + SLOT, 0, r);

    do {
        uint8_t* abase = smem + sa * SLOT;
        uint8_t* bbase = smem + sb * SLOT;
        const int sa1 = sa + 2 >= NSLOT ? sa + 2 - NSLOT : sa + 2;
        const int sb1 = sb + 2 >= NSLOT ? sb + 2 - NSLOT : sb + 2;
        const int sa2 = sa + 4 >= NSLOT ? sa + 4 - NSLOT : sa + 4;
        uint8_t* anext = smem + sa1 * SLOT;
        uint8_t* bnext = smem + sb1 * SLOT;
        const uint32_t a2 = smem0 + (uint32_t)(sa2 * SLOT);   // A(j+2): the slot of B(j-1)
        const uint32_t b2 = smem0 + (uint32_t)(sa * SLOT);    // B(j+2): the slot of A(j)
        const uint32_t kreq = (uint32_t)min(j + 2, klast);
        u32x4 rn_lo, rn_hi;
        uint32_t rnx[8];   // the same eight values once they have arrived
        if constexpr (A_GK) roff_request(min(j + 3, klast), rn_lo, rn_hi);
        FENCE();
        SUBSTEP(fa0, fb0, READ_ONE(fa1, fb1, abase, bbase, 1, r), STAGE_AT(m, PREP_A, LOAD_A, a2, kreq));
        if constexpr (A_GK) {
            asm volatile("s_waitcnt vmcnt(%2)" : "+v"(rn_lo), "+v"(rn_hi) : "n"(NIA) : "memory");
            rnx[0] = rn_lo[0]; rnx[1] = rn_lo[1]; rnx[2] = rn_lo[2]; rnx[3] = rn_lo[3];
            rnx[4] = rn_hi[0]; rnx[5] = rn_hi[1]; rnx[6] = rn_hi[2]; rnx[7] = rn_hi[3];
        } else {
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NIA) : "memory");
        }
        __syncthreads();
        FENCE();
        // (WGRAD1 takes the new row offsets over one register per eighth of the substep, each copy in
        // an issue slot of its own: left to the compiler, the eight copies sit in a row at the
        // loop's back edge, two MFMAs' worth of issue cycles)
#define TAKE_AT(m_)                                                                               \
    do {                                                                                          \
        if constexpr (A_GK) {                                                                     \
            if ((m_) % 8 == 5)                                                                    \
                asm volatile("v_mov_b32 %0, %1" : "=v"(rcur[(m_) / 8]) : "v"(rnx[(m_) / 8]));     \
        }                                                                                         \
    } while (0)
        SUBSTEP(fa1, fb1, READ_ONE(fa0, fb0, anext, bnext, 0, r), STAGE_AT(m, PREP_B, LOAD_B, b2, kreq); TAKE_AT(m));
#undef TAKE_AT
        sa = sa1; sb = sb1;
    } while (++j < nk);
    // no staging write may still be in flight when the workgroup gives its LDS back
    // (the MFMAs are inline assembly, so the compiler does not count the wait states their results
    // need before the epilogue reads the accumulators: 16 idle cycles cover the 4-pass MFMA)
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    // pin every accumulator to its accumulation register at the loop exit (keeps the register
    // allocator from shuffling them between the loop and the epilogue)
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jj = 0; jj < FN; ++jj) asm volatile("" : "+a"(acc[i][jj]));
#undef STAGE_AT
#undef ROFF_TAKE
#undef SUBSTEP
#undef READ_ONE
#undef READ_A
#undef READ_B
#undef TR_JOIN
#undef TR_READ
#undef FENCE
#undef PREP_A
#undef PREP_B
#undef LOAD_A
#undef LOAD_B

    // ---- epilogue ------------------------------------------------------------------------------
    // In block (i, j) a lane holds row i*16 + l16 and the four columns j*16 + 4*grp + 0..3.  Stored
    // from there, a wave instruction would touch 16 rows with 8 or 16 bytes each.  Instead each
    // wave turns one 16-row band (i) at a time through its own 32 KB of the (now idle) ring:
    // vectors are written at [row][chunk ^ row] (16-byte chunks, so both directions are
    // conflict-free), read back with a lane per 16-byte chunk of a row, and leave as full 256- or
    // 512-byte row segments.  DGRAD2's saved activation derivatives come in the same way, staged
    // one band ahead.
    __syncthreads();   // every wave is done reading fragments
    {
        uint8_t* wreg = smem + uwave * 32768;
        constexpr bool OUT_F32 = TOKENS;   // weight gradients; every activation-like output is 16-bit
        constexpr int ESZ = OUT_F32 ? 4 : 2;
        constexpr int RPB = TN * ESZ;                 // bytes per staged row (TN columns)
        constexpr int CPRO = RPB / 16;                // 16-byte chunks per staged row
        constexpr int BAND = 16;                      // rows per band = rows of an MFMA block
        constexpr int H_OFF = BAND * RPB;             // FC1: second output of a band, behind the first
        constexpr int G_OFF = 16384, G_BUF = BAND * 256;   // DGRAD2: two bands of saved derivatives
        static_assert(TN == 128, "epilogue staging is laid out for 128-column wave tiles");
        const size_t ldo = (size_t)g.N;
        const int wrow0 = wm * TM, wcol0 = wn * TN;
        // DGRAD2: stage the saved F'(pre)[band][128 cols] (16-bit, 256 B rows, chunk ^ (row & 15))
        // with direct loads; instruction t covers rows 4t..4t+3
        constexpr int GI = BAND / 4;                  // staging instructions per band
        rsrc_t rp;
        uint32_t pre_voff = 0;
        if constexpr (OP == OP_DGRAD2) {
            rp = make_rsrc(g.pre_in + (size_t)m0 * ldo, (uint32_t)mvalid * (uint32_t)ldo * 2u);
            pre_voff = (uint32_t)((wrow0 + (lane >> 4)) * (int)ldo + n0 + wcol0) * 2u;
        }
        auto stage_pre = [&](int band, int buf) {
            if constexpr (OP == OP_DGRAD2) {
#pragma unroll
                for (int t = 0; t < GI; ++t) {
                    const int row = 4 * t + (lane >> 4);
                    const int c = (lane & 15) ^ (row & 15);
                    dtl16(rp, wreg + G_OFF + buf * G_BUF + t * 1024,
                          pre_voff + (uint32_t)((band * BAND + 4 * t) * (int)ldo + c * 8) * 2u, 0u);
                }
            }
        };
        // Output window of this wave: a buffer resource from (first row, first column) of the wave
        // tile to the end of its last valid row, so stores to rows past the segment are dropped by
        // the range check; a lane whose 16-byte chunk lies past the last valid column gets an
        // offset outside any window.  Instruction t of a band stores rows RPI_O*t + lane/CPRO; the
        // chunk a lane holds there is (lane % CPRO) ^ row = c0 ^ (RPI_O*t) (row < 16, RPI_O*t has
        // no bit in common with lane/CPRO), so the per-lane offsets of the NST instructions are the
        // same for every band and the band's row offset is a scalar.
        constexpr int RPI_O = 1024 / RPB;            // rows per store instruction
        constexpr int NST = BAND / RPI_O;            // store instructions per band and output
        const int mv_w = min(TM, mvalid - wrow0), nv_w = min(TN, nvalid - wcol0);
        const int obytes = __builtin_amdgcn_readfirstlane(
            (mv_w > 0 && nv_w > 0) ? ((mv_w - 1) * (int)ldo + nv_w) * ESZ : 0);
        const size_t o0 = ((size_t)(m0 + wrow0) * ldo + (size_t)(n0 + wcol0)) * ESZ;
        // (wave-uniform, but derived from the wave number: say so, or every store is wrapped in a loop
        // over the distinct resources of the lanes)
        auto uniform_ptr = [](uint8_t* p_) {
            const uint64_t b = (uint64_t)p_;
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
            return (uint8_t*)(((uint64_t)hi << 32) | lo);
        };
        uint8_t* obase0 = TOKENS ? reinterpret_cast<uint8_t*>(tok_out) : reinterpret_cast<uint8_t*>(g.out0);
        const __amdgpu_buffer_rsrc_t ro0 = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(obase0 + o0), 0, obytes, 0x00020000);
        __amdgpu_buffer_rsrc_t ro1 = ro0;
        if constexpr (OP == OP_FC1)
            ro1 = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(reinterpret_cast<uint8_t*>(g.out1) + o0), 0, obytes, 0x00020000);
        const int ldo_b = __builtin_amdgcn_readfirstlane((int)ldo * ESZ);   // bytes per output row
        int ovoff[NST];
        {
            const int q = lane / CPRO, c0 = (lane % CPRO) ^ q;
#pragma unroll
            for (int t = 0; t < NST; ++t) {
                const int c = c0 ^ (RPI_O * t);
                ovoff[t] = c * 16 < nv_w * ESZ ? q * (int)ldo * ESZ + c * 16 : (int)0x80000000;
            }
        }
        stage_pre(0, 0);
        float cs0 = 0.f, cs1 = 0.f;   // DGRAD2: sums of columns 2*lane, 2*lane+1 over this wave's rows (ESS, Table 5 row 8)
        // The bands run as a two-stage pipeline over two LDS band buffers: the reads that fetch band
        // i-1 back from LDS are issued before the arithmetic of band i and their results are stored
        // (and, DGRAD2, added up) after it, so neither the write-to-read turn-around of LDS nor the
        // latency of the reads is waited for.  LDS executes a wave's instructions in order, so the
        // writes of band i+1 cannot overtake the reads of band i-1 from the same buffer.
        constexpr int BAND_BYTES = BAND * RPB;
        constexpr int BUF_STRIDE = (OP == OP_FC1 ? 2 : 1) * BAND_BYTES;   // FC1 stages two outputs per band
        static_assert(H_OFF == BAND_BYTES && 2 * BUF_STRIDE <= G_OFF, "band buffers overlap");
        u32x4 d0[NST], d1[OP == OP_FC1 ? NST : 1];
        uint32_t cw[OP == OP_DGRAD2 ? BAND : 1];
        auto band_reads = [&](int buf) __attribute__((always_inline)) {
            uint8_t* wb = wreg + buf * BUF_STRIDE;
#pragma unroll
            for (int t = 0; t < NST; ++t) {
                d0[t] = *reinterpret_cast<const u32x4*>(wb + t * 1024 + lane * 16);
                if constexpr (OP == OP_FC1) d1[t] = *reinterpret_cast<const u32x4*>(wb + H_OFF + t * 1024 + lane * 16);
            }
            if constexpr (OP == OP_DGRAD2) {
                // bias-gradient partial: the band holds the rounded dpre values the weight gradient
                // will read; rows past the segment and columns past N are exact zeros
#pragma unroll
                for (int row = 0; row < BAND; ++row)
                    cw[row] = *reinterpret_cast<const uint32_t*>(
                        wb + row * RPB + ((((lane >> 2) ^ row)) << 4) + (lane & 3) * 4);
            }
        };
        auto band_store_one = [&](int i, int t) __attribute__((always_inline)) {
            const int soff = (i * BAND + RPI_O * t) * ldo_b;
            __builtin_amdgcn_raw_buffer_store_b128(d0[t], ro0, ovoff[t], soff, 0);
            if constexpr (OP == OP_FC1) __builtin_amdgcn_raw_buffer_store_b128(d1[t], ro1, ovoff[t], soff, 0);
        };
        auto band_stores = [&](int i, bool with_stores) __attribute__((always_inline)) {
            if (with_stores) {
#pragma unroll
                for (int t = 0; t < NST; ++t) band_store_one(i, t);
            }
            if constexpr (OP == OP_DGRAD2) {
#pragma unroll
                for (int row = 0; row < BAND; ++row) {
                    float c0, c1;
                    unpack2<F16>(cw[row], c0, c1);
                    cs0 += c0; cs1 += c1;
                }
            }
        };
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            uint8_t* wb = wreg + (i & 1) * BUF_STRIDE;
            if (i > 0) band_reads((i - 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (OP == OP_DGRAD2) {
                // the next band's derivatives are requested before this band's are awaited; the
                // counter also holds stores of earlier bands, which are older than both
                if (i + 1 < FM) stage_pre(i + 1, (i + 1) & 1);
                if (i + 1 < FM) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(GI) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            // -- registers -> LDS band
            // (the band's accumulators are claimed in their accumulation registers at this point:
            // otherwise the register allocator permutes and copies a few hundred of them ahead of
            // the first band)
#pragma unroll
            for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = j * 16 + 4 * grp;                  // column inside the wave tile
                f32x4 v = acc[i][j];
                if constexpr (OP == OP_FC1 || OP == OP_FC2) {
                    const u32x2 bb = biasv[j];
                    float b0, b1, b2, b3;
                    unpack2<F16>(bb.x, b0, b1); unpack2<F16>(bb.y, b2, b3);
                    v[0] += b0; v[1] += b1; v[2] += b2; v[3] += b3;
                }
                if constexpr (OUT_F32) {
                    // straight from the accumulation registers (an LDS store may take its data from
                    // them; through ordinary registers it is 256 more copies per wave and tile)
                    const int c = col >> 2;
                    const uint32_t la = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)(wb + l16 * RPB + ((c ^ l16) << 4));
                    asm volatile("ds_write_b128 %0, %1" : : "v"(la), "a"(acc[i][j]) : "memory");
                } else {
                    const int c = col >> 3;
                    const uint32_t off = (uint32_t)(l16 * RPB + ((c ^ l16) << 4) + (grp & 1) * 8);
                    if constexpr (OP == OP_FC1) {
                        float hh[4], gg[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) act_both<ACT>(v[r], hh[r], gg[r]);
                        u32x2 pz, hz;
                        pz.x = pack2<F16>(gg[0], gg[1]); pz.y = pack2<F16>(gg[2], gg[3]);
                        hz.x = pack2<F16>(hh[0], hh[1]); hz.y = pack2<F16>(hh[2], hh[3]);
                        *reinterpret_cast<u32x2*>(wb + off) = pz;
                        *reinterpret_cast<u32x2*>(wb + H_OFF + off) = hz;
                    } else if constexpr (OP == OP_FC2 || OP == OP_DGRAD1) {
                        u32x2 z;
                        z.x = pack2<F16>(v[0], v[1]); z.y = pack2<F16>(v[2], v[3]);
                        *reinterpret_cast<u32x2*>(wb + off) = z;
                    } else {   // DGRAD2
                        const u32x2 pp = *reinterpret_cast<const u32x2*>(wreg + G_OFF + (i & 1) * G_BUF + off);
                        float p0, p1, p2, p3;
                        unpack2<F16>(pp.x, p0, p1); unpack2<F16>(pp.y, p2, p3);
                        u32x2 d;
                        d.x = pack2<F16>(v[0] * p0, v[1] * p1);
                        d.y = pack2<F16>(v[2] * p2, v[3] * p3);
                        *reinterpret_cast<u32x2*>(wb + off) = d;
                    }
                }
                // the previous band's stores go out one at a time between the blocks of this band's
                // arithmetic: issued in a row behind it they fill the address queue of the texture
                // unit and the wave waits (5 % of fc1's cycles)
                if (i > 0 && j % (FN / NST) == FN / NST - 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    band_store_one(i - 1, j / (FN / NST));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (i > 0) band_stores(i - 1, false);   // (DGRAD2: the previous band's column sums)
        }
        band_reads((FM - 1) & 1);
        band_stores(FM - 1, true);
        if constexpr (OP == OP_DGRAD2) {
            const int col = wcol0 + 2 * lane;
            if (col < nvalid)
                *reinterpret_cast<float2*>(g.colpart + (size_t)(row_tile * WM + wm) * ldo + n0 + col) =
                    make_float2(cs0, cs1);
        }
    }
}

template <int BM, int BN, int WM, int WN, int OP, int ACT = HEXA_ACT_GELU_TANH, bool F16 = false>
__global__ __launch_bounds__(WM * WN * 64, 1) void gemm_bf16(GemmArgs g) {
    gemm_tile<BM, BN, WM, WN, OP, ACT, F16>(g, (int)blockIdx.x);
}

// Two independent contractions in one grid (the paper's fused backward kernel, Sec. 3.2 "Fused
// Kernel in Backward Propagation": the input gradient and the weight gradient of one linear layer
// do not depend on each other), so the tail of one fills with tiles of the other.  Both item counts
// are multiples of 8 (XCD mapping).  Workgroups start roughly in slot order, so the contraction
// with the longer tiles should come first: normally the row GEMM OPA (slots [0, items_a)), but the
// token contraction OPB when routing is so skewed that one expert's chunk runs many times longer
// than a row-GEMM tile (flag `order` of the work-list header, set by build_worklists; with Zipf
// routing at C5's shape the largest expert's tiles run 1582 K-blocks against 32 or 128).
template <int BM, int BN, int WM, int WN, int OPA, int OPB, bool F16 = false>
__global__ __launch_bounds__(WM * WN * 64, 1) void gemm_bf16_pair(GemmArgs ga, GemmArgs gb, int items_a, int order) {
    const int item = (int)blockIdx.x;
    const int items_b = (int)gridDim.x - items_a;
    const bool b_first = ga.worklist[order] != 0;
    const bool is_b = b_first ? item < items_b : item >= items_a;
    const int local = b_first ? (is_b ? item : item - items_b) : (is_b ? item - items_a : item);
    if (is_b) gemm_tile<BM, BN, WM, WN, OPB, HEXA_ACT_GELU_TANH, F16>(gb, local);
    else gemm_tile<BM, BN, WM, WN, OPA, HEXA_ACT_GELU_TANH, F16>(ga, local);
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
    const size_t stride = (size_t)gridDim.x * 256;
    // four elements per thread and pass, their loads issued together (one at a time, the few
    // workgroups of a split expert are a chain of memory latencies)
    for (size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x; i0 < n4; i0 += 4 * stride) {
        float4 s[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) s[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c = 0; c < nch; ++c) {
            const float4* src = reinterpret_cast<const float4*>(kpart + (size_t)(slot + c) * mn);
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = i0 + u * stride < n4 ? src[i0 + u * stride] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 4; ++u) { s[u].x += v[u].x; s[u].y += v[u].y; s[u].z += v[u].z; s[u].w += v[u].w; }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u * stride < n4) dst[i0 + u * stride] = s[u];
    }
}

constexpr int kNumCUs = 256;

// Work-item slots of a row GEMM with at most tm_max row tiles and tn column tiles (a multiple of 8):
// per XCD, enough for either way of dealing the last groups (see gemm_tile).
inline int row_gemm_slots(int tm_max, int tn) {
    const int per_group = kGroupM * tn;
    const int ngroups = ceil_div(tm_max, kGroupM);
    const int split = (ngroups / kXcds) * per_group + (kXcds - 1) * ceil_div(per_group, kXcds);
    const int whole = ceil_div(ngroups, kXcds) * per_group;
    return kXcds * (split > whole ? split : whole);
}

template <int BM, int BN, int WM, int WN, int OP, int ACT = HEXA_ACT_GELU_TANH, bool F16 = false>
void launch_rows(const MoeDims& D, const GemmArgs& g, hipStream_t st, const char* label) {
    ProfScope ps(st, label);
    auto kern = gemm_bf16<BM, BN, WM, WN, OP, ACT, F16>;
    constexpr int lds = NSLOT * (BM > BN ? BM : BN) * ROWB;
    const int tm_max = D.A / BM + D.E;
    const int grid = row_gemm_slots(tm_max, ceil_div(g.N, BN));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds, st, g);
}

// Row GEMM OPA and token contraction OPB of one linear layer's backward in one grid, then the
// split-K finisher of OPB.
template <int BM, int BN, int WM, int WN, int OPA, int OPB, bool F16 = false>
void launch_pair(const MoeDims& D, const GemmArgs& ga, const GemmArgs& gb, hipStream_t st,
                 const char* label, const char* label_fin) {
    auto kern = gemm_bf16_pair<BM, BN, WM, WN, OPA, OPB, F16>;
    constexpr int lds = NSLOT * (BM > BN ? BM : BN) * ROWB;
    const int tm_max = D.A / BM + D.E;
    const int items_a = row_gemm_slots(tm_max, ceil_div(ga.N, BN));
    const int tmn = ceil_div(gb.M, BM) * ceil_div(gb.N, BN);
    const int items_b = kXcds * ceil_div(tmn, kXcds) * (D.A / gb.chunk_len + D.E);
    {
        ProfScope ps(st, label);
        hipLaunchKernelGGL(kern, dim3(items_a + items_b), dim3(WM * WN * 64), lds, st, ga, gb, items_a,
                           OPB == OP_WGRAD2 ? 2 : 3);
    }
    ProfScope ps(st, label_fin);
    const size_t mn = (size_t)gb.M * gb.N;
    const int gx = (int)((mn / 4 + 255) / 256 < 1024 ? (mn / 4 + 255) / 256 : 1024);
    hipLaunchKernelGGL(wgrad_finish, dim3(gx, D.E), dim3(256), 0, st, gb.offsets, D.E, gb.chunk_len, mn,
                       gb.kpart, reinterpret_cast<float*>(gb.out0));
}

constexpr int TBM = 256, TBN = 256, TWM = 2, TWN = 2;

}  // namespace

// Every contraction kernel needs the whole 160 KB of LDS as dynamic shared memory, which a kernel
// may only use after its attribute has been raised, once per device.
template <typename K>
static hipError_t allow_full_lds(K kern) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, NSLOT * TBM * ROWB);
}
template <bool F16>
static hipError_t device_init_dtype() {
    hipError_t e = allow_full_lds(gemm_bf16<TBM, TBN, TWM, TWN, OP_FC1, HEXA_ACT_GELU_TANH, F16>);
    if (e == hipSuccess) e = allow_full_lds(gemm_bf16<TBM, TBN, TWM, TWN, OP_FC1, HEXA_ACT_RELU, F16>);
    if (e == hipSuccess) e = allow_full_lds(gemm_bf16<TBM, TBN, TWM, TWN, OP_FC1, HEXA_ACT_SILU, F16>);
    if (e == hipSuccess) e = allow_full_lds(gemm_bf16<TBM, TBN, TWM, TWN, OP_FC2, HEXA_ACT_GELU_TANH, F16>);
    if (e == hipSuccess) e = allow_full_lds(gemm_bf16_pair<TBM, TBN, TWM, TWN, OP_DGRAD2, OP_WGRAD2, F16>);
    if (e == hipSuccess) e = allow_full_lds(gemm_bf16_pair<TBM, TBN, TWM, TWN, OP_DGRAD1, OP_WGRAD1, F16>);
    return e;
}
hipError_t gemm_bf16_device_init() {
    static_assert(TBM == TBN, "one LDS size for all instantiations");
    const hipError_t e = device_init_dtype<false>();
    return e != hipSuccess ? e : device_init_dtype<true>();
}

// Row-tile height and partial rows per tile of the DGRAD2 column-sum partials (for the finisher).
int gemm_row_tile() { return TBM; }
int gemm_colpart_rows_per_tile() { return TWM; }

// Tokens per split-K chunk of the token contractions: an expert is cut only when its rows alone
// would give every CU a tile's worth of work for longer than the whole contraction takes on
// average (chunk = the rows that make one tile per CU of the chip: A * tiles / CUs).  Shorter chunks
// balance no better, because the grid is shared with the row GEMM of the same layer, whose tiles
// fill the gaps, and every extra chunk costs a partial d x f tile written and read back (measured:
// a quarter of this length made C3 5.6 %, C4 1.9 % and C5 under Zipf routing 0.5 % slower; half
// as many chunks again made C3 and C4 slower).
int wgrad_chunk_len(const MoeDims& D) {
    const long long tmn = (long long)ceil_div(D.d, TBM) * ceil_div(D.f, TBN);
    long long L = (long long)D.A * tmn / kNumCUs;
    L = (L + 63) / 64 * 64;
    if (L < 1024) L = 1024;
    // one item's rows are addressed with 32-bit byte offsets: L * max(d, f) * 2 < 2^32
    const long long cap = (0xffffffffLL / (2LL * (D.d > D.f ? D.d : D.f))) / 64 * 64;
    if (L > cap) L = cap;
    return (int)L;
}

// Capacities of the work lists (see build_worklists): row tiles, token-contraction items.
static int worklist_rt_cap(const MoeDims& D) { return D.A / TBM + D.E; }
static int worklist_it_cap(const MoeDims& D) { return D.A / wgrad_chunk_len(D) + D.E; }
size_t gemm_worklist_ints(const MoeDims& D) {
    return 4 + 4 * (size_t)worklist_rt_cap(D) + 4 * (size_t)worklist_it_cap(D);
}
static void launch_worklists(const MoeDims& D, const hexa_moe_idx& idx, const MoeWorkspace& ws, hipStream_t st) {
    ProfScope ps(st, "worklists");
    hipLaunchKernelGGL(build_worklists, dim3(1), dim3(1024), 0, st, idx.offsets, D.E, TBM,
                       wgrad_chunk_len(D), ws.worklist, worklist_rt_cap(D), D.d, D.f);
}

// Upper bound on split-K slots: only experts with more than one chunk use slots, and
// sum over those of ceil(n_e / L) <= 2 A / L.
size_t wgrad_max_slots(const MoeDims& D) {
    return 2 * (size_t)(D.A / wgrad_chunk_len(D)) + 2;
}

template <bool F16>
static hipError_t fwd_impl(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* b1,
                           const bf16_t* W2, const bf16_t* b2, const hexa_moe_idx& idx,
                           const MoeWorkspace& ws, hipStream_t st) {
    GemmArgs g{};
    g.offsets = idx.offsets; g.perm = idx.perm; g.topk = D.k; g.E = D.E;
    g.worklist = ws.worklist; g.rt_cap = worklist_rt_cap(D);
    launch_worklists(D, idx, ws, st);
    g.A = x; g.a_rows = D.T; g.B = W1; g.bias = b1; g.out0 = ws.pre; g.out1 = ws.h; g.K = D.d; g.N = D.f;
    if (D.act == HEXA_ACT_RELU) launch_rows<TBM, TBN, TWM, TWN, OP_FC1, HEXA_ACT_RELU, F16>(D, g, st, "fc1");
    else if (D.act == HEXA_ACT_SILU) launch_rows<TBM, TBN, TWM, TWN, OP_FC1, HEXA_ACT_SILU, F16>(D, g, st, "fc1");
    else launch_rows<TBM, TBN, TWM, TWN, OP_FC1, HEXA_ACT_GELU_TANH, F16>(D, g, st, "fc1");
    g.A = (const bf16_t*)ws.h; g.B = W2; g.bias = b2; g.out0 = ws.o; g.out1 = nullptr; g.K = D.f; g.N = D.d;
    launch_rows<TBM, TBN, TWM, TWN, OP_FC2, HEXA_ACT_GELU_TANH, F16>(D, g, st, "fc2");
    return hipGetLastError();
}

template <bool F16>
static hipError_t bwd_impl(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* W2,
                           const hexa_moe_idx& idx, const MoeWorkspace& ws, float* dW1, float* dW2,
                           hipStream_t st) {
    GemmArgs g{};
    g.offsets = idx.offsets; g.perm = idx.perm; g.topk = D.k; g.E = D.E;
    g.kpart = ws.kpart; g.chunk_len = wgrad_chunk_len(D);
    // the work lists are the ones the forward pass built (part of the state it saves in the workspace)
    g.worklist = ws.worklist; g.rt_cap = worklist_rt_cap(D);
    {   // WGRAD1's row-offset table; entries past a segment's end point behind the last row of x
        ProfScope ps(st, "rowoff");
        const int total = D.A + 64 * D.E;
        hipLaunchKernelGGL(build_rowoff, dim3(ceil_div(total, 256)), dim3(256), 0, st, idx.offsets, idx.perm,
                           D.E, D.k, (uint32_t)D.d * 2u, (uint32_t)D.T * (uint32_t)D.d * 2u, total, ws.rowoff);
    }
    // 2nd linear layer: dpre = (do W2^T) * F'(pre)  and  dW2[e] = h^T do
    GemmArgs r = g, t = g;
    r.A = (const bf16_t*)ws.dout; r.B = W2; r.pre_in = (const bf16_t*)ws.pre; r.out0 = ws.dpre;
    r.colpart = ws.colpart; r.K = D.d; r.N = D.f;
    t.A = (const bf16_t*)ws.h; t.B = (const bf16_t*)ws.dout; t.out0 = dW2; t.M = D.f; t.N = D.d;
    launch_pair<TBM, TBN, TWM, TWN, OP_DGRAD2, OP_WGRAD2, F16>(D, r, t, st, "bwd_fc2", "wgrad2_finish");
    // 1st linear layer: dxp = dpre W1^T  and  dW1[e] = x[perm/k]^T dpre
    r = g; t = g;
    r.A = (const bf16_t*)ws.dpre; r.B = W1; r.out0 = ws.dxp; r.K = D.f; r.N = D.d;
    t.A = x; t.a_rows = D.T; t.rowoff = ws.rowoff;
    t.B = (const bf16_t*)ws.dpre; t.out0 = dW1; t.M = D.d; t.N = D.f;
    launch_pair<TBM, TBN, TWM, TWN, OP_DGRAD1, OP_WGRAD1, F16>(D, r, t, st, "bwd_fc1", "wgrad1_finish");
    return hipGetLastError();
}

// The 16-bit paths: all pointers are raw 16-bit storage, bf16 or (f16 = true) IEEE fp16.
hipError_t launch_bf16_fwd(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* b1,
                           const bf16_t* W2, const bf16_t* b2, const hexa_moe_idx& idx,
                           const MoeWorkspace& ws, hipStream_t st, bool f16) {
    return f16 ? fwd_impl<true>(D, x, W1, b1, W2, b2, idx, ws, st)
               : fwd_impl<false>(D, x, W1, b1, W2, b2, idx, ws, st);
}

hipError_t launch_bf16_bwd(const MoeDims& D, const bf16_t* x, const bf16_t* W1, const bf16_t* W2,
                           const hexa_moe_idx& idx, const MoeWorkspace& ws, float* dW1, float* dW2,
                           hipStream_t st, bool f16) {
    return f16 ? bwd_impl<true>(D, x, W1, W2, idx, ws, dW1, dW2, st)
               : bwd_impl<false>(D, x, W1, W2, idx, ws, dW1, dW2, st);
}

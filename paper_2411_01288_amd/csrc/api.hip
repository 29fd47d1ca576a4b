// C ABI of libhexa_moe: argument checks, workspace layout, and the launch sequence of the
// layer (HEXA-MoE App. B Table 5).  See include/hexa_moe.h for the contract.
#include "common.h"

#include <atomic>
#include <mutex>
#include <vector>

namespace {

constexpr int kMaxExperts = 1024;

}  // namespace

hexa_status hexa_check_shape(const hexa_moe_shape* s, MoeDims* D) {
    if (!s) return HEXA_ERR_NULL;
    if (s->T <= 0 || s->d_model <= 0 || s->d_ff <= 0 || s->E <= 0 || s->k <= 0) return HEXA_ERR_SHAPE;
    if (s->E > kMaxExperts) return HEXA_ERR_SHAPE;
    if ((long long)s->T * s->k > 0x7fffffffLL) return HEXA_ERR_SHAPE;
    if (s->dtype != HEXA_F32 && s->dtype != HEXA_BF16 && s->dtype != HEXA_F16) return HEXA_ERR_UNSUPPORTED;
    if (s->activation < HEXA_ACT_GELU_TANH || s->activation > HEXA_ACT_SILU) return HEXA_ERR_UNSUPPORTED;
    if (s->dtype != HEXA_F32) {
        if (s->d_model % 64 != 0 || s->d_ff % 64 != 0) return HEXA_ERR_UNSUPPORTED;
        // the 16-bit kernels address x (gathered rows), one expert's weight matrix and the rows of
        // one 256-row tile of any activation matrix with 32-bit byte offsets; the output window of a
        // tile (256 rows of fp32 at most) must stay below 2^31 bytes, the offset that masks a lane
        const unsigned long long wide = (unsigned long long)(s->d_model > s->d_ff ? s->d_model : s->d_ff);
        if (((unsigned long long)s->T + 1ull) * s->d_model * 2ull > 0xffffffffull ||   // x and one more row: the offset that masks a gathered row points there
            (unsigned long long)s->d_model * s->d_ff * 2ull > 0xffffffffull ||
            256ull * wide * 4ull > 0x7fffffffull)
            return HEXA_ERR_UNSUPPORTED;
    }
    D->T = s->T; D->d = s->d_model; D->f = s->d_ff; D->E = s->E; D->k = s->k; D->A = s->T * s->k;
    D->act = s->activation;
    return HEXA_OK;
}

namespace {

hexa_status check_shape(const hexa_moe_shape* s, MoeDims* D) { return hexa_check_shape(s, D); }

// Carve the workspace.  base may be NULL (size query).
MoeWorkspace layout(const MoeDims& D, int dtype, void* base) {
    MoeWorkspace w{};
    const size_t es = dtype == HEXA_F32 ? 4 : 2;
    const size_t A = (size_t)D.A, d = (size_t)D.d, f = (size_t)D.f;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void* p = base ? (void*)((uint8_t*)base + off) : nullptr;
        off += align_up(bytes, 256);
        return p;
    };
    w.pre = take(A * f * es);
    w.h = take(A * f * es);
    w.o = take(A * d * es);
    w.dout = take(A * d * es);
    w.dpre = take(A * f * es);
    w.dxp = take(A * d * es);
    {   // column-sum staging: the prologue's tiles, or (bf16) two partial rows per 256-row GEMM tile
        size_t rows = colsum_partial_rows(D);
        const size_t rows_gemm = A / 128 + 2 * (size_t)D.E;
        if (rows < rows_gemm) rows = rows_gemm;
        w.colpart = (float*)take(rows * (d > f ? d : f) * 4);
    }
    if (dtype != HEXA_F32) {
        w.rowoff = (uint32_t*)take((A + 64 * (size_t)D.E) * 4);
        w.kpart_slots = wgrad_max_slots(D);
        w.kpart = (float*)take(w.kpart_slots * d * f * 4);
        w.worklist = (int32_t*)take(gemm_worklist_ints(D) * 4);
    }
    w.total_bytes = off;
    return w;
}

bool any_null(std::initializer_list<const void*> ps) {
    for (const void* p : ps)
        if (!p) return true;
    return false;
}

hexa_status dev(hipError_t e) { return e == hipSuccess ? HEXA_OK : HEXA_ERR_DEVICE; }

// The kernels access tensors with 16-byte vectors and carve the workspace in 256-byte steps.
bool misaligned(std::initializer_list<const void*> ps, uintptr_t a) {
    for (const void* p : ps)
        if (p && ((uintptr_t)p & (a - 1)) != 0) return true;
    return false;
}

// One-time set-up per device (kernel launch attributes), with that device current.  The size
// query runs it too, so a caller that sized its workspace on the device has done it before any
// stream capture begins.
std::atomic<bool> g_dev_ready[kMaxDevices];
std::mutex g_dev_mu;
hipError_t ensure_device_init() {
    int d = -1;
    hipError_t e = hipGetDevice(&d);
    if (e != hipSuccess) return e;
    if (d < 0 || d >= kMaxDevices) return hipErrorInvalidDevice;
    if (g_dev_ready[d].load(std::memory_order_acquire)) return hipSuccess;
    std::lock_guard<std::mutex> lk(g_dev_mu);
    if (g_dev_ready[d].load(std::memory_order_relaxed)) return hipSuccess;
    e = gemm_bf16_device_init();
    if (e == hipSuccess) g_dev_ready[d].store(true, std::memory_order_release);
    return e;
}

}  // namespace

extern "C" {

size_t hexa_moe_padded_capacity(const hexa_moe_shape* shape, int32_t blk) {
    MoeDims D;
    if (blk <= 0 || check_shape(shape, &D) != HEXA_OK) return 0;
    return (size_t)D.A + (size_t)D.E * (size_t)(blk - 1);
}

hexa_status hexa_moe_padded_index(const hexa_moe_shape* shape, hexa_moe_idx idx, int32_t blk, int32_t* v,
                                  size_t v_entries, int32_t* idx_pad, void* stream) {
    MoeDims D;
    const hexa_status s = check_shape(shape, &D);
    if (s != HEXA_OK) return s;
    if (blk <= 0 || (size_t)D.A + (size_t)D.E * (size_t)(blk - 1) > 0x7fffffffull) return HEXA_ERR_SHAPE;
    if (any_null({idx.offsets, idx.perm, v, idx_pad})) return HEXA_ERR_NULL;
    if (v_entries < hexa_moe_padded_capacity(shape, blk)) return HEXA_ERR_WORKSPACE;
    return dev(launch_padded_index(D, idx, blk, (long long)v_entries, v, idx_pad, (hipStream_t)stream));
}

hexa_status hexa_moe_allocate(int32_t n, const double* latency, int64_t total, int64_t granule,
                              int64_t* share) {
    if (!latency || !share) return HEXA_ERR_NULL;
    if (n <= 0 || granule <= 0 || total < 0 || total % granule != 0) return HEXA_ERR_SHAPE;
    double wsum = 0.0;
    for (int i = 0; i < n; ++i) {
        if (!(latency[i] > 0.0) || latency[i] > 1e300) return HEXA_ERR_SHAPE;
        wsum += 1.0 / latency[i];
    }
    const int64_t units = total / granule;
    std::vector<double> frac((size_t)n);
    int64_t given = 0;
    for (int i = 0; i < n; ++i) {
        const double ideal = (1.0 / latency[i]) / wsum * (double)units;
        int64_t fl = (int64_t)ideal;            // ideal >= 0
        if (fl > units) fl = units;
        frac[(size_t)i] = ideal - (double)fl;
        share[i] = fl;
        given += fl;
    }
    // hand the remaining granules to the largest fractional parts; on rounding noise that leaves
    // more than n granules over (it cannot in exact arithmetic), keep cycling
    for (int64_t left = units - given; left > 0; --left) {
        int best = 0;
        for (int i = 1; i < n; ++i)
            if (frac[(size_t)i] > frac[(size_t)best]) best = i;
        share[best] += 1;
        frac[(size_t)best] -= 1.0;
    }
    for (int i = 0; i < n; ++i) share[i] *= granule;
    return HEXA_OK;
}

size_t hexa_moe_index_scratch_bytes(const hexa_moe_shape* shape) {
    MoeDims D;
    if (check_shape(shape, &D) != HEXA_OK) return 0;
    return index_scratch_bytes(D);
}

size_t hexa_moe_workspace_bytes(const hexa_moe_shape* shape) {
    MoeDims D;
    if (check_shape(shape, &D) != HEXA_OK) return 0;
    if (shape->dtype != HEXA_F32) (void)ensure_device_init();   // no device here: the entry points will report it
    return layout(D, shape->dtype, nullptr).total_bytes;
}

const char* hexa_moe_status_string(int s) {
    switch (s) {
        case HEXA_OK: return "ok";
        case HEXA_ERR_NULL: return "a required pointer is NULL";
        case HEXA_ERR_SHAPE: return "invalid shape";
        case HEXA_ERR_UNSUPPORTED: return "unsupported dtype, feature size or pointer alignment";
        case HEXA_ERR_WORKSPACE: return "scratch or workspace too small or misaligned";
        case HEXA_ERR_DEVICE: return "kernel launch failed";
    }
    return "unknown status";
}

hexa_status hexa_moe_index(const hexa_moe_shape* shape, const int32_t* topk_idx, hexa_moe_idx out,
                           void* scratch, size_t scratch_bytes, void* stream) {
    MoeDims D;
    const hexa_status s = check_shape(shape, &D);
    if (s != HEXA_OK) return s;
    if (any_null({topk_idx, out.counts, out.offsets, out.perm, out.inv, scratch})) return HEXA_ERR_NULL;
    if (scratch_bytes < index_scratch_bytes(D)) return HEXA_ERR_WORKSPACE;
    return dev(launch_index(D, topk_idx, out, scratch, (hipStream_t)stream));
}

hexa_status hexa_moe_fwd(const hexa_moe_shape* shape, const void* x, const int32_t* topk_idx,
                         const float* gate, const void* W1, const void* b1, const void* W2,
                         const void* b2, hexa_moe_idx idx, void* y, void* workspace,
                         size_t workspace_bytes, void* stream) {
    MoeDims D;
    const hexa_status s = check_shape(shape, &D);
    if (s != HEXA_OK) return s;
    if (any_null({x, topk_idx, gate, W1, b1, W2, b2, idx.counts, idx.offsets, idx.perm, idx.inv, y,
                  workspace}))
        return HEXA_ERR_NULL;
    const MoeWorkspace ws = layout(D, shape->dtype, workspace);
    if (workspace_bytes < ws.total_bytes || misaligned({workspace}, 256)) return HEXA_ERR_WORKSPACE;
    if (misaligned({x, W1, b1, W2, b2, y}, 16)) return HEXA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (shape->dtype != HEXA_F32 && (e = ensure_device_init()) != hipSuccess) return dev(e);
    if (shape->dtype == HEXA_F32) {
        e = launch_f32_fwd(D, (const float*)x, (const float*)W1, (const float*)b1, (const float*)W2,
                           (const float*)b2, idx, ws, st);
        if (e == hipSuccess) e = launch_combine_y<float>(D, (const float*)ws.o, idx.inv, gate, (float*)y, st);
    } else {
        const bool f16 = shape->dtype == HEXA_F16;
        e = launch_bf16_fwd(D, (const bf16_t*)x, (const bf16_t*)W1, (const bf16_t*)b1,
                            (const bf16_t*)W2, (const bf16_t*)b2, idx, ws, st, f16);
        if (e == hipSuccess) {
            if (f16) e = launch_combine_y<f16_t>(D, (const f16_t*)ws.o, idx.inv, gate, (f16_t*)y, st);
            else e = launch_combine_y<bf16_t>(D, (const bf16_t*)ws.o, idx.inv, gate, (bf16_t*)y, st);
        }
    }
    return dev(e);
}

hexa_status hexa_moe_bwd(const hexa_moe_shape* shape, const void* dY, const void* x,
                         const int32_t* topk_idx, const float* gate, const void* W1, const void* W2,
                         hexa_moe_idx idx, void* workspace, size_t workspace_bytes, void* dx,
                         float* dW1, float* db1, float* dW2, float* db2, float* dgate, void* stream) {
    MoeDims D;
    const hexa_status s = check_shape(shape, &D);
    if (s != HEXA_OK) return s;
    if (any_null({dY, x, topk_idx, gate, W1, W2, idx.counts, idx.offsets, idx.perm, idx.inv, workspace,
                  dx, dW1, db1, dW2, db2}))
        return HEXA_ERR_NULL;
    const MoeWorkspace ws = layout(D, shape->dtype, workspace);
    if (workspace_bytes < ws.total_bytes || misaligned({workspace}, 256)) return HEXA_ERR_WORKSPACE;
    if (misaligned({dY, x, W1, W2, dx, dW1, db1, dW2, db2}, 16)) return HEXA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (shape->dtype != HEXA_F32 && (e = ensure_device_init()) != hipSuccess) return dev(e);
    if (shape->dtype == HEXA_F32) {
        e = launch_bwd_prologue<float>(D, (const float*)dY, (const float*)ws.o, idx.perm,
                                       idx.offsets, gate, (float*)ws.dout, dgate, ws.colpart, db2, st);
        if (e == hipSuccess)
            e = launch_f32_bwd(D, (const float*)x, (const float*)W1, (const float*)W2, idx, ws, dW1, dW2, st);
        if (e == hipSuccess)
            e = launch_segment_colsum<float>(D, (const float*)ws.dpre, D.f, idx.offsets, ws.colpart, db1, st);
        if (e == hipSuccess) e = launch_combine_dx<float>(D, (const float*)ws.dxp, idx.inv, (float*)dx, st);
    } else {
        const bool f16 = shape->dtype == HEXA_F16;
        if (f16)
            e = launch_bwd_prologue<f16_t>(D, (const f16_t*)dY, (const f16_t*)ws.o,
                                           idx.perm, idx.offsets, gate, (f16_t*)ws.dout, dgate, ws.colpart, db2, st);
        else
            e = launch_bwd_prologue<bf16_t>(D, (const bf16_t*)dY, (const bf16_t*)ws.o,
                                            idx.perm, idx.offsets, gate, (bf16_t*)ws.dout, dgate, ws.colpart, db2, st);
        if (e == hipSuccess)
            e = launch_bf16_bwd(D, (const bf16_t*)x, (const bf16_t*)W1, (const bf16_t*)W2, idx, ws,
                                dW1, dW2, st, f16);
        if (e == hipSuccess)
            e = launch_tile_colsum_finish(D, ws.colpart, D.f, idx.offsets, db1, st);
        if (e == hipSuccess) {
            if (f16) e = launch_combine_dx<f16_t>(D, (const f16_t*)ws.dxp, idx.inv, (f16_t*)dx, st);
            else e = launch_combine_dx<bf16_t>(D, (const bf16_t*)ws.dxp, idx.inv, (bf16_t*)dx, st);
        }
    }
    return dev(e);
}

}  // extern "C"

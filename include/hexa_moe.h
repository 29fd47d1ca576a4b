/* hexa_moe.h -- C ABI of the MI355X (gfx950) expert-specific MoE FFN layer.
 *
 * One top-k Mixture-of-Experts FFN layer, forward and backward, computed with
 * routing-indexed ("expert-specific") operators: no capacity padding, no token
 * dropping, all experts resident on one GPU.  (HEXA-MoE, arXiv 2411.01288:
 * operators ESMM / ESS / ESTMM of Sec. 3.1; layer dataflow of App. B Table 5;
 * re-index vector of Sec. 3.2 and App. B Alg. 1.)
 *
 * Notation: T tokens (the paper's N), d = d_model, f = d_ff, E experts, k = top-k,
 * A = T*k assignments; flat assignment id a = t*k + j belongs to token t = a / k,
 * expert e_a = topk_idx[a], gate g_a = gate[a].
 *
 * General rules
 *   - Every pointer marked "dev" is device memory of the current HIP device;
 *     the caller owns all of it.  No entry point allocates, frees or
 *     synchronises; all work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns at once.
 *   - All tensors are dense, row-major, without strides.
 *   - Element type `shape.dtype` (HEXA_F32, HEXA_BF16 or HEXA_F16) applies to x, W1, b1,
 *     W2, b2, y, dY, dx.  gate and dgate are float.  Weight and bias gradients
 *     are float (the accumulation type).  Index tensors are int32.
 *   - Outputs are overwritten, never accumulated into.
 *   - Errors are return codes.  Argument checks run on the host before any
 *     launch: HEXA_ERR_NULL, _SHAPE, _UNSUPPORTED and _WORKSPACE mean that nothing
 *     was enqueued.  HEXA_ERR_DEVICE reports a failed launch or set-up call
 *     (hipGetLastError); launches of the same call that preceded it may already
 *     be queued, and the outputs are then undefined.
 *   - Alignment: every tensor pointer must be 16-byte aligned (the kernels use
 *     16-byte vector accesses), else HEXA_ERR_UNSUPPORTED; the workspace base
 *     must be 256-byte aligned, else HEXA_ERR_WORKSPACE.
 *   - HEXA_BF16 and HEXA_F16 (the MFMA paths) need d % 64 == 0 and f % 64 == 0
 *     (the K loop of the contraction kernels runs in blocks of 64, one 128-byte
 *     line per operand row; the paper's kernels likewise assume feature sizes
 *     divisible by the tile, App. B), (T+1)*d*2 < 2^32, d*f*2 < 2^32 and
 *     256*max(d,f)*4 < 2^31 (32-bit byte offsets inside x, inside one expert's
 *     weight matrix and inside one 256-row tile of an activation or gradient
 *     matrix);
 *     HEXA_F32 takes any positive sizes.  E <= 1024.
 *   - The first hexa_moe_workspace_bytes, hexa_moe_fwd or hexa_moe_bwd call for a
 *     16-bit shape on a device raises the shared-memory limit of the contraction
 *     kernels there (once per device, thread-safe).  That set-up call must not
 *     fall inside a stream capture; sizing the workspace on the device before
 *     capturing takes care of it.
 *   - Expert ids must satisfy 0 <= topk_idx < E (App. B Table 4).  An id outside
 *     that range is not an error return (the host cannot see it): that
 *     assignment is dropped from the index (inv = -1, offsets[E] < A), it
 *     contributes nothing to y, and its dx/dgate contributions are zero.  A
 *     caller that wants the check compares offsets[E] with A.
 */
#ifndef HEXA_MOE_H
#define HEXA_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HEXA_API __attribute__((visibility("default")))

typedef enum {
    HEXA_OK = 0,
    HEXA_ERR_NULL = 1,        /* a required pointer is NULL */
    HEXA_ERR_SHAPE = 2,       /* a size is <= 0, A overflows int32, or E > 1024 */
    HEXA_ERR_UNSUPPORTED = 3, /* dtype or activation unknown, a 16-bit size rule (see above) is not met,
                                 or a tensor pointer is not 16-byte aligned */
    HEXA_ERR_WORKSPACE = 4,   /* scratch / workspace smaller than the *_bytes() query, its base misaligned,
                                 or (hexa_moe_index_static) the shape needs more than the built-in scratch */
    HEXA_ERR_DEVICE = 5       /* a launch or a set-up call failed (hipGetLastError) */
} hexa_status;

typedef enum { HEXA_F32 = 0, HEXA_BF16 = 1, HEXA_F16 = 2 } hexa_dtype;

/* The activation F between the two linear layers (App. B Table 5 rows 2 and 7).  The paper does not
 * name it; 0, GELU in its tanh form (constants sqrt(2/pi), 0.044715), is the reading used for every
 * benchmark workload.  ReLU takes derivative 0 at 0. */
typedef enum { HEXA_ACT_GELU_TANH = 0, HEXA_ACT_RELU = 1, HEXA_ACT_SILU = 2 } hexa_activation;

typedef struct {
    int32_t T, d_model, d_ff, E, k;
    int32_t dtype;      /* hexa_dtype */
    int32_t activation; /* hexa_activation */
} hexa_moe_shape;

/* The re-index structures (Sec. 3.2; App. B Alg. 1 and Table 4), all dev:
 *   counts [E]    n_e = number of assignments routed to expert e
 *   offsets[E+1]  exclusive prefix sum of counts; offsets[0] = 0, offsets[E] = A
 *   perm   [A]    the re-index vector v without padding: flat assignment ids
 *                 grouped by expert; inside a group in ascending id (the paper
 *                 leaves that order to atomics; this library fixes it so the
 *                 result is unique)
 *   inv    [A]    inverse of perm: inv[perm[p]] = p
 */
typedef struct {
    int32_t *counts, *offsets, *perm, *inv;
} hexa_moe_idx;

/* Bytes of device scratch hexa_moe_index needs (0 on an invalid shape). */
HEXA_API size_t hexa_moe_index_scratch_bytes(const hexa_moe_shape *shape);

/* Bytes of device workspace shared by hexa_moe_fwd and hexa_moe_bwd (0 on an
 * invalid shape).  It holds what the forward pass saves for the backward pass
 * (pre-activations or the activation's derivative at them, activations,
 * per-assignment expert outputs, in perm order, and the tile lists derived from
 * the index) plus backward staging.  256-byte alignment of the base is required. */
HEXA_API size_t hexa_moe_workspace_bytes(const hexa_moe_shape *shape);

/* Text for a status code; any other integer gives "unknown status" (hence int, not the enum). */
HEXA_API const char *hexa_moe_status_string(int status);

/* Re-index build (App. B Alg. 1; Sec. 3.2 "Re-Index based Expert-Specific
 * Operators"), for all k routing slots at once.
 *   topk_idx [T,k] dev, in       routing choice R_j(x_t)
 *   out      dev, out            counts, offsets, perm, inv as described above
 *   scratch  dev, >= hexa_moe_index_scratch_bytes(); contents undefined after
 * Integer work; the result is bit-exact and independent of scheduling. */
HEXA_API hexa_status hexa_moe_index(const hexa_moe_shape *shape, const int32_t *topk_idx,
                           hexa_moe_idx out, void *scratch, size_t scratch_bytes,
                           void *stream);

/* hexa_moe_index for callers that cannot allocate device memory (code under HIP stream capture,
 * tight serving loops, harnesses that forbid hipMalloc): same inputs, same outputs, same kernels,
 * but the chunk-histogram scratch is a fixed array of HEXA_INDEX_STATIC_SCRATCH_BYTES that the
 * library holds in each GPU's memory from load until the process ends.  The call allocates and
 * frees nothing and takes no scratch argument.
 *   - Limit: hexa_moe_index_scratch_bytes(shape) <= HEXA_INDEX_STATIC_SCRATCH_BYTES, else
 *     HEXA_ERR_WORKSPACE with nothing enqueued.  1 MiB covers min(ceil(T*k/64), 1024) * E <= 262 144:
 *     any T*k when E <= 256, any E <= 1024 when T*k <= 16 384.
 *   - The first call on a device looks the array's address up there (one host call, no stream
 *     work; make it outside a capture) and returns HEXA_ERR_DEVICE if that fails.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap on one GPU
 *     (different streams, or different host threads on different streams) race.  Calls on one
 *     stream are ordered and safe; nothing needs clearing between calls. */
#define HEXA_INDEX_STATIC_SCRATCH_BYTES (1u << 20)
HEXA_API hexa_status hexa_moe_index_static(const hexa_moe_shape *shape, const int32_t *topk_idx,
                                  hexa_moe_idx out, void *stream);

/* The paper's own form of the index (App. B Alg. 1; Sec. 3.2), derived from hexa_moe_index's output
 * for callers written against it: every expert's sub-vector padded with -1 up to a multiple of the
 * tile size blk.
 *   idx      as written by hexa_moe_index (offsets and perm are read)               dev, in
 *   v        [v_entries] int32, v_entries >= hexa_moe_padded_capacity() = A + E*(blk-1)   dev, out
 *            expert e's flat assignment ids (ascending; token ids when k = 1) at
 *            v[idx_pad[e] ...], then -1 up to idx_pad[e+1]; -1 from idx_pad[E] (the paper's N') on
 *   idx_pad  [E+1] int32: starts of the padded sub-vectors (the paper's idx_)     dev, out
 * Bit-exact.  (The printed listing rounds the counts down; Sec. 3.2 pads them up, which is what fits
 * every token, and what is done here.) */
HEXA_API size_t hexa_moe_padded_capacity(const hexa_moe_shape *shape, int32_t blk);
HEXA_API hexa_status hexa_moe_padded_index(const hexa_moe_shape *shape, hexa_moe_idx idx, int32_t blk,
                                  int32_t *v, size_t v_entries, int32_t *idx_pad, void *stream);

/* Forward (App. B Table 5 rows 1-3; ESMM of Sec. 3.1):
 *   pre_a = x_t W1[e_a] + b1[e_a];  h_a = F(pre_a);  o_a = h_a W2[e_a] + b2[e_a]
 *   y_t   = sum_j gate[t,j] * o_{t*k+j}
 * (the paper's table sums the k slots unweighted; the gate factor is this
 * library's reading, equal to the paper's for gate == 1).
 *   x [T,d], W1 [E,d,f], b1 [E,f], W2 [E,f,d], b2 [E,d]   dev, in, shape.dtype
 *   topk_idx [T,k] int32, gate [T,k] float                 dev, in
 *   idx        as written by hexa_moe_index for this topk_idx  dev, in
 *   y [T,d]    dev, out, shape.dtype
 *   workspace  dev, >= hexa_moe_workspace_bytes(); afterwards holds the saved
 *              state hexa_moe_bwd reads
 * bf16 / fp16: products in MFMA of that type with fp32 accumulation; h, F'(pre) and the
 * per-assignment outputs o are stored rounded to the element type (round-to-nearest-even), the k-slot sum runs
 * in fp32. */
HEXA_API hexa_status hexa_moe_fwd(const hexa_moe_shape *shape, const void *x, const int32_t *topk_idx,
                         const float *gate, const void *W1, const void *b1, const void *W2,
                         const void *b2, hexa_moe_idx idx, void *y, void *workspace,
                         size_t workspace_bytes, void *stream);

/* Backward (App. B Table 5 rows 4-10; ESS and ESTMM of Sec. 3.1), with
 * do_a = gate_a * dY_t:
 *   db2[e] = sum_{a in e} do_a            dW2[e] = sum_{a in e} h_a^T do_a
 *   dh_a = do_a W2[e_a]^T                 dpre_a = dh_a * F'(pre_a)
 *   db1[e] = sum_{a in e} dpre_a          dW1[e] = sum_{a in e} x_t^T dpre_a
 *   dx_t = sum_j dpre_{t*k+j} W1[e]^T     dgate[t,j] = <dY_t, o_{t*k+j}>
 *   dY [T,d]                                    dev, in, shape.dtype
 *   x, topk_idx, gate, W1, W2, idx              dev, in, as given to hexa_moe_fwd
 *   workspace  dev, as left by hexa_moe_fwd for the same inputs (its saved part is
 *              only read, so hexa_moe_bwd may be called again; staging is rewritten)
 *   dx [T,d] shape.dtype; dW1 [E,d,f], db1 [E,f], dW2 [E,f,d], db2 [E,d] float
 *                                               dev, out
 *   dgate [T,k] float                           dev, out, or NULL to skip
 * Experts with no tokens get exact zeros in dW1, db1, dW2, db2.  All sums run
 * in a fixed order: results are reproducible run to run. */
HEXA_API hexa_status hexa_moe_bwd(const hexa_moe_shape *shape, const void *dY, const void *x,
                         const int32_t *topk_idx, const float *gate, const void *W1,
                         const void *W2, hexa_moe_idx idx, void *workspace,
                         size_t workspace_bytes, void *dx, float *dW1, float *db1, float *dW2,
                         float *db2, float *dgate, void *stream);

/* Router front-end: the step before hexa_moe_index.  The paper takes the routing choice
 * {R_j(x)} as given (Sec. 3.1; App. B Table 5); this entry point produces it from router logits:
 * per token the k largest of E logits, equal logits to the lower expert id, slot j = the j-th
 * largest; gate weights per gate_mode.  Its outputs are what hexa_moe_index / fwd / bwd take.
 *   logits   [T,E] float  dev, in   (a NaN counts as -inf: it is selected only after every other
 *                                    logit of its row and then gets gate 0; a row whose largest
 *                                    logit is -inf or NaN gets NaN gates)
 *   topk_idx [T,k] int32  dev, out  bit-exact (comparisons only)
 *   gate     [T,k] float  dev, out
 * shape: T, E, k are used (d_model, d_ff, dtype ignored).  k <= min(E, 64), E <= 1024, else
 * HEXA_ERR_UNSUPPORTED / HEXA_ERR_SHAPE. */
typedef enum {
    HEXA_GATE_SOFTMAX_SELECTED = 0, /* softmax over the k selected logits (gates sum to 1) */
    HEXA_GATE_SOFTMAX_ALL = 1       /* softmax over all E logits, evaluated at the selected ones */
} hexa_gate_mode;
HEXA_API hexa_status hexa_moe_route(const hexa_moe_shape *shape, const float *logits, int32_t gate_mode,
                           int32_t *topk_idx, float *gate, void *stream);

/* Heterogeneous-aware allocation (Sec. 3.4, Eq. 1 and Eq. 2), a host-only helper: splits `total`
 * units of work (the global batch for the data-centric setting, Eq. 1; the FFN hidden size for the
 * model-centric one, Eq. 2) over n devices in proportion to 1 / latency[i], where latency[i] > 0 is
 * device i's measured time on a common benchmark task.  Shares are multiples of `granule` (>= 1; the
 * bf16 path of this library needs hidden-size shares that are multiples of 64) and sum to `total`
 * exactly: every device gets the floor of its ideal share in granules and the granules left over go to
 * the largest fractional parts (ties to the lower device index), the rounding the paper asks for
 * without fixing one.  total must be a non-negative multiple of granule.
 *   latency [n] host, in;  share [n] host, out.  Returns HEXA_ERR_NULL / HEXA_ERR_SHAPE on bad input. */
HEXA_API hexa_status hexa_moe_allocate(int32_t n, const double *latency, int64_t total, int64_t granule,
                              int64_t *share);

#ifdef __cplusplus
}
#endif
#endif /* HEXA_MOE_H */

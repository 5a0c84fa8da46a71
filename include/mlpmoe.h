/*
 * mlpmoe.h -- C ABI of the MI355X (gfx950) branched SwiGLU MLP forward.
 *
 * The operation (MLPMoE, Sec. 3.1):
 *
 *     branch_b(x) = alpha_b * W_down^(b) [ SiLU(W_gate^(b) x) (.) W_up^(b) x ]
 *     MLPMoE(x)   = sum_{b=0}^{B-1} branch_b(x)
 *
 * where the B branches are contiguous slices of the intermediate dimension,
 * d_inter = sum_b d_b.  Branches removed by Compensated Branch Pruning
 * (Sec. 3.3) are skipped, and neurons removed by per-branch differential
 * sparsity (Sec. 3.2, structured form) are compacted out of the weight
 * buffers, so the widths d_b may differ from branch to branch.
 *
 * Layouts (all row-major, no padding between rows):
 *     x       [T, d_model]
 *     W_gate  [d_inter, d_model]    row j          = neuron j
 *     W_up    [d_inter, d_model]    row j          = neuron j
 *     W_down  [d_model, d_inter]    column j       = neuron j
 *     out     [T, d_model]          float, overwritten (never accumulated into)
 * Branch b owns neurons branch_offsets[b] .. branch_offsets[b+1]-1.
 *
 * Pointer kinds: x, W_*, out, workspaces and gather lists passed to
 * mlpmoe_compact are DEVICE pointers owned by the caller; branch_offsets,
 * alpha and active_mask are HOST pointers, read during the call and free for
 * reuse when it returns.  `stream` is a hipStream_t passed as void* (NULL =
 * the default stream).  Forward calls enqueue work and return without
 * synchronising.
 *
 * Every function returns MLPMOE_OK (0) or a negative MLPMOE_ERR_* code.
 * Argument errors are detected on the host before anything is enqueued; the
 * library never throws, aborts or prints.
 */
#ifndef MLPMOE_H
#define MLPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MLPMOE_MAX_BRANCHES 64

/* Exported-symbol marker: the library is built with hidden visibility by default. */
#if defined(__GNUC__)
#define MLPMOE_API __attribute__((visibility("default")))
#else
#define MLPMOE_API
#endif

enum {
    MLPMOE_OK = 0,
    MLPMOE_ERR_NULL = -1,        /* a required pointer is NULL                              */
    MLPMOE_ERR_SHAPE = -2,       /* a size is negative, zero where it may not be, or too big */
    MLPMOE_ERR_OFFSETS = -3,     /* offsets do not start at 0, decrease, or miss d_inter    */
    MLPMOE_ERR_UNSUPPORTED = -4, /* the requested kernel path cannot run these arguments    */
    MLPMOE_ERR_WORKSPACE = -5,   /* workspace missing, too small or misaligned              */
    MLPMOE_ERR_HIP = -6,         /* a HIP runtime call failed                               */
    MLPMOE_ERR_ALIGN = -7        /* a device pointer is not 16-byte aligned                 */
};

/* Kernel path selection for the *_ws entry points. */
enum {
    MLPMOE_PATH_AUTO = 0,    /* library picks: decode for T <= 16, MFMA otherwise, generic if unaligned */
    MLPMOE_PATH_GENERIC = 1, /* LDS-tiled FMA kernels: any shape and alignment                        */
    MLPMOE_PATH_MFMA = 2,    /* bf16 MFMA prefill kernels (needs d_model%8==0 and offsets%8==0)       */
    MLPMOE_PATH_DECODE = 3,  /* weight-streaming kernels, T <= 16 (same alignment needs as MFMA)      */
    /* MLPMOE_PATH_MFMA picks a tile shape per launch from the sizes; these force one, for both kernels   */
    MLPMOE_PATH_MFMA_WIDE = 4,   /* 256 tokens x (128 + 128) neurons / 256 output features             */
    MLPMOE_PATH_MFMA_NARROW = 5, /* 256 tokens x (64 + 64) neurons / 128 output features               */
    MLPMOE_PATH_MFMA_SMALL = 6,  /* 128 tokens x (64 + 64) / 128, 4 waves, two workgroups per CU       */
    MLPMOE_PATH_MFMA_MIXED = 7,  /* gate+up: WIDE for the full rounds of 256 workgroups; a remainder of at
                                    most half a round as halves of a wide tile (NARROW's), of at most a
                                    quarter of a round as quarters (WIDE if there is none); down: chosen */
    MLPMOE_PATH_MFMA_DEEP = 8,   /* SMALL's tile with four K tiles requested ahead, one workgroup per CU */
    MLPMOE_PATH_MFMA_SLIM = 9    /* 64 tokens x (64 + 64) / 128, 4 waves, five K tiles requested ahead   */
};

/* Human-readable name of a status code (static string, never NULL). */
MLPMOE_API const char *mlpmoe_status_string(int status);

/*
 * What the HIP runtime said when a call of THIS thread last returned MLPMOE_ERR_HIP: the failing
 * runtime call or kernel launch and hipGetErrorString() of its code, e.g.
 * "decode_down launch: invalid configuration argument".  Points into thread-local storage owned
 * by the library (valid until the thread's next failing call); an empty string if none failed.
 */
MLPMOE_API const char *mlpmoe_last_error_detail(void);

/*
 * mlpmoe_slice -- host only; touches no GPU.
 * Builds the branch table of one MLP (Sec. 3.1 slicing, Sec. 3.1 scalar gates,
 * Sec. 3.3 pruning rule).
 *
 *   d_inter, B    intermediate width of the dense MLP and number of branches,
 *                 1 <= B <= MLPMOE_MAX_BRANCHES, d_inter >= 0.  Branch b gets
 *                 floor(d_inter/B) neurons, the first d_inter mod B branches one more.
 *   K_keep        0 or >= B: every branch active, alpha_b = 1.
 *                 0 < K_keep < B: keep the first K_keep branches with
 *                 alpha_b = sqrt(B / K_keep); the rest get alpha_b = 0, active_mask 0.
 *   neuron_keep   NULL, or d_inter bytes: neuron j survives iff neuron_keep[j] != 0.
 *                 Surviving neurons keep their order; d_b becomes the survivor count.
 *   pad_to        >= 1.  Each branch width is rounded up to a multiple of pad_to with
 *                 padding rows (gather index -1, to be filled with zeros: a zero gate/up
 *                 row and a zero down column contribute exactly nothing).  The MFMA and
 *                 decode paths need pad_to to be a multiple of 8.
 *   branch_offsets [B+1] out: prefix sums of the (padded) widths; [B] is the row count
 *                 of the compacted layer.
 *   alpha [B] out, active_mask [B] out.
 *   gather_index  NULL, or room for gather_capacity entries: source neuron of every
 *                 compacted row, or -1 for a padding row.
 *   gather_capacity  entries available in gather_index; d_inter + B*(pad_to-1) always suffices.
 * Errors: NULL (outputs), SHAPE (B, d_inter, pad_to out of range; gather_capacity too small).
 */
MLPMOE_API int mlpmoe_slice(int d_inter, int B, int K_keep, const uint8_t *neuron_keep, int pad_to,
                 int32_t *branch_offsets, float *alpha, uint8_t *active_mask,
                 int32_t *gather_index, int gather_capacity);

/*
 * mlpmoe_slice_rows -- mlpmoe_slice (Sec. 3.1 slicing, Sec. 3.3 rule, compaction of kept neurons) with
 * one more kind of padding: after every branch has been rounded up to a multiple of pad_to, the row
 * count of the whole compacted layer is rounded up to a multiple of pad_rows_to (1 .. 4096) with
 * further padding rows at the end of the LAST branch (gather index -1).  That row count is the
 * leading dimension of the compacted W_down: a multiple of 64 makes every row of a bf16 W_down
 * start on a 128-byte line, which the kernels' row-piece loads want (an 8B-shaped layer compacted
 * to 11544 rows: the decode down projection takes 28.1 us at T = 16 as it is and 24.5 us with 11584
 * rows).  gather_capacity: d_inter + B*(pad_to-1) + pad_rows_to-1 always suffices.  Everything else
 * as for mlpmoe_slice, which is this call with pad_rows_to = 1.
 */
MLPMOE_API int mlpmoe_slice_rows(int d_inter, int B, int K_keep, const uint8_t *neuron_keep, int pad_to,
                                 int pad_rows_to, int32_t *branch_offsets, float *alpha, uint8_t *active_mask,
                                 int32_t *gather_index, int gather_capacity);

/*
 * mlpmoe_compact -- applies a gather list on the device (weight preparation, not
 * part of the per-token path).  For r in [0, n_rows):
 *     W_gate_c[r, :] = gather[r] >= 0 ? W_gate[gather[r], :] : 0      (same for W_up)
 *     W_down_c[:, r] = gather[r] >= 0 ? W_down[:, gather[r]] : 0
 * elem_bytes is 2 (bf16) or 4 (float).  Source buffers have d_inter_src neurons;
 * destination buffers have n_rows neurons and must not overlap the sources.
 * gather is a DEVICE pointer to n_rows int32 values, each -1 or in [0, d_inter_src)
 * (the caller guarantees the range; it is not re-checked on the device).
 */
MLPMOE_API int mlpmoe_compact(const void *W_gate, const void *W_up, const void *W_down, const int32_t *gather,
                   int n_rows, int d_model, int d_inter_src, int elem_bytes, void *W_gate_c,
                   void *W_up_c, void *W_down_c, void *stream);

/*
 * Bytes of device workspace a forward call with these sizes may use (gated
 * intermediate H[T, d_inter], split-K partial sums, and the tile tables of the
 * routed forward).  Independent of the branch table.  Returns 0 for invalid sizes.
 */
MLPMOE_API size_t mlpmoe_workspace_bytes(int T, int d_model, int d_inter, int B, int elem_bytes);

/*
 * mlpmoe_forward_bf16 -- MLPMoE(x) of Sec. 3.1 for bf16 x and weights, float out.
 *
 *   x, W_gate, W_up, W_down   device, bf16, layouts above, 16-byte aligned bases.
 *   branch_offsets [B+1], alpha [B], active_mask [B]   host.  active_mask[b] == 0:
 *       branch b contributes nothing and none of its weights are read (non-finite
 *       values inside it cannot reach out).  alpha_b == 0 with the mask set is
 *       computed like any other value.
 *   T >= 0 tokens (T == 0 is a no-op), d_model >= 1, d_inter = branch_offsets[B] >= 0,
 *   1 <= B <= MLPMOE_MAX_BRANCHES.  d_b == 0 is legal.
 *   out    device float [T, d_model]; every element is written (zeros if nothing is active).
 *
 * Arithmetic: gate and up products accumulate in fp32; h = alpha_b * SiLU(g) * u is
 * formed in fp32 and rounded ONCE to bf16 (nearest even); the down projection
 * accumulates those bf16 values against W_down in fp32 across all branches.
 * Results are bitwise reproducible from run to run: sums are formed in a fixed order; the one place
 * that uses floating-point atomics (the decode down projection of wide layers) adds exactly two
 * partial sums into a zero, which gives the same number in either order.
 *
 * Workspace: the block given to mlpmoe_set_workspace() for the current device if there is
 * one -- the call then never allocates and returns MLPMOE_ERR_WORKSPACE if the block is too
 * small.  Otherwise a per-device buffer the library owns and grows with hipMalloc when a call
 * needs more than any earlier one (that growth synchronises the device; while `stream` is
 * recording a graph it is refused with MLPMOE_ERR_WORKSPACE instead).  Either way all calls
 * of this kind on one device share one block: calls that overlap in time on one device
 * (different streams) must use the *_ws form with distinct workspaces.
 *
 * Errors: NULL, SHAPE, OFFSETS, ALIGN, WORKSPACE (too small / allocation failed), HIP.
 */
MLPMOE_API int mlpmoe_forward_bf16(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                        const int32_t *branch_offsets, const float *alpha,
                        const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                        float *out, void *stream);

/* Same operation and signature; the storage type defaults to bf16. */
MLPMOE_API int mlpmoe_forward(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                   const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                   int T, int d_model, int d_inter, int B, float *out, void *stream);

/*
 * mlpmoe_forward_f32 -- same operation for float x and weights; no intermediate
 * rounding, fp32 accumulation throughout (LDS-tiled FMA kernels, any shape).
 */
MLPMOE_API int mlpmoe_forward_f32(const float *x, const float *W_gate, const float *W_up, const float *W_down,
                       const int32_t *branch_offsets, const float *alpha,
                       const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                       float *out, void *stream);

/*
 * mlpmoe_forward_bf16_out_bf16 -- the bf16 forward with the result stored as bf16: out is
 * [T, d_model] bf16 (device, 16-byte aligned), each element the fp32 sum over branches rounded once
 * to nearest even.  Everything else (arguments, arithmetic up to that rounding, errors) is
 * mlpmoe_forward_bf16's, and so are the kernels, except that for T <= 16 the float result adds
 * the two halves of K separately, which can move a sum by a float rounding.  The rounding alone moves an element by up to 2^-9 of its magnitude, about
 * 1e-2 of rms(out) for the largest elements: for callers whose next operation takes bf16 anyway
 * (Sec. 3.1 defines the sum; its storage precision is the caller's choice).  The _ws form takes a
 * caller-owned workspace and a path like mlpmoe_forward_bf16_ws and never allocates.
 */
MLPMOE_API int mlpmoe_forward_bf16_out_bf16(const void *x, const void *W_gate, const void *W_up,
                                 const void *W_down, const int32_t *branch_offsets, const float *alpha,
                                 const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                                 void *out, void *stream);
MLPMOE_API int mlpmoe_forward_bf16_out_bf16_ws(const void *x, const void *W_gate, const void *W_up,
                                    const void *W_down, const int32_t *branch_offsets, const float *alpha,
                                    const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                                    void *out, void *workspace, size_t workspace_bytes, int path,
                                    void *stream);

/*
 * mlpmoe_forward_bf16_noalloc -- mlpmoe_forward_bf16 for callers that cannot allocate device memory
 * and have no workspace to hand over: code recorded into a HIP graph, tight serving loops, harnesses
 * that forbid allocation.  Same arguments, arithmetic, kernels and results (bit for bit) as
 * mlpmoe_forward_bf16_ws with MLPMOE_PATH_AUTO; the workspace is a fixed block of
 * MLPMOE_NOALLOC_SCRATCH_BYTES that is part of the library's device image (every GPU the library runs
 * on holds its own copy from the moment the code is loaded until the process ends).  The call
 * allocates and frees nothing and synchronises nothing.  The first call on a device looks the block's
 * address up (once per device); make that call outside a graph capture.
 * Limit: mlpmoe_workspace_bytes(T, d_model, d_inter, B, 2) <= MLPMOE_NOALLOC_SCRATCH_BYTES (all decode
 * sizes T <= 16 of layers up to d_inter = 262144; prefill of small layers), otherwise
 * MLPMOE_ERR_WORKSPACE and nothing is enqueued (mlpmoe_last_error_detail() says how much was needed).
 * All calls on one GPU share that GPU's block, which keeps the last call's contents (nothing in it has
 * to start at zero: every value a kernel reads from it was written by the same call): calls that
 * overlap in time on one GPU (different streams) race on it and must not be made.
 */
#define MLPMOE_NOALLOC_SCRATCH_BYTES (16u << 20)
MLPMOE_API int mlpmoe_forward_bf16_noalloc(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                                const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                                int T, int d_model, int d_inter, int B, float *out, void *stream);

/*
 * mlpmoe_set_workspace -- gives the entry points that take no workspace argument (mlpmoe_forward,
 * mlpmoe_forward_bf16, mlpmoe_forward_f32, mlpmoe_forward_bf16_out_bf16, mlpmoe_forward_routed_*)
 * a caller-owned device block to work in on the CURRENT device, e.g. a PyTorch tensor.  From then
 * on those calls allocate nothing and synchronise nothing on that device: a call that needs more
 * than `bytes` (mlpmoe_workspace_bytes) returns MLPMOE_ERR_WORKSPACE.  dev_ptr: device, 256-byte
 * aligned, owned by the caller, who keeps it alive until it is replaced or cleared and all work
 * enqueued with it has finished; its contents are scratch.  dev_ptr == NULL clears the setting
 * (back to the library-owned buffer).  Errors: WORKSPACE (misaligned, or bytes == 0), HIP.
 */
MLPMOE_API int mlpmoe_set_workspace(void *dev_ptr, size_t bytes);

/*
 * Layout of a workspace while and after a bf16 forward runs in it: it begins with the gated
 * intermediate of Sec. 3.1's bracket, H[t][j] = bf16(alpha_b SiLU(g) u), row-major [T, ld] with
 * ld = mlpmoe_hidden_ld(d_inter) (d_inter rounded up to a multiple of 64; 0 for d_inter < 0) and
 * column j = neuron j of the weight buffers.  Columns of inactive branches are never written.
 * For tests and debugging; float storage keeps H as float with the same ld.
 */
MLPMOE_API int mlpmoe_hidden_ld(int d_inter);

/*
 * Caller-owned workspace forms.  workspace: device pointer, 256-byte aligned, at
 * least mlpmoe_workspace_bytes(T, d_model, d_inter, B, elem_bytes) bytes; its
 * contents are scratch.  path: one of MLPMOE_PATH_*; a path that cannot run the
 * given arguments returns MLPMOE_ERR_UNSUPPORTED and enqueues nothing.
 * These calls never allocate device memory.
 */
MLPMOE_API int mlpmoe_forward_bf16_ws(const void *x, const void *W_gate, const void *W_up, const void *W_down,
                           const int32_t *branch_offsets, const float *alpha,
                           const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                           float *out, void *workspace, size_t workspace_bytes, int path,
                           void *stream);

MLPMOE_API int mlpmoe_forward_f32_ws(const float *x, const float *W_gate, const float *W_up,
                          const float *W_down, const int32_t *branch_offsets, const float *alpha,
                          const uint8_t *active_mask, int T, int d_model, int d_inter, int B,
                          float *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * mlpmoe_forward_routed_bf16 / _ws -- the forward with a per-token set of branches.
 *
 * The paper names dynamic routing over the branches as the natural next step (Sec. 7, Sec. 8) and does
 * not define it; the reading implemented here: route is a device array [T, B] of bytes, and token t
 * sums the branches b with active_mask[b] != 0 AND route[t * B + b] != 0,
 *     out[t] = sum over those b of alpha[b] * W_down^(b) [ SiLU(W_gate^(b) x_t) (.) W_up^(b) x_t ].
 * All other arguments, layouts and rounding are those of mlpmoe_forward_bf16 (bf16 storage only).
 * When every branch offset is a multiple of 8 (mlpmoe_slice with pad_to = 8) the kernels skip work
 * per (tile of 256 tokens, branch) pair that no token of the tile is routed to -- for T <= 16 per
 * branch no token takes, whose weights are then never read -- so tokens grouped by route make the
 * call proportionally cheaper; other tables take the generic kernels, which only mask.
 * The _ws form takes a caller-owned workspace of mlpmoe_workspace_bytes() bytes and never allocates.
 */
MLPMOE_API int mlpmoe_forward_routed_bf16(const void *x, const void *W_gate, const void *W_up,
                                          const void *W_down, const int32_t *branch_offsets,
                                          const float *alpha, const uint8_t *active_mask, const uint8_t *route,
                                          int T, int d_model, int d_inter, int B, float *out, void *stream);
MLPMOE_API int mlpmoe_forward_routed_bf16_ws(const void *x, const void *W_gate, const void *W_up,
                                             const void *W_down, const int32_t *branch_offsets,
                                             const float *alpha, const uint8_t *active_mask,
                                             const uint8_t *route, int T, int d_model, int d_inter, int B,
                                             float *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The routed forward for float x and weights: same reading of the routing, no intermediate rounding,
 * fp32 accumulation throughout (the LDS-tiled FMA kernels; they mask and do not skip).  The _ws form
 * takes mlpmoe_workspace_bytes(T, d_model, d_inter, B, 4) bytes.
 */
MLPMOE_API int mlpmoe_forward_routed_f32(const float *x, const float *W_gate, const float *W_up,
                                         const float *W_down, const int32_t *branch_offsets, const float *alpha,
                                         const uint8_t *active_mask, const uint8_t *route, int T, int d_model,
                                         int d_inter, int B, float *out, void *stream);
MLPMOE_API int mlpmoe_forward_routed_f32_ws(const float *x, const float *W_gate, const float *W_up,
                                            const float *W_down, const int32_t *branch_offsets,
                                            const float *alpha, const uint8_t *active_mask, const uint8_t *route,
                                            int T, int d_model, int d_inter, int B, float *out, void *workspace,
                                            size_t workspace_bytes, void *stream);

/*
 * mlpmoe_fade -- Fractal Fade weight preparation (Sec. 3.2), in place, on the device.
 *
 * For every branch b with sparsity[b] > 0, and separately for the branch's rows of W_gate and of
 * W_up (row-major [d_inter, d_model]; W_down is not touched): take the linear-interpolation
 * quantile of the absolute values of that block at fraction sparsity[b] (position
 * p = s (n - 1) in the ascending order statistics, n = d_b * d_model) and set every entry whose
 * absolute value is not strictly greater than it to zero (the entry times 0: it keeps its sign).
 * Branches with sparsity[b] <= 0, and empty branches, are left exactly as they are.
 *
 *   W_gate, W_up    device, bf16 (elem_bytes 2, d_model a multiple of 8) or float (elem_bytes 4,
 *                   d_model a multiple of 4), MLPMOE_ERR_UNSUPPORTED otherwise; 16-byte aligned.
 *                   Float entries are compared as doubles with the threshold interpolated in
 *                   double from the two neighbouring order statistics
 *   branch_offsets  host, B + 1 entries as for mlpmoe_forward
 *   sparsity        host, B doubles in [0, 1] (MLPMOE_ERR_SHAPE outside), or NULL for the
 *                   schedule of Sec. 3.2: s_b = 0.9 * b / B, branch 0 dense
 *   thresholds      host, 2 * B floats or NULL: [2b] gate, [2b+1] up; the interpolated quantile
 *                   rounded to float (NaN for branches left alone)
 *   kept            host, 2 * B 64-bit counts or NULL: entries of the block that survive
 *                   (the block size for branches left alone)
 * Allocates and frees a device scratch buffer of B * 131088 bytes (bf16) or B * 655424 bytes (float)
 * and synchronises `stream` before it returns, for float storage also once in between (this is
 * offline weight preparation, not part of the forward).
 * Not-a-number entries are not supported (their place in the order is undefined).
 */
MLPMOE_API int mlpmoe_fade(void *W_gate, void *W_up, const int32_t *branch_offsets, const double *sparsity,
                           int d_model, int d_inter, int B, int elem_bytes, float *thresholds,
                           long long *kept, void *stream);

/*
 * mlpmoe_fade_neurons -- the structured form of the fade: which whole neurons each branch keeps.
 *
 * Sec. 3.2 zeroes single weights; the layers whose branches have different widths keep and drop
 * whole neurons instead, and the paper gives no rule for choosing them.  The reading implemented
 * here: the score of neuron j is the squared Euclidean norm of its W_gate row and its W_up row
 * together (accumulated in double), and branch b keeps the keep_count[b] neurons with the largest
 * scores, equal scores in order of index.  The result feeds mlpmoe_slice (neuron_keep) and
 * mlpmoe_compact; the weights are not changed.
 *
 *   W_gate, W_up    device, row-major [d_inter, d_model], bf16 (elem_bytes 2, d_model a multiple of 8)
 *                   or float (elem_bytes 4, d_model a multiple of 4): MLPMOE_ERR_UNSUPPORTED
 *                   otherwise; 16-byte aligned
 *   branch_offsets  host, B + 1 entries as for mlpmoe_forward
 *   keep_count      host, B entries, 0 <= keep_count[b] <= d_b (MLPMOE_ERR_SHAPE outside)
 *   neuron_keep     host, d_inter bytes: 1 = kept, 0 = dropped
 *   scores          host, d_inter doubles, or NULL
 * Allocates and frees 9 * d_inter bytes of device scratch and synchronises `stream` before it
 * returns (offline weight preparation).  Not-a-number weights are not supported.
 */
MLPMOE_API int mlpmoe_fade_neurons(const void *W_gate, const void *W_up, const int32_t *branch_offsets,
                        const int32_t *keep_count, int d_model, int d_inter, int B, int elem_bytes,
                        uint8_t *neuron_keep, double *scores, void *stream);

/*
 * Per-kernel timing (measurement aid; the arithmetic is unchanged and nothing is skipped).
 * While enabled, every kernel a forward call launches is bracketed by a pair of HIP events
 * recorded on the call's own stream.
 *   mlpmoe_profile_enable(capacity)  creates 2*capacity events on the current device and
 *                                    starts recording; capacity in [1, 65536].
 *   mlpmoe_profile_collect(ids, ms, capacity)  waits for the recorded events, writes up to
 *       capacity records in launch order (ids[i] = MLPMOE_KERNEL_*, ms[i] = duration in
 *       milliseconds), clears the record list and returns the number written (>= 0), or a
 *       negative error.  Launches beyond the enabled capacity are not recorded.
 *   mlpmoe_profile_disable()         stops recording and destroys the events.
 * Not thread safe; intended for one benchmarking thread.
 */
enum {
    MLPMOE_KERNEL_GATE_UP_MFMA = 1,
    MLPMOE_KERNEL_DOWN_MFMA = 2,
    MLPMOE_KERNEL_SPLITK_REDUCE = 3,
    MLPMOE_KERNEL_DECODE_GATE_UP = 4,
    MLPMOE_KERNEL_DECODE_DOWN = 5,
    MLPMOE_KERNEL_GATE_UP_GENERIC = 6,
    MLPMOE_KERNEL_DOWN_GENERIC = 7,
    MLPMOE_KERNEL_FILL_ZERO = 8,
    MLPMOE_KERNEL_ROUTE_TILES = 9
};
MLPMOE_API int mlpmoe_profile_enable(int capacity);
MLPMOE_API int mlpmoe_profile_collect(int *ids, float *ms, int capacity);
MLPMOE_API int mlpmoe_profile_disable(void);

/*
 * Plan: the branch table of one layer, checked and turned into the kernels' form once, together
 * with a device workspace large enough for any T up to max_T.  For callers that run the same
 * layer many times (decode loops, captured graphs): mlpmoe_plan_forward does no per-branch host
 * work, allocates nothing and synchronises nothing.
 *
 *   mlpmoe_plan_create   branch_offsets / alpha / active_mask / sizes as for mlpmoe_forward (host
 *                        arrays, copied); elem_bytes 2 (bf16) or 4 (float); max_T >= 1.  Allocates the
 *                        workspace on the current device.  *plan is NULL on failure.
 *   mlpmoe_plan_forward  x [T, d_model], weights and out [T, d_model] float: device pointers, 16-byte
 *                        aligned, same layouts as mlpmoe_forward; 0 <= T <= max_T (MLPMOE_ERR_SHAPE
 *                        otherwise); launches on `stream`.  Calls that share a plan share its workspace:
 *                        they must be ordered on one stream (or otherwise not overlap).
 *   mlpmoe_plan_destroy  synchronises the plan's device, frees the workspace and the plan (NULL is fine).
 */
typedef struct mlpmoe_plan mlpmoe_plan;
MLPMOE_API int mlpmoe_plan_create(const int32_t *branch_offsets, const float *alpha, const uint8_t *active_mask,
                                  int d_model, int d_inter, int B, int elem_bytes, int max_T,
                                  mlpmoe_plan **plan);
MLPMOE_API int mlpmoe_plan_forward(const mlpmoe_plan *plan, const void *x, const void *W_gate, const void *W_up,
                                   const void *W_down, int T, float *out, void *stream);
MLPMOE_API int mlpmoe_plan_destroy(mlpmoe_plan *plan);

/* Frees the library-owned per-device workspaces (synchronises each device first). */
MLPMOE_API int mlpmoe_release(void);

#ifdef __cplusplus
}
#endif
#endif /* MLPMOE_H */

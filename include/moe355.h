/*
 * moe355 -- one GPU's share of an expert-parallel MoE layer on AMD MI355X (gfx950).
 *
 * The calls follow the problem statement of "Accelerating MoE with Dynamic In-Switch Computing on
 * Multi-GPUs" (DySHARP): the gate produces the routing before Dispatch (Sec. III-E), Dispatch places
 * each token in the dense per-expert layout tensors of the GPUs that host its experts (Sec. III-D,
 * AL Table), the experts run GEMM-1 and GEMM-2 (Sec. II-A), GEMM-2's epilogue applies the gate weight
 * and Combine is an unweighted reduction of the k scaled outputs (Sec. III-C).  On one GPU the
 * multicast of Dispatch becomes "read each token row once per GPU" and the in-switch reduction of
 * Combine becomes "reduce a token's local partial outputs before its single write-back" (Sec. II-C).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; nothing is allocated, freed, copied to
 *     the host or synchronised by the library (one exception, stated where it is declared:
 *     moe_forward_status).  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on that stream only (one exception, stated where it is declared: moe_fused_backward
 *     with weight gradients), and is complete in that stream's order when the stream reaches the end of it.
 *   - State the library keeps between calls: per-device caches of two launch properties (the number of
 *     compute units, and that a kernel's dynamic-LDS limit has been raised), the static device scratch
 *     of moe_build_dispatch_noalloc, and moe_fused_backward's per-device side stream with its three events.
 *     Nothing else: every result depends on the arguments only.  These are set up by the first call that
 *     needs them on a device, which therefore must not run under stream capture.
 *   - Arrays are dense and row-major.  Inputs are never modified.  Outputs are fully overwritten.
 *   - Return value: MOE_OK (0) or a negative moe_status.  Argument validation happens before the first
 *     HIP call, so the error paths can be exercised on a host without a GPU.  No exception or abort
 *     crosses this boundary.
 *   - T == 0 is valid: tables describe an empty layer and y is not touched.
 *   - Preconditions that are NOT checked (the result is then unspecified, but no access leaves the
 *     caller's buffers): logits are finite; the k expert ids of a token are distinct and in [0, E).
 */
#ifndef MOE355_H
#define MOE355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE355_API __attribute__((visibility("default")))

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1, /* null pointer, E % R != 0, k out of range, bad local range, misaligned row size */
  MOE_ERR_UNSUPPORTED = -2, /* dtype or extent this build has no kernel for                                   */
  MOE_ERR_WORKSPACE = -3,   /* workspace pointer null or smaller than the matching *_workspace_bytes()         */
  MOE_ERR_HIP = -4          /* a kernel launch was rejected by the runtime                                     */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

/*
 * Layer shape.  T tokens, hidden size d, expert FFN width f, E experts in total, k experts per token,
 * R virtual ranks ("GPUs" of the expert-parallel group; expert e lives on rank e / (E/R), Sec. III-D).
 * This GPU hosts ranks [local_rank_begin, local_rank_end), i.e. experts
 * [local_rank_begin*E/R, local_rank_end*E/R), E_loc of them.
 * Limits: E % R == 0; 1 <= k <= min(E, 32); E <= 4096; d and f multiples of 8 (rows are 16-byte multiples).
 * dtype is the element type of x, the expert weights and y; accumulation is always fp32.
 */
typedef struct {
  int32_t T, d, f, E, k, R;
  int32_t local_rank_begin, local_rank_end;
  int32_t dtype; /* moe_dtype */
} moe_shape;

/*
 * Dispatch tables (all device pointers, caller-allocated).  A "pair" is (token t, slot j), id p = t*k + j.
 *   counts[e]        pairs routed to expert e  (the nactive[expert] of Sec. III-E)            [E]
 *   offsets[e]       first layout row of expert e; offsets[E] = number of valid pairs          [E+1]
 *   perm[row]        pair id stored in layout row `row` (token id list per tile, Sec. IV-B)    [T*k]
 *   inv_perm[p]      layout row of pair p (algebraic -> layout index, Sec. III-D); rows of one  [T*k]
 *                    expert are handed out in ascending token order
 *   rank_counts[r]   distinct tokens that have at least one slot on rank r                      [R]
 *   rank_offsets[r]  exclusive prefix sum; rank_offsets[R] = U_all, the number of entries below [R+1]
 *   dedup_tok[u]     token of entry u; entries are ordered by (rank, token)                     [T*min(k,R)]
 *   dedup_mask[u]    bit j set iff slot j of that token lies on that rank                       [T*min(k,R)]
 *   pair_to_dedup[p] entry index of (rank of pair p, token of pair p)                           [T*k]
 * Only the first rank_offsets[R] entries of dedup_tok / dedup_mask are written.
 */
typedef struct {
  int32_t *counts;
  int32_t *offsets;
  int32_t *perm;
  int32_t *inv_perm;
  int32_t *rank_counts;
  int32_t *rank_offsets;
  int32_t *dedup_tok;
  uint32_t *dedup_mask;
  int32_t *pair_to_dedup;
} moe_dispatch;

/*
 * Host-only size queries (no HIP call).  Return 0 for an invalid shape.  moe_workspace_bytes is enough for every
 * call of a step (moe_build_dispatch, then moe_fused_forward, on one stream with one buffer); the two specific
 * queries let a caller that keeps the buffers apart size the small one (dispatch: a few hundred KiB) on its own.
 */
MOE355_API size_t moe_workspace_bytes(const moe_shape *shape);
MOE355_API size_t moe_dispatch_workspace_bytes(const moe_shape *shape);
MOE355_API size_t moe_forward_workspace_bytes(const moe_shape *shape);
/* Bytes of the packed gate/up buffer (which = 0) or the packed down buffer (which = 1). */
MOE355_API size_t moe_packed_weight_bytes(const moe_shape *shape, int which);

/*
 * Gate network ahead of the routing (Sec. II-A: the experts of a token are "selected by the gate network"; the
 * reading used is a bias-free linear map).  logits [T,E] fp32 = x [T,d] times the rows of W_r [E,d] (one row per
 * expert, element type of the layer), accumulated in fp32 in a fixed order: the same inputs give the same bits,
 * and so the same routing.  x and W_r must be 16-byte aligned; workspace >= moe_router_workspace_bytes(shape)
 * (partial sums of the parts the reduction range is cut into).  The result feeds moe_route_topk.
 */
MOE355_API size_t moe_router_workspace_bytes(const moe_shape *shape);
MOE355_API int moe_router_logits(const moe_shape *shape, const void *x, const void *W_r, float *logits,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gate network and routing in one call (the "gate network" of Sec. II-A that selects each token's experts, from the
 * token rows to the picks): topk_idx / topk_w are those moe_route_topk gives on the logits moe_router_logits gives,
 * bit for bit (the same partial products, added in the same order), but the logits are summed inside the kernel that
 * picks and are written to `logits` [T,E] fp32 only if that pointer is not NULL.  x, W_r as for moe_router_logits;
 * workspace >= moe_route_from_x_workspace_bytes(shape), 16-byte aligned.
 */
MOE355_API size_t moe_route_from_x_workspace_bytes(const moe_shape *shape);
MOE355_API int moe_route_from_x(const moe_shape *shape, const void *x, const void *W_r, float *logits,
                                int32_t *topk_idx, float *topk_w, void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * Routing (Sec. II-A: each token activates the top-k experts chosen by the gate).
 * logits [T,E] fp32.  For each token the k largest logits are selected (ties: lower expert index first)
 * and reported in descending order in topk_idx [T,k]; topk_w [T,k] is the softmax over the logits
 * renormalised over the k picks (fp32, sums to 1).
 */
MOE355_API int moe_route_topk(const moe_shape *shape, const float *logits, int32_t *topk_idx, float *topk_w,
                              void *stream);

/*
 * Routing with the gate variants of DeepSeek-V3-style models (the paper evaluates that model and leaves the gate
 * function open, Sec. II-A).  gate = MOE_GATE_SOFTMAX: selection value logit + bias, weights as moe_route_topk;
 * gate = MOE_GATE_SIGMOID: s = 1 / (1 + exp(-logit)), selection value s + bias, weights = picked s divided by
 * their sum.  bias [E] fp32 (device; NULL = none) steers the selection only and never enters the weights.
 * Selection values are formed in fp32; k largest, lowest index on ties, slot order = pick order.  Other
 * arguments, outputs and errors as moe_route_topk; an unknown gate gives MOE_ERR_INVALID_ARG.
 */
#define MOE_GATE_SOFTMAX 0
#define MOE_GATE_SIGMOID 1
MOE355_API int moe_route_topk_gate(const moe_shape *shape, const float *logits, const float *bias, int gate,
                                   int32_t *topk_idx, float *topk_w, void *stream);

/*
 * Dispatch tables from the routing (Sec. III-D AL Table / Sec. III-E nactive / Sec. II-B redundancy).
 * Fills every array of `out` for all E experts and all R ranks (local or not).  The result is unique:
 * integer-exact and independent of scheduling.  workspace >= moe_dispatch_workspace_bytes(shape).
 */
MOE355_API int moe_build_dispatch(const moe_shape *shape, const int32_t *topk_idx, const moe_dispatch *out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * moe_build_dispatch for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same tables, bit for bit; the scratch (chunk histograms) is a static
 * device array of 64 * MOE_NOALLOC_MAX_COUNTERS int32 (256 KiB, held by every GPU the library runs on until the
 * process ends) instead of a caller workspace, so shapes with E + R > MOE_NOALLOC_MAX_COUNTERS are rejected with
 * MOE_ERR_UNSUPPORTED.  The call allocates and frees nothing.  All calls on one GPU share that GPU's array: calls
 * that overlap in time on the same GPU (different streams, different threads) race; calls on one stream do not.
 */
#define MOE_NOALLOC_MAX_COUNTERS 1024
MOE355_API int moe_build_dispatch_noalloc(const moe_shape *shape, const int32_t *topk_idx, const moe_dispatch *out,
                                          void *stream);

/*
 * One-off re-tiling of the static expert weights into the layout the GEMM kernels stream
 * (not part of the per-step path).  Inputs are the plain "input x output" matrices of the local experts:
 * W_gate, W_up [E_loc, d, f], W_down [E_loc, f, d].  Outputs are opaque buffers of
 * moe_packed_weight_bytes(shape, 0 / 1) bytes, 256-byte aligned, valid for any T.
 */
MOE355_API int moe_pack_weights(const moe_shape *shape, const void *W_gate, const void *W_up, const void *W_down,
                                void *packed_gate_up, void *packed_down, void *stream);

/*
 * Fused Dispatch -> GEMM-1 -> SwiGLU -> GEMM-2 (x gate weight) -> Combine for the local experts
 * (Sec. II-A, III-C, IV-A).  x [T,d]; y [T,d], y[t] = sum over the local slots j of token t of
 * topk_w[t,j] * FFN_{e(t,j)}(x[t]); rows of tokens without a local slot are written as zeros.
 * Token rows are gathered straight into the GEMM-1 tiles (no dispatched copy of x is materialised);
 * each y row is written exactly once, without atomics.  When moe_forward_gemm_launches(shape) is 1 (bf16 layers
 * with fewer than 256 rows per expert on average, T*k < 256*E), GEMM-1 and GEMM-2 run in ONE launch of resident
 * workgroups: a GEMM-2 tile starts as soon as the h rows of its 256-row tile are complete (per-tile readiness
 * counters in the workspace), the one-GPU form of the tile-granular GEMM-1 => GEMM-2 hand-over of the fused
 * kernel (Sec. IV-A, IV-B); otherwise the two GEMMs are two launches.  The result is the same either way.
 * A wait inside the resident kernel is bounded; if one gives up (corrupt tables; it cannot happen otherwise) the rows
 * computed from the incomplete tile are written as NaN and moe_forward_status reports 1 for this workspace.
 * `tables` must come from moe_build_dispatch on the same shape and topk_idx.
 * workspace >= moe_forward_workspace_bytes(shape), 256-byte aligned; its contents are scratch.  x, y and the
 * packed weights must be 16-byte aligned (MOE_ERR_INVALID_ARG otherwise).
 */
MOE355_API int moe_fused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                 const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                 const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                 void *stream);

/*
 * moe_fused_forward with the kernel boundaries marked for measurement: `events` points at five hipEvent_t
 * (created by the caller with timing enabled; a NULL entry is skipped) which are recorded on `stream`
 * [0] before the first kernel, [1] after the tile-table kernel, [2] after GEMM-1, [3] after GEMM-2 (recorded
 * together, after the one launch, when moe_forward_gemm_launches(shape) is 1), [4] after Combine.
 * The kernels and their order are those of moe_fused_forward.
 */
MOE355_API int moe_fused_forward_timed(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                       const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                       const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                       void *stream, void *const *events);

/*
 * *flag (host) = 0, or 1 if a wait inside the resident GEMM kernel of the last forward call that used `workspace`
 * gave up.  The one call of this library that copies to the host and synchronises with `stream`; for diagnostics.
 *
 * moe_fused_forward_bounded: moe_fused_forward_one_launch with the bound on the polls of one wait given by the caller
 * (max_polls >= 1, each poll about a microsecond; the library's default is several seconds) and with every GEMM-2 tile
 * waiting for wait_extra more GEMM-1 tiles than exist (0 = the real count).  With wait_extra > 0 and a small bound
 * every wait gives up, all kernels still exit normally, y holds NaN in every row with a local slot and
 * moe_forward_status reports 1: the way the give-up path is tested.
 */
MOE355_API int moe_forward_status(const void *workspace, int32_t *flag, void *stream);
MOE355_API int moe_fused_forward_bounded(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                         const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                         const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                         void *stream, int max_polls, int wait_extra);

/* 1 or 2: GEMM launches of moe_fused_forward for this shape (host-only; 0 for an invalid shape). */
MOE355_API int moe_forward_gemm_launches(const moe_shape *shape);

/*
 * moe_fused_forward with the choice between the two forms of the GEMM-1 => GEMM-2 hand-over made by the caller
 * (comparison of the two, timing of the two GEMMs apart): _two_launch keeps a kernel boundary between the GEMMs,
 * _one_launch runs the resident kernel with per-tile readiness counters (bf16 layers only, MOE_ERR_UNSUPPORTED
 * otherwise).  Same arguments, workspace and result as moe_fused_forward; `events` may be NULL, otherwise five
 * events as in moe_fused_forward_timed.
 */
MOE355_API int moe_fused_forward_two_launch(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                            const float *topk_w, const moe_dispatch *tables,
                                            const void *packed_gate_up, const void *packed_down, void *y,
                                            void *workspace, size_t workspace_bytes, void *stream,
                                            void *const *events);
MOE355_API int moe_fused_forward_one_launch(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                            const float *topk_w, const moe_dispatch *tables,
                                            const void *packed_gate_up, const void *packed_down, void *y,
                                            void *workspace, size_t workspace_bytes, void *stream,
                                            void *const *events);

/*
 * moe_fused_forward_resident: the tile table, then ONE launch of resident workgroups (one per compute unit) that runs
 * GEMM-1 (token gather fused), GEMM-2 and Combine: the fused-kernel structure of Sec. IV-A with readiness-gated issue
 * (Sec. IV-B, IV-C) on one GPU.  A workgroup that finds no GEMM-1 item left takes GEMM-2 items (each waits for the
 * counter of its M tile's GEMM-1 items), and one that finds no GEMM-2 item left reduces tokens, one wave per token:
 * the wave waits for the counters of finished GEMM-2 items of every M tile that holds one of the token's rows, then
 * sums the rows in slot order.  y is bit-identical to moe_fused_forward's.  bf16 layers with at most 4091 local experts (the
 * tile table's LDS), MOE_ERR_UNSUPPORTED otherwise.  Arguments as
 * moe_fused_forward_one_launch ([2] and [3] of `events` are recorded together after the launch, [4] right after);
 * max_polls: bound on the polls of one wait (0 = the library's default of several seconds); wait_extra: every wait
 * expects that many more finished tiles than exist (0 in normal use; > 0 with a small bound is the test of the
 * give-up path: all kernels still exit, rows computed from incomplete data are NaN, moe_forward_status reports 1).
 */
MOE355_API int moe_fused_forward_resident(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                          const float *topk_w, const moe_dispatch *tables,
                                          const void *packed_gate_up, const void *packed_down, void *y,
                                          void *workspace, size_t workspace_bytes, void *stream,
                                          void *const *events, int max_polls, int wait_extra);

/*
 * Phase-split entry points, used to measure Dispatch and Combine on their own (Sec. VI "pure
 * communication" test) and as building blocks of the unfused comparison path.
 *
 * moe_dispatch_gather: materialise the local layout tensor xs [P_cap, d] (P_cap = T*min(k,E_loc) rows):
 *   every entry of the dedup table that belongs to a local rank reads its token row once and writes it
 *   to the layout row of each of its slots (the one-GPU form of the multicast of Sec. II-C).
 * moe_combine_reduce: rows [P_cap, d] fp32 are the gate-weighted expert outputs in layout order;
 *   y[t] = sum of the rows of t's local slots (slot order), one write per token, zeros if none.
 */
MOE355_API int moe_dispatch_gather(const moe_shape *shape, const void *x, const moe_dispatch *tables, void *xs,
                                   void *stream);
MOE355_API int moe_combine_reduce(const moe_shape *shape, const float *rows, const int32_t *topk_idx,
                                  const moe_dispatch *tables, void *y, void *stream);

/*
 * Unfused comparison path (Sec. V-C style baseline without redundancy removal): explicit gather copy,
 * the same grouped GEMMs on the copied rows, then a scatter-add of every weighted row into a zeroed fp32
 * buffer with atomics, then a cast to y.  Same arguments as moe_fused_forward; needs
 * moe_unfused_workspace_bytes(shape).
 */
MOE355_API size_t moe_unfused_workspace_bytes(const moe_shape *shape);
MOE355_API int moe_unfused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                   const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                   const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                   void *stream);

/*
 * FP8 form of the expert GEMMs (Sec. V-A: the DeepSeek-V3 runs use FP8 GEMM kernels; the paper gives no scheme).
 * For bf16 layers (shape->dtype == MOE_BF16) with d % 16 == 0 and f % 16 == 0, MOE_ERR_UNSUPPORTED otherwise.
 * Operands of both GEMMs are E4M3 codes of the OCP 8-bit floating point format (round to nearest even, saturating
 * at +-448), products are accumulated in fp32:
 *   x       one scale per token   = largest magnitude of the row / 448 (1 for a zero row), code = cvt(x / scale);
 *   weights one scale per expert and output column, same rule over the reduction index;
 *   h       code = cvt(silu(g) * u / h_scale[le]) with a given (calibrated, static) scale per local expert
 *           (finite and > 0; values beyond 448 * h_scale[le] saturate);
 *   g, u = (sum of code products) * scale(token) * scale(column);  o = (sum) * h_scale[le] * scale(column) * w.
 * y, the tables, the gate weights and the reduction are those of moe_fused_forward (y in bf16).
 *
 * moe_fp8_pack_weights: one-off; quantises the bf16 weights (same layouts as moe_pack_weights) and writes the
 *   tiles followed by the column scales into buffers of moe_fp8_packed_weight_bytes(shape, 0 / 1) bytes, 16-byte
 *   aligned.
 * moe_fp8_quantize_rows: the activation quantiser on its own: x [rows, cols] bf16 (16-byte aligned, cols % 8 == 0)
 *   -> codes [rows, cols] (8-byte aligned), scales [rows].  moe_fp8_fused_forward runs it on x internally.
 * moe_fp8_fused_forward: as moe_fused_forward with the packed FP8 weights and h_scale [E_loc] (device);
 *   workspace >= moe_fp8_forward_workspace_bytes(shape), 256-byte aligned; the two GEMMs run as one or two launches
 *   by the rule of moe_forward_gemm_launches.  `events` may be NULL, otherwise five events as in
 *   moe_fused_forward_timed ([1] follows the quantisation of x and the tile table).
 */
MOE355_API size_t moe_fp8_packed_weight_bytes(const moe_shape *shape, int which);
MOE355_API size_t moe_fp8_forward_workspace_bytes(const moe_shape *shape);
MOE355_API int moe_fp8_pack_weights(const moe_shape *shape, const void *W_gate, const void *W_up, const void *W_down,
                                    void *packed_gate_up, void *packed_down, void *stream);
MOE355_API int moe_fp8_quantize_rows(int64_t rows, int cols, const void *x, void *codes, float *scales, void *stream);
MOE355_API int moe_fp8_fused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                     const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                     const void *packed_down, const float *h_scale, void *y, void *workspace,
                                     size_t workspace_bytes, void *stream, void *const *events);

/*
 * Training path (the paper's end-to-end results cover forward and backward, Sec. V; it gives no formulas: these are
 * the derivatives of the layer as moe_fused_forward computes it).  bf16 layers with f % 64 == 0, MOE_ERR_UNSUPPORTED
 * otherwise.  For a local row (token t, slot j, local expert le, gate weight w) and the incoming gradient dy_t:
 *   dh_raw = dy_t Wd^T, d_topk_w[t,j] = <o, dy_t> (formed as <w o, dy_t> / w from the kept rows; reported as 0 where
 *   w underflowed to exactly 0), dh = w dh_raw, dg = dh u silu'(g), du = dh silu(g),
 *   dx_t = sum over the local slots of dg Wg^T + du Wu^T,
 *   dW_gate[le] = sum over the expert's rows of x_t^T dg, dW_up likewise with du, dW_down[le] = sum of h^T (w dy_t).
 * Only local slots contribute (one GPU's share): dx rows of tokens without a local slot are zero, d_topk_w is zero
 * for slots whose expert is not local.
 *
 * moe_fused_forward_train: moe_fused_forward that also keeps g, u (bf16) and every weighted expert output row (fp32)
 *   in `kept` (caller-owned, >= moe_train_kept_bytes(shape), 256-byte aligned), which the backward call reads.
 *   The two GEMMs run as one or two launches by the rule of moe_forward_gemm_launches.
 * moe_pack_weights_backward: one-off; the transposed uses of the weights in the layout the GEMM kernels stream:
 *   packed_down_t (W_down^T) and packed_gate_up_t ([W_gate^T ; W_up^T]), moe_backward_packed_weight_bytes(shape, 0 / 1)
 *   bytes, 16-byte aligned.  Inputs as for moe_pack_weights.
 * moe_fused_backward: x, dy [T,d] bf16; the routing and tables of the forward; dx [T,d] bf16 and d_topk_w [T,k] fp32
 *   are written in full.  dW_gate, dW_up [E_loc,d,f] and dW_down [E_loc,f,d] (bf16, 16-byte aligned, written in full, zero for
 *   an expert without rows) are computed when all three pointers are non-NULL and skipped when all three are NULL.
 *   workspace >= moe_backward_workspace_bytes(shape), 256-byte aligned.  Sums run in a fixed order: same inputs,
 *   same bits.  With weight gradients, the transposed copies of the operands are made on a stream of the library's
 *   own (one per device, default priority, created by the first such call and kept) beside the two GEMMs: it waits
 *   for an event recorded on `stream` and `stream` waits for its last kernel before the products start, so the call's
 *   work is ordered in `stream` like any other call's, also inside a stream capture (later calls only: see above).
 *   Calls from several host threads on one device share that side stream: the library serialises their enqueueing
 *   (a mutex held for the duration of the call) and their side work runs in turn; they still need separate workspaces.
 */
MOE355_API size_t moe_train_kept_bytes(const moe_shape *shape);
MOE355_API size_t moe_backward_workspace_bytes(const moe_shape *shape);
MOE355_API size_t moe_backward_packed_weight_bytes(const moe_shape *shape, int which);
MOE355_API int moe_pack_weights_backward(const moe_shape *shape, const void *W_gate, const void *W_up,
                                         const void *W_down, void *packed_down_t, void *packed_gate_up_t,
                                         void *stream);
MOE355_API int moe_fused_forward_train(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                       const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                       const void *packed_down, void *y, void *kept, size_t kept_bytes,
                                       void *workspace, size_t workspace_bytes, void *stream);
MOE355_API int moe_fused_backward(const moe_shape *shape, const void *x, const void *dy, const int32_t *topk_idx,
                                  const float *topk_w, const moe_dispatch *tables, const void *packed_down_t,
                                  const void *packed_gate_up_t, const void *kept, size_t kept_bytes, void *dx,
                                  float *d_topk_w, void *dW_gate, void *dW_up, void *dW_down, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Backward of moe_route_topk's weights (a softmax over the k picked logits; the selection is piecewise constant):
 * dlogits [T,E] fp32 (written in full) = w_j (d_topk_w_j - sum_i w_i d_topk_w_i) at the picked experts, 0 elsewhere.
 * topk_idx, topk_w as written by moe_route_topk; d_topk_w [T,k] fp32, e.g. from moe_fused_backward.
 */
MOE355_API int moe_route_backward(const moe_shape *shape, const int32_t *topk_idx, const float *topk_w,
                                  const float *d_topk_w, float *dlogits, void *stream);

/* Static string for a status code. */
MOE355_API const char *moe_status_string(int status);

/*
 * Measurement harness only (define MOE355_BENCH before including this header; no part of the layer calls it): one
 * launch of `workgroups` x 512 threads in which every wave issues `iters` rounds of eight independent bf16 32x32x16
 * matrix-core instructions on pseudo-random register operands, the rate this device's matrix cores sustain when
 * nothing has to be loaded.  *flops (host) receives the floating point operations of the launch; the caller times it.
 * sink: device scratch of >= workgroups * 512 floats.
 */
#ifdef MOE355_BENCH
MOE355_API int moe_probe_mfma_rate(int workgroups, int iters, float *sink, size_t sink_floats, double *flops,
                                   void *stream);
#endif

#ifdef __cplusplus
}
#endif
#endif /* MOE355_H */

/*
 * camera.h -- C ABI of the MI355X (gfx950) CAMERA micro-expert scoring library.
 *
 * The library computes, for one MoE layer, what the paper's Algorithm 1
 * ("CAMERA -- Micro-Experts Ranking") computes, and the two decisions that
 * Algorithms 2 and 3 take from its ranking.  A micro-expert (e, c) is gate row
 * c, up row c and down column c of expert e (Section "From Expert to
 * Micro-Expert", Eq. 3); its global index in every per-layer vector is
 * e * d_ff + c (0-based).
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless the comment says HOST.  All tensors
 *     are row-major.  The caller owns every buffer and the stream; the library
 *     keeps nothing of the caller's beyond the stream work it enqueues.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue their kernels on it and return without waiting.  A context
 *     must not be used from two streams at the same time: its workspace is
 *     shared by consecutive calls and ordered only by the stream.
 *   - Return value: CAMERA_OK (0) or a negative camera_status.  All argument
 *     checks run on the host before any GPU call; camera_last_error() then
 *     names the offending argument.  No exception or abort crosses this ABI.
 *   - The context owns a grow-only device workspace (hipMalloc on first use and
 *     on growth, which synchronises the device) and, for the ranking calls, a
 *     small persistent selection state made on their first use.
 *   - NaN / Inf in the inputs: results unspecified (not checked).
 *   - Device data pointers must be 16-byte aligned; for CAMERA_BF16 d_model and
 *     ldx must be multiples of 8, for CAMERA_F32 multiples of 4.
 */
#ifndef CAMERA_H_
#define CAMERA_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct camera_ctx camera_ctx; /* opaque, library-owned */

enum camera_status {
  CAMERA_OK = 0,
  CAMERA_EINVAL = -1,       /* NULL pointer, value out of range */
  CAMERA_ESHAPE = -2,       /* size / stride / alignment not accepted */
  CAMERA_EDTYPE = -3,       /* unknown dtype code */
  CAMERA_EWORKSPACE = -4,   /* workspace allocation failed */
  CAMERA_EHIP = -5,         /* a HIP runtime call failed (text in camera_last_error) */
  CAMERA_EUNSUPPORTED = -6  /* valid request outside the built limits */
};

enum camera_dtype { CAMERA_F32 = 0, CAMERA_BF16 = 1 };

enum camera_flags {
  CAMERA_ACCUMULATE = 1, /* phi2 / phi_inf already hold earlier token chunks: merge into them */
  CAMERA_NO_FINALIZE = 2 /* more chunks follow: leave omega2 and energy untouched */
};

/* Limits of this build. */
#define CAMERA_MAX_EXPERTS 256   /* routed experts per call */
#define CAMERA_MAX_SEGMENTS 512  /* expert segments in select / alloc */
#define CAMERA_MAX_LEVELS 8      /* precision classes in camera_alloc_bits */
#define CAMERA_MAX_ROW_ALIGN 512 /* largest row alignment (elements) of the compacted W_down blocks */

/* Kernel groups for camera_profile_read. */
enum camera_kernel_id {
  CAMERA_K_ROUTE = 0,
  CAMERA_K_BUCKET = 1,
  CAMERA_K_GEMM = 2,     /* grouped gate/up contraction + fused epilogue */
  CAMERA_K_DOWN_NORM = 3,
  CAMERA_K_FINALIZE = 4,
  CAMERA_K_RANK = 5,
  CAMERA_K_GATHER = 6,   /* camera_gather_micro_experts */
  CAMERA_K_DOWN_GEMM = 7, /* camera_layer_forward: hidden activations times W_down^T */
  CAMERA_K_COMBINE = 8,  /* camera_layer_forward: sum over a token's experts; camera_output_error */
  CAMERA_K_COMPACT_HIDDEN = 9, /* camera_layer_forward_compact: Lambda on the kept gate / up rows */
  CAMERA_K_COMPACT_DOWN = 10,  /* camera_layer_forward_compact: Lambda times the kept W_down columns */
  CAMERA_K_COUNT = 11
};

/* Create / destroy a context bound to HIP device `device`.  Creation touches no
 * GPU; device resources are made on the first compute call. */
int camera_create(camera_ctx** out, int device);
int camera_destroy(camera_ctx* ctx);

/* HOST string describing the last error of this context (valid until its next
 * call); with ctx == NULL, the last error of a failed camera_create. */
const char* camera_last_error(const camera_ctx* ctx);

/* Library ABI version (currently 1). */
int camera_version(void);

/*
 * A = Top&Norm(R X)  -- Algorithm 1, line 2; router weights A_i(x) of Eq. 2.
 *
 *   X        [n x d_model], row stride ldx elements, `dtype`
 *   W_r      [n_experts x d_model], row stride ldr, `dtype`  (router R)
 *   bias     [n_experts] float32 added to the logits, or NULL
 *   topk_idx [n x top_k] int32 out: the top_k experts with the largest logits,
 *            largest first, equal logits to the lower expert index
 *   topk_w   [n x top_k] float32 out: softmax probability (over all n_experts)
 *            of each kept expert; with renorm != 0 divided by the sum of the
 *            kept probabilities ("Norm"), so each row sums to 1
 * Logits are accumulated in float32.  1 <= top_k <= n_experts <= CAMERA_MAX_EXPERTS.
 * n == 0 is accepted and does nothing.
 */
int camera_route_topk(camera_ctx* ctx, void* stream,
                      const void* X, int dtype, int64_t n, int64_t d_model, int64_t ldx,
                      const void* W_r, int64_t ldr, const float* bias,
                      int n_experts, int top_k, int renorm,
                      int32_t* topk_idx, float* topk_w);

/*
 * Algorithm 1, lines 3-10 for one group of experts: per micro-expert
 *   phi2    = sum_j Lambda[j,c]^2            (line 7)
 *   phi_inf = (max_j |Lambda[j,c]|)^2        (line 8)
 *   omega2  = sum_r W_down[r,c]^2            (line 5)
 *   energy  = [(1-alpha) phi2 + alpha phi_inf] * omega2     (line 10, energy with
 *             the balance coefficient alpha)
 * with Lambda[j,c] = a_j * silu(<w_gate_c, x_j>) * <w_up_c, x_j>  (line 6, Eq. 4)
 * taken over the tokens j routed to the expert.  Lambda is never stored.
 *
 *   X         [n x d_model], row stride ldx, `dtype`
 *   topk_idx  [n x top_k] int32 and topk_w [n x top_k] float32 as written by
 *             camera_route_topk.  Entries outside [0, n_experts) are ignored.
 *             Both NULL (top_k ignored): every expert sees every token with
 *             weight 1 -- a shared expert or a dense FFN.
 *   W_gate, W_up  [n_experts][d_ff][d_model] `dtype`, expert stride stride_gu
 *             elements (>= d_ff*d_model), rows contiguous
 *   W_down    [n_experts][d_model][d_ff] `dtype`, expert stride stride_down
 *             elements; column c belongs to micro-expert c
 *   alpha     in [0, 1]
 *   flags     0: one call covers all tokens.  CAMERA_ACCUMULATE: phi2 / phi_inf
 *             are in-out and this chunk of tokens is merged into them (sum /
 *             max).  CAMERA_NO_FINALIZE: omega2 and energy are not written (may
 *             be NULL).
 *   phi2, phi_inf, omega2, energy   float32 [n_experts * d_ff] out
 * Contractions run on bf16 MFMA with float32 accumulation (CAMERA_BF16) or in
 * float32 FMA (CAMERA_F32); the result does not depend on launch order (no
 * floating-point atomics).  n == 0 gives phi2 = phi_inf = 0 (or leaves them
 * unchanged under CAMERA_ACCUMULATE).
 */
int camera_score_layer(camera_ctx* ctx, void* stream,
                       const void* X, int dtype, int64_t n, int64_t d_model, int64_t ldx,
                       const int32_t* topk_idx, const float* topk_w, int top_k,
                       int n_experts, int64_t d_ff,
                       const void* W_gate, const void* W_up, int64_t stride_gu,
                       const void* W_down, int64_t stride_down,
                       float alpha, int flags,
                       float* phi2, float* phi_inf, float* omega2, float* energy);

/*
 * S = TopSelect(R, 1 - lambda)  -- Algorithm 2 (CAMERA-P), line 9, on the
 * ranking of Algorithm 1 line 11.  The order is the stable ascending order of
 * (energy, index); the first n_prune = floor(ratio * n_micro + 1e-6)
 * micro-experts are removed, the rest kept.  -0.0 counts as +0.0.
 *
 *   energy          float32 [n_micro]
 *   seg_offsets     HOST int64 [n_seg + 1], rising from 0 to n_micro: expert
 *                   boundaries (n_seg <= CAMERA_MAX_SEGMENTS)
 *   ratio           lambda in [0, 1]
 *   keep_mask       uint8 [n_micro] out: 1 kept, 0 pruned
 *   kept_per_expert int32 [n_seg] out: kept micro-experts of every segment
 *   kept_idx        int32 [n_micro - n_prune] out or NULL: kept global indices,
 *                   ascending (so grouped by expert)
 *   rank            uint32 [n_micro] out or NULL: position of every micro-expert
 *                   in the ascending order (0 = most redundant)
 */
int camera_select_prune(camera_ctx* ctx, void* stream,
                        const float* energy, int64_t n_micro,
                        const int64_t* seg_offsets, int n_seg, double ratio,
                        uint8_t* keep_mask, int32_t* kept_per_expert,
                        int32_t* kept_idx, uint32_t* rank);

/*
 * camera_select_prune for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, order, counts and outputs as
 * camera_select_prune without the `rank` output, but the kernels' scratch (class bytes, select histograms,
 * per-workgroup counts) lies in a static device array of the library instead of the context workspace: the
 * call makes no hipMalloc / hipFree and no other allocating call.  The array (1.5 MiB) exists once per GPU
 * for the life of the process and serves n_micro <= CAMERA_NOALLOC_MAX_MICRO; larger inputs are refused with
 * CAMERA_EUNSUPPORTED before anything is launched.  All calls on one GPU share that array, whatever their
 * context or stream: calls that overlap in time on one GPU race (order them on one stream or with events).
 * The first call on a device looks up the array's address (no stream work); make it outside a graph capture.
 */
#define CAMERA_NOALLOC_MAX_MICRO (1 << 20)
int camera_select_prune_noalloc(camera_ctx* ctx, void* stream,
                                const float* energy, int64_t n_micro,
                                const int64_t* seg_offsets, int n_seg, double ratio,
                                uint8_t* keep_mask, int32_t* kept_per_expert, int32_t* kept_idx);

/*
 * TopSelect at several ratios from one pass over the ranking (the masks at 20 / 40 / 60 % of "Main Results"
 * come from one set of scores).  Same order and counts as camera_select_prune.
 *   ratios          HOST [n_ratios], each in [0, 1], not falling; n_ratios <= CAMERA_MAX_LEVELS - 1
 *   keep_bits       uint8 [n_micro] out: bit k is set iff the micro-expert is kept at ratios[k]
 *                   (bit k of element i == keep_mask[i] of camera_select_prune at ratios[k])
 *   kept_per_expert int32 [n_ratios x n_seg] out: row k = kept_per_expert of camera_select_prune at ratios[k]
 */
int camera_select_prune_multi(camera_ctx* ctx, void* stream,
                              const float* energy, int64_t n_micro,
                              const int64_t* seg_offsets, int n_seg,
                              int n_ratios, const double* ratios,
                              uint8_t* keep_bits, int32_t* kept_per_expert);

/*
 * S_1..S_L = ListSplitByRatio(R, r_1..r_L) and the per-expert GetSubIndex --
 * Algorithm 3 (CAMERA-Q), lines 5-8; precision levels and proportions as in the
 * appendix "Mixed-precision Settings".  Class 0 is the fraction ratios[0] with
 * the highest energy and gets bits[0]; boundaries are the cumulative floors
 * cut_m = floor((r_1+..+r_m) * n_micro + 1e-6) counted from the most important
 * end, on the same order as camera_select_prune.
 *
 *   bits, ratios   HOST arrays [n_levels]; ratios >= 0 and sum to 1 (1e-9)
 *   bit_of         uint8 [n_micro] out: bit width of every micro-expert
 *   level_count    int32 [n_seg x n_levels] out: class sizes per expert
 *   perm           int32 [n_micro] out or NULL: inside every expert's range,
 *                  the members of class 0 first, then class 1, ..., each in
 *                  ascending index order (the reordering that colocates equal
 *                  precision inside an expert, Section "Mixed-precision
 *                  Strategy CAMERA-Q")
 */
int camera_alloc_bits(camera_ctx* ctx, void* stream,
                      const float* energy, int64_t n_micro,
                      const int64_t* seg_offsets, int n_seg,
                      int n_levels, const int* bits, const double* ratios,
                      uint8_t* bit_of, int32_t* level_count, int32_t* perm);

/*
 * Both decisions of a layer from one pass over its ranking: the CAMERA-P masks at n_ratios pruning ratios
 * (Algorithm 2, line 9: TopSelect) and one CAMERA-Q bit allocation (Algorithm 3, lines 5-8: ListSplitByRatio and
 * GetSubIndex).  The pruning thresholds and the class boundaries are all cuts on the same stable ascending order of
 * (energy, index), so one set of selection passes serves both.  Arguments and outputs as in
 * camera_select_prune_multi (ratios, keep_bits, kept_per_expert) and camera_alloc_bits (bits, level_ratios, bit_of,
 * level_count, perm), bit for bit the same results as those two calls.  n_ratios >= 1, n_levels >= 1 and
 * n_ratios + n_levels - 1 <= CAMERA_MAX_LEVELS - 1 (the cuts one pass carries).
 */
int camera_rank_decisions(camera_ctx* ctx, void* stream,
                          const float* energy, int64_t n_micro,
                          const int64_t* seg_offsets, int n_seg,
                          int n_ratios, const double* ratios, uint8_t* keep_bits, int32_t* kept_per_expert,
                          int n_levels, const int* bits, const double* level_ratios,
                          uint8_t* bit_of, int32_t* level_count, int32_t* perm);

/*
 * W_up, W_gate, W_down <- W_up[S,:], W_gate[S,:], W_down[:,S]  -- Algorithm 2 (CAMERA-P), lines 10-13: only
 * the micro-experts in S are kept, and all three of their vectors move together.  With the `perm` of
 * camera_alloc_bits as the index list (count NULL) the same call is the reordering inside every expert
 * that colocates micro-experts of equal precision (Section "Mixed-precision Strategy CAMERA-Q").
 *
 *   W_gate, W_up, W_down, strides, n_experts, d_ff, d_model, dtype: one group of experts, as in
 *               camera_score_layer.  d_ff * element size must not exceed 65536 bytes.
 *   index       int32 [n_index]: global micro-expert indices index_base + e*d_ff + c, grouped by
 *               expert in expert order -- camera_select_prune's kept_idx or camera_alloc_bits' perm
 *               (for the second group of a layer: its slice of them, with index_base = the global
 *               index of the group's first micro-expert)
 *   count       int32 [n_experts]: entries of `index` that belong to each expert (camera_select_prune's
 *               kept_per_expert), or NULL: d_ff each
 *   down_row_align   the rows of every W_down_out block are ld(e) = count[e] rounded up to a multiple of
 *               this many elements long, the surplus filled with zeros; 1: no padding.  64 (bf16: 128
 *               bytes) makes every row start on a cache line, which is what camera_layer_forward_compact
 *               reads fastest.  1 <= down_row_align <= CAMERA_MAX_ROW_ALIGN.
 *   W_gate_out, W_up_out   [n_index][d_model] out, `dtype`: row r is the gate / up row of index[r]
 *   W_down_out  out, `dtype`, d_model * (ld(0) + ... + ld(n_experts-1)) elements: expert e's block starts
 *               at element d_model * (ld(0) + ... + ld(e-1)) and is [d_model][ld(e)] row-major; its column
 *               j < count[e] is the down column of the expert's j-th entry
 *   Any of the three outputs may be NULL (skipped); the matching input may then be NULL too.
 * Values are copied bit for bit.  An entry that does not lie inside its expert's range gives a zero
 * row / column; if the counts add up to less than n_index the remaining output rows are left
 * untouched, if to more, the surplus entries are ignored.  n_index == 0 does nothing.
 */
int camera_gather_micro_experts(camera_ctx* ctx, void* stream, int dtype,
                                int n_experts, int64_t d_ff, int64_t d_model,
                                const void* W_gate, const void* W_up, int64_t stride_gu,
                                const void* W_down, int64_t stride_down,
                                const int32_t* index, int64_t n_index, int64_t index_base,
                                const int32_t* count, int down_row_align,
                                void* W_gate_out, void* W_up_out, void* W_down_out);

/*
 * The comparison variant CAMERA-Q-dagger (Section "Experimental Setup", mixed-precision paragraph; Section
 * "Micro-Expert Integrity"): mixed precision by slicing every matrix along its input dimension, W_up[:, s_k],
 * W_gate[:, s_k], W_down[:, s_k], as single-matrix schemes do that rank input channels by H = X X^T.  For W_down the
 * input dimension is d_ff, so its split is CAMERA-Q's own.  For W_up and W_gate it is d_model; the statistic such
 * schemes rank by is returned here:
 *   h[e * d_model + c] = sum over the tokens j routed to expert e of X[j, c]^2        (the diagonal of X_e^T X_e)
 * camera_alloc_bits on h (segments of d_model per expert) then gives the bit width of every input column and the
 * per-expert reordering, and camera_gather_micro_experts with W_up (or W_gate) in the place of W_down, d_ff and
 * d_model exchanged, applies it (the columns of equal precision side by side).
 *   X, dtype, n, d_model, ldx: as in camera_score_layer
 *   topk_idx  [n x top_k] int32, entries outside [0, n_experts) ignored; NULL: every expert sees every token
 *   h         float32 [n_experts * d_model] out
 * float32 accumulation in a fixed order (bit-reproducible).  n == 0 gives zeros.
 */
int camera_input_channel_energy(camera_ctx* ctx, void* stream,
                                const void* X, int dtype, int64_t n, int64_t d_model, int64_t ldx,
                                const int32_t* topk_idx, int top_k, int n_experts, float* h);

/*
 * The layer output over a subset of the micro-experts (Eq. 1-2; the output recomputed after pruning in
 * Algorithm 2, line 14):
 *   Y[j, :] = sum over experts e and kept channels c of  Lambda_e[j, c] * W_down,e[:, c],
 *   Lambda_e[j, c] = a_j,e * silu(<w_gate_c, x_j>) * <w_up_c, x_j>           (Eq. 4)
 * X, routing, weights, strides: as in camera_score_layer; d_ff and stride_down multiples of 8 (CAMERA_BF16) or 4
 * (CAMERA_F32).
 *   keep_mask  uint8 [n_experts * d_ff], 0 = pruned (gate row, up row and down column all drop out), or NULL:
 *              every micro-expert kept (the original layer).  For the second group of a layer pass the
 *              group's slice of camera_select_prune's keep_mask.
 *   flags      0: Y is overwritten; CAMERA_ACCUMULATE: the group's output is added to Y (routed experts
 *              first, then the shared ones into the same Y)
 *   Y          float32 [n x d_model] in-out, rows contiguous
 * With CAMERA_BF16 Lambda is rounded to bf16 before the second contraction, as the hidden activations of a
 * 16-bit model are (CAMERA_F32 keeps it in float32); both contractions accumulate in float32, and a token's experts are added in the order of its
 * top-k list (no floating-point atomics: the result does not depend on launch order).  The context
 * workspace grows by n*top_k*(2*d_ff + 4*d_model) bytes.  n == 0 does nothing.
 *
 * camera_output_error: distance of a pruned layer's output from the original one, per token
 *   per_token [n x 4] float32 out: ||y - y_hat||^2, ||y||^2, ||y_hat||^2, <y, y_hat>
 * (their sums over tokens give the decoding error of the Lemma, ||Y - Y_hat||_F and the cosine
 * similarity reported for hidden states after pruning).  Y, Y_hat [n x d_model] float32, rows contiguous.
 */
int camera_layer_forward(camera_ctx* ctx, void* stream,
                         const void* X, int dtype, int64_t n, int64_t d_model, int64_t ldx,
                         const int32_t* topk_idx, const float* topk_w, int top_k,
                         int n_experts, int64_t d_ff,
                         const void* W_gate, const void* W_up, int64_t stride_gu,
                         const void* W_down, int64_t stride_down,
                         const uint8_t* keep_mask, int flags, float* Y);

/*
 * The output of a pruned layer from its compacted weights (Algorithm 2, line 14, on the matrices that
 * lines 10-13 leave: expert e keeps count[e] micro-experts), for the small token batches of decoding
 * (the decoding-speed comparison of a pruned MoE layer, batch of 64 tokens).  Same result as
 * camera_layer_forward with the keep mask that the compaction was made from, but only the kept
 * weights are read, each activated expert's once per 64 of its tokens, and the experts that no token
 * of the batch selected are not read at all: the call is bound by HBM reads, not by arithmetic.
 *
 *   X, n, d_model, ldx, topk_idx, topk_w, top_k, n_experts, flags, Y: as in camera_layer_forward
 *               (topk_idx = topk_w = NULL: every token goes through every expert with weight 1).
 *               Any n is accepted: small batches stream an expert's weights once per 32 of its
 *               tokens; from 64 tokens per expert on average the call runs on the tiled MFMA kernel
 *               of camera_layer_forward with per-expert widths, provided down_row_align is a
 *               multiple of 8 and d_model a multiple of 16 (else it stays on the streaming kernels).
 *   n_shared    experts n_experts .. n_experts + n_shared - 1 are shared experts: every token goes
 *               through them with weight 1, in the same launches as the routed ones (a decoding
 *               batch is too small to fill the chip with the shared experts alone).  0 without routing.
 *   dtype       CAMERA_BF16 only (CAMERA_EUNSUPPORTED otherwise); Lambda is rounded to bf16 before
 *               the second contraction, float32 accumulation in both
 *   count       HOST int32 [n_experts + n_shared]: kept micro-experts of every expert (>= 0, any value)
 *   down_row_align   the row alignment the W_down blocks were gathered with: ld(e) = count[e] rounded
 *               up to a multiple of it.  Any value gives the same result; rows that start on 128-byte
 *               lines (64 for bf16) are read about a third faster than rows of odd lengths.
 *   W_gate_c, W_up_c   [sum(count)][d_model]: the kept rows, expert after expert
 *   W_down_c    expert e's block starts at element d_model * (ld(0) + ... + ld(e-1)) and is
 *               [d_model][ld(e)] row-major, zero beyond column count[e]
 *               (the three outputs of camera_gather_micro_experts, unchanged; with shared experts:
 *               the outputs of the call for the shared group written behind those of the routed group)
 *   n_experts + n_shared <= CAMERA_MAX_EXPERTS.
 */
int camera_layer_forward_compact(camera_ctx* ctx, void* stream,
                                 const void* X, int dtype, int64_t n, int64_t d_model, int64_t ldx,
                                 const int32_t* topk_idx, const float* topk_w, int top_k,
                                 int n_experts, int n_shared, const int32_t* count, int down_row_align,
                                 const void* W_gate_c, const void* W_up_c, const void* W_down_c,
                                 int flags, float* Y);
int camera_output_error(camera_ctx* ctx, void* stream, const float* Y, const float* Y_hat,
                        int64_t n, int64_t d_model, float* per_token);

/*
 * Per-kernel-group timing for benchmarks.  With profiling on, every launch
 * group is bracketed by HIP events on the caller's stream.
 * camera_profile_read waits for the recorded events, returns the summed
 * milliseconds and the number of launch groups since the last reset, and
 * resets that group's record.
 */
int camera_profile_enable(camera_ctx* ctx, int on);
int camera_profile_read(camera_ctx* ctx, int kernel_id, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* CAMERA_H_ */

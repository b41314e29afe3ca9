// Internal declarations shared by the translation units of libcamera_hip.
// Host-side launchers; each enqueues on `stream` and returns hipGetLastError().
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/camera.h"

namespace camera {

// ---- device-side helpers used by several kernels ---------------------------
constexpr int kWave = 64;

// Tables that describe how the routed (token, expert) pairs are laid out after
// bucketing.  All live in the context workspace.
struct BucketTables {
  int32_t* counts;        // [n_experts]        pairs per expert
  int32_t* offsets;       // [n_experts + 1]    first slot of each expert
  int32_t* tile_offset;   // [n_experts + 1]    first M-tile of each expert
  int32_t* tile_expert;   // [max_tiles]        expert of each M-tile slot
  int32_t* perm;          // [P]                token id of each slot (NULL: identity per expert)
  float* w_perm;          // [P]                routing weight of each slot (NULL: 1)
  int32_t* slot_of;       // [P]                slot of each (token, k) pair, -1 if its expert id is invalid (optional)
  int32_t* block_hist;    // [n_blocks x n_experts] scratch of the counting sort
  const void* zeros;      // 256 zero bytes (source of K-tail chunks for direct-to-LDS loads)
};

// ---- route.hip --------------------------------------------------------------
hipError_t launch_route_topk(hipStream_t stream, const void* X, int dtype, int64_t n, int64_t d_model,
                             int64_t ldx, const void* W_r, int64_t ldr, const float* bias, int n_experts,
                             int top_k, int renorm, const void* zeros /* 16 readable zero bytes */, int32_t* topk_idx,
                             float* topk_w);

// ---- bucket.hip -------------------------------------------------------------
// Pairs per block of the counting sort.
constexpr int kBucketChunk = 1024;
inline int64_t bucket_blocks(int64_t n_pairs) { return (n_pairs + kBucketChunk - 1) / kBucketChunk; }

// Stable counting sort of the n*top_k pairs by expert, then the M-tile tables
// for tiles of `tile_m` rows.
// (topk_w may be NULL: w_perm is then left unwritten.)
hipError_t launch_bucket(hipStream_t stream, const int32_t* topk_idx, const float* topk_w, int64_t n, int top_k,
                         int n_experts, int tile_m, int max_tiles, const BucketTables& t);
// Tables for the dense case: every expert sees tokens 0..n-1 with weight 1.
hipError_t launch_dense_tables(hipStream_t stream, int64_t n, int n_experts, int tile_m, int max_tiles,
                               const BucketTables& t);

// ---- gemm.hip ---------------------------------------------------------------
// M-tile height used by the grouped contraction for `dtype`.
int gemm_tile_m(int dtype, int64_t d_ff);
// What the contraction does with its two products G = X_e W_gate^T and U = X_e W_up^T:
//   kStats   Lambda = a silu(G) U is reduced to per-M-tile column statistics part_phi2 / part_max [max_tiles x d_ff]
//   kHidden  Lambda, zeroed where keep[e*d_ff + c] == 0 (keep may be NULL), is stored in hidden[bucket slot][d_ff],
//            rounded to bf16 by the bf16 kernel, as float32 by the float32 kernel
//   kProduct G goes to product[slot][c], U to product[slot][c + col_gap], row stride ld_product; in this mode X is
//            indexed by bucket slot, not by token (the hidden activations are the left operand)
struct GemmEpilogue {
  enum Mode { kStats = 0, kHidden = 1, kProduct = 2 };
  int mode = kStats;
  float* part_phi2 = nullptr;
  float* part_max = nullptr;
  void* hidden = nullptr;
  const uint8_t* keep = nullptr;
  float* product = nullptr;
  int64_t ld_product = 0;
  int col_gap = 0;
};
hipError_t launch_grouped_gemm(hipStream_t stream, int dtype, const void* X, int64_t ldx, int64_t d_model,
                               int64_t d_ff, int n_experts, const void* W_gate, const void* W_up,
                               int64_t stride_gu, int max_tiles, const BucketTables& t, const GemmEpilogue& ep);

// ---- norm.hip ---------------------------------------------------------------
// Row splits used for a [d_model x d_ff] matrix; omega_part is [splits x n_experts*d_ff].
int down_norm_splits(int n_experts, int64_t d_model, int64_t d_ff);
hipError_t launch_down_norm(hipStream_t stream, int dtype, const void* W_down, int64_t stride_down,
                            int n_experts, int64_t d_model, int64_t d_ff, int splits, float* omega_part);

// Input-channel energies h[e][c] = sum over the tokens in expert e's bucket of X[token][c]^2; part is
// [splits x n_experts*d_model] scratch, added in split order.
int input_energy_splits(int n_experts, int64_t d_model, int dtype);
hipError_t launch_input_energy(hipStream_t stream, int dtype, const void* X, int64_t ldx, int n_experts,
                               int64_t d_model, const BucketTables& t, int splits, float* part, float* h);

// Reduce the per-tile statistics in tile order, merge with earlier chunks,
// reduce omega partials in split order and form the energy.
hipError_t launch_finalize(hipStream_t stream, int n_experts, int64_t d_ff, const BucketTables& t,
                           const float* part_phi2, const float* part_max, const float* omega_part, int splits,
                           float alpha, int accumulate, int finalize, float* phi2, float* phi_inf,
                           float* omega2, float* energy);

// ---- rank.hip ---------------------------------------------------------------
struct RankCuts {
  int n_cuts;                          // <= CAMERA_MAX_LEVELS - 1
  int64_t cut_rank[CAMERA_MAX_LEVELS]; // element is "below cut q" iff its ascending rank < cut_rank[q]
  uint8_t out_of_below[CAMERA_MAX_LEVELS + 1];   // first output byte for "below k cuts"
  uint8_t out2_of_below[CAMERA_MAX_LEVELS + 1];  // second output byte for "below k cuts" (optional output)
};
struct SegTable {
  int n_seg;
  int32_t off[CAMERA_MAX_SEGMENTS + 1];
};
// What the per-segment kernel derives from the class bytes (class = number of cuts an element is below; an
// element below k cuts is below the k cuts of highest rank, so the class fixes which cuts those are).
struct SegOutputs {
  int n_classes;                 // n_cuts + 1, <= CAMERA_MAX_LEVELS
  int n_ratios;                  // pruning ratios (0: no kept counts)
  int n_levels;                  // precision levels (0: no level counts)
  uint32_t prune_cuts_of_class;  // 4 bits per class: how many of the pruning cuts its members are below
  uint32_t level_of_class;       // 4 bits per class: precision level of its members
  int32_t* kept;                 // [n_ratios][n_seg]: kept at ratio k = members of the classes below <= n_ratios-1-k pruning cuts
  int32_t* level_count;          // [n_seg][n_levels]
  int32_t* perm;                 // optional: inside every segment level 0 first, then level 1, ..., ascending index inside a level
};
// Bytes of the persistent select state (zero when made, self-cleaning afterwards) and the int32 words of
// per-call workspace the rank kernels need for n_micro keys.
size_t rank_state_bytes();
int64_t rank_workspace_words(int64_t n_micro, int want_rank);
// class_out[i] = number of cuts element i is below; byte_out[i] = out_of_below[class_out[i]], byte_out2
// (optional) likewise from out2_of_below.  kept_idx (optional): ascending indices of the elements below no cut.
hipError_t launch_classify(hipStream_t stream, const float* energy, int64_t n_micro, const RankCuts& cuts,
                           uint8_t* class_out, uint8_t* byte_out, uint8_t* byte_out2, int32_t* kept_idx, void* state,
                           int32_t* ws);
hipError_t launch_segment_outputs(hipStream_t stream, const uint8_t* class_out, const SegTable& seg,
                                  const SegOutputs& out);
// Full stable ascending rank by LSD radix sort.
hipError_t launch_full_rank(hipStream_t stream, const float* energy, int64_t n_micro, uint32_t* rank,
                            int32_t* ws);

// ---- forward.hip -----------------------------------------------------------
// Y[token] (+)= sum of the product rows of the token's slots (routed: slot_of[token*top_k + k], k ascending;
// slot_of == nullptr: rows e*n + token for e ascending).  product is [pairs][d_model] float32, Y [n][d_model].
hipError_t launch_combine(hipStream_t stream, const float* product, const int32_t* slot_of, int64_t n, int top_k,
                          int n_experts, int64_t d_model, int accumulate, float* Y);
// per_token [n][4] = ||y - y_hat||^2, ||y||^2, ||y_hat||^2, <y, y_hat>
hipError_t launch_output_error(hipStream_t stream, const float* Y, const float* Y_hat, int64_t n, int64_t d_model,
                               int64_t ldy, int64_t ldh, float* per_token);

// ---- compact.hip ------------------------------------------------------------
// Where each expert's kept micro-experts sit in the compacted matrices, passed to the kernels by value.
struct CompactRows {                          // W_gate_c / W_up_c
  int n_experts;
  int32_t row_off[CAMERA_MAX_EXPERTS + 1];    // first compact row of each expert (prefix of the kept counts)
  int32_t tile_off[CAMERA_MAX_EXPERTS + 1];   // first 32-row tile of each expert
};
struct CompactDown {                          // W_down_c
  int n_experts;
  int k_round;                                // MFMA path: the K extent of an expert is its count rounded up to this
                                              // (8, or 64 when the row alignment is a multiple of 64: no K tail)
  int32_t count[CAMERA_MAX_EXPERTS];          // kept micro-experts of each expert
  int32_t ld_off[CAMERA_MAX_EXPERTS + 1];     // prefix of the row lengths (count rounded up to the row alignment):
                                              // expert e's block starts at element d_model * ld_off[e]
  int32_t chunk_off[CAMERA_MAX_EXPERTS + 1];  // first K chunk of each expert
};
// K chunks of an expert with `count` kept micro-experts in the second contraction: chunks of at most
// kCompactChunk elements, at most kCompactMaxChunks of them (0 for an expert that keeps nothing).
constexpr int kCompactChunk = 3072;
constexpr int kCompactMaxChunks = 8;
inline int compact_chunks(int count) {
  const int c = (count + kCompactChunk - 1) / kCompactChunk;
  return c > kCompactMaxChunks ? kCompactMaxChunks : c;
}
// Bucket tables (counts, offsets, perm, w_perm, slot_of) of the pairs (token, routed choice k < top_k) and
// (token, appended expert n_experts + s, weight 1), in one launch; n * (top_k + n_shared) <= kCompactSmallPairs.
constexpr int kCompactSmallPairs = 2048;
hipError_t launch_compact_bucket_small(hipStream_t stream, const int32_t* topk_idx, const float* topk_w, int64_t n,
                                       int top_k, int n_experts, int n_shared, const BucketTables& t);
// idx_aug / w_aug [n][top_k + n_shared]: the routed choices followed by the appended experts with weight 1.
hipError_t launch_compact_append_shared(hipStream_t stream, const int32_t* topk_idx, const float* topk_w, int64_t n,
                                        int top_k, int n_experts, int n_shared, int32_t* idx_aug, float* w_aug);
// token_groups: grid rows of 32 tokens per expert; the last one also takes what lies beyond.
// hidden [slots][ldh] bf16 <- a silu(x w_gate) (x w_up) on the kept rows; columns [count, round8(count)) zero.
hipError_t launch_compact_hidden(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model, const void* W_gate,
                                 const void* W_up, const CompactRows& tab, const BucketTables& t, int token_groups,
                                 void* hidden, int ldh);
// partial [chunk within its expert][n_slots][d_model] float32 <- hidden times the chunk of the expert's W_down block.
hipError_t launch_compact_down(hipStream_t stream, const void* hidden, int ldh, const void* W_down, int64_t d_model,
                               const CompactDown& tab, const BucketTables& t, int token_groups, int64_t n_slots,
                               float* partial);
// Y[token] (+)= the partial rows of the token's slots (experts in k order, chunks in chunk order).
hipError_t launch_compact_combine(hipStream_t stream, const float* partial, const CompactDown& tab,
                                  const BucketTables& t, int64_t n, int terms, int64_t d_model, int64_t n_slots,
                                  int accumulate, float* Y);

// The two contractions of the compacted layer in the grouped MFMA kernel (gemm.hip), for batches large enough
// to fill its 256-row tiles.  d_model must be a multiple of 16 and the rows of the W_down blocks a multiple of 8
// elements long (16-byte tile loads).  k_round (8, or 64 when every row length is a multiple of 64): the K extent of
// an expert in the second contraction is its kept count rounded up to it.  The hidden buffer holds expert e's rows
// back to back, that many elements each: at most pairs * round_up(widest count, k_round) elements.
// scratch: kCompactGemmScratchWords int32 words, 8-byte aligned, shared by the two launches of a call.
constexpr int kCompactGemmScratchWords = (CAMERA_MAX_EXPERTS + 1 + 16) + 2 * CAMERA_MAX_EXPERTS;
hipError_t launch_compact_hidden_gemm(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model,
                                      const void* W_gate, const void* W_up, const CompactRows& tab, int widest,
                                      int max_tiles, const BucketTables& t, int32_t* scratch, void* hidden,
                                      int k_round);
hipError_t launch_compact_down_gemm(hipStream_t stream, const void* hidden, int64_t d_model, const void* W_down,
                                    const CompactDown& tab, int max_tiles, const BucketTables& t, int32_t* scratch,
                                    float* product);

// Gather of kept micro-experts (gather.hip).  off: [n_experts + 1] exclusive prefix of the per-expert
// entry counts (count == nullptr: d_ff each), off_ld: the same of the counts rounded up to a multiple of
// row_align (row lengths of the W_down blocks); both written by launch_gather_offsets.
hipError_t launch_gather_offsets(hipStream_t stream, const int32_t* count, int n_experts, int64_t d_ff, int row_align,
                                 int32_t* off, int32_t* off_ld);
hipError_t launch_gather_rows(hipStream_t stream, int dtype, const void* W_gate, const void* W_up, int64_t stride_gu,
                              int n_experts, int64_t d_ff, int64_t d_model, const int32_t* index, int64_t n_index,
                              int64_t index_base, const int32_t* off, void* gate_out, void* up_out);
hipError_t launch_gather_cols(hipStream_t stream, int dtype, const void* W_down, int64_t stride_down, int n_experts,
                              int64_t d_ff, int64_t d_model, const int32_t* index, int64_t n_index,
                              int64_t index_base, const int32_t* off, const int32_t* off_ld, void* down_out);

}  // namespace camera

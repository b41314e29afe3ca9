// Token -> expert bucketing: a stable counting sort of the n*top_k routed
// (token, expert) pairs by expert.  This is the explicit form of the masking
// by A[:, i] in Algorithm 1, line 6: expert i only ever sees the tokens whose
// routing weight to it is non-zero.
//
// Three launches, all integer work:
//   count   : every block histograms its 1024 consecutive pairs (LDS atomics)
//   scan    : one block turns the per-block histograms into exclusive bases,
//             and builds counts / offsets / the M-tile tables of the GEMM
//   scatter : every wave walks its 256 consecutive pairs 64 at a time; the
//             position of a pair inside its expert is found with wavefront
//             ballots (one per bit of the expert id gives the lanes of equal
//             expert) and popcounts of the lower lanes, so equal experts keep
//             their pair order (stable, deterministic).
#include "camera_internal.h"

namespace camera {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kPairsPerWave = kBucketChunk / kWavesPerBlock;  // 256
static_assert(kPairsPerWave % kWave == 0, "wave chunk must be whole wavefronts");

__global__ __launch_bounds__(kThreads) void bucket_count_kernel(const int32_t* __restrict__ topk_idx,
                                                                int64_t n_pairs, int n_experts,
                                                                int32_t* __restrict__ block_hist) {
  __shared__ int32_t hist[CAMERA_MAX_EXPERTS];
  for (int e = threadIdx.x; e < n_experts; e += kThreads) hist[e] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kBucketChunk;
  for (int i = threadIdx.x; i < kBucketChunk; i += kThreads) {
    const int64_t p = base + i;
    if (p < n_pairs) {
      const int e = topk_idx[p];
      if (e >= 0 && e < n_experts) atomicAdd(&hist[e], 1);
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < n_experts; e += kThreads)
    block_hist[(int64_t)blockIdx.x * n_experts + e] = hist[e];
}

// One block.  Thread e owns expert e.
__global__ __launch_bounds__(CAMERA_MAX_EXPERTS) void bucket_scan_kernel(int32_t* __restrict__ block_hist,
                                                                        int n_blocks, int n_experts, int tile_m,
                                                                        int max_tiles, int32_t* __restrict__ counts,
                                                                        int32_t* __restrict__ offsets,
                                                                        int32_t* __restrict__ tile_offset,
                                                                        int32_t* __restrict__ tile_expert) {
  __shared__ int32_t s_cnt[CAMERA_MAX_EXPERTS];
  __shared__ int32_t s_off[CAMERA_MAX_EXPERTS + 1];
  __shared__ int32_t s_toff[CAMERA_MAX_EXPERTS + 1];
  const int e = threadIdx.x;
  int32_t total = 0;
  if (e < n_experts) {
    // exclusive prefix over blocks, in place; eight independent loads at a time, because a lone
    // workgroup has nothing else to hide their latency with
    int b = 0;
    for (; b + 8 <= n_blocks; b += 8) {
      int32_t c[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) c[u] = block_hist[(int64_t)(b + u) * n_experts + e];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        block_hist[(int64_t)(b + u) * n_experts + e] = total;
        total += c[u];
      }
    }
    for (; b < n_blocks; ++b) {
      const int32_t c = block_hist[(int64_t)b * n_experts + e];
      block_hist[(int64_t)b * n_experts + e] = total;
      total += c;
    }
    s_cnt[e] = total;
  }
  __syncthreads();
  if (e == 0) {  // n_experts <= 256: a serial scan is a few hundred cycles
    int32_t off = 0, toff = 0;
    for (int i = 0; i < n_experts; ++i) {
      s_off[i] = off;
      s_toff[i] = toff;
      off += s_cnt[i];
      toff += (s_cnt[i] + tile_m - 1) / tile_m;
    }
    s_off[n_experts] = off;
    s_toff[n_experts] = toff;
  }
  __syncthreads();
  if (e < n_experts) {
    counts[e] = s_cnt[e];
    offsets[e] = s_off[e];
    tile_offset[e] = s_toff[e];
    for (int t = s_toff[e]; t < s_toff[e + 1] && t < max_tiles; ++t) tile_expert[t] = e;
  }
  if (e == 0) {
    offsets[n_experts] = s_off[n_experts];
    tile_offset[n_experts] = s_toff[n_experts] < max_tiles ? s_toff[n_experts] : max_tiles;
  }
}

__global__ __launch_bounds__(kThreads) void bucket_scatter_kernel(const int32_t* __restrict__ topk_idx,
                                                                  const float* __restrict__ topk_w,
                                                                  int64_t n_pairs, int top_k, int n_experts,
                                                                  const int32_t* __restrict__ block_base,
                                                                  const int32_t* __restrict__ offsets,
                                                                  int32_t* __restrict__ perm,
                                                                  float* __restrict__ w_perm,
                                                                  int32_t* __restrict__ slot_of) {
  // next[w][e]: next free slot of expert e for wave w of this block
  __shared__ int32_t next[kWavesPerBlock][CAMERA_MAX_EXPERTS];
  const int wave = threadIdx.x / kWave;
  const int lane = threadIdx.x % kWave;
  const int64_t block_first = (int64_t)blockIdx.x * kBucketChunk;
  const int64_t wave_first = block_first + (int64_t)wave * kPairsPerWave;

  for (int i = threadIdx.x; i < kWavesPerBlock * CAMERA_MAX_EXPERTS; i += kThreads) (&next[0][0])[i] = 0;
  __syncthreads();
  // per-wave histogram of its own 256 pairs
  for (int it = 0; it < kPairsPerWave / kWave; ++it) {
    const int64_t p = wave_first + it * kWave + lane;
    if (p < n_pairs) {
      const int e = topk_idx[p];
      if (e >= 0 && e < n_experts) atomicAdd(&next[wave][e], 1);
    }
  }
  __syncthreads();
  // turn the histograms into first slots: expert base + block base + earlier waves
  for (int e = threadIdx.x; e < n_experts; e += kThreads) {
    int32_t run = offsets[e] + block_base[(int64_t)blockIdx.x * n_experts + e];
    for (int w = 0; w < kWavesPerBlock; ++w) {
      const int32_t c = next[w][e];
      next[w][e] = run;
      run += c;
    }
  }
  __syncthreads();

  const uint64_t lower_lanes = (1ull << lane) - 1ull;
  for (int it = 0; it < kPairsPerWave / kWave; ++it) {
    const int64_t p = wave_first + it * kWave + lane;
    int e = -1;
    if (p < n_pairs) {
      e = topk_idx[p];
      if (e < 0 || e >= n_experts) e = -1;
    }
    // The lanes that hold the same expert, from one ballot per bit of the id (eight bits: ids are below 256):
    // a lane keeps the lanes that agree with it on every bit.  Its slot is the expert's next free one plus the
    // number of such lanes below it; the lowest lane of every group then moves the expert's counter on.
    uint64_t same = __ballot(e >= 0);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
      const uint64_t ones = __ballot((e >> bit) & 1);
      same &= ((e >> bit) & 1) ? ones : ~ones;
    }
    int slot = -1;
    if (e >= 0) slot = next[wave][e] + __popcll(same & lower_lanes);
    // every lane has read next[] before the first lane of its group moves it on
    __builtin_amdgcn_wave_barrier();
    if (e >= 0 && (same & lower_lanes) == 0) next[wave][e] += __popcll(same);
    __builtin_amdgcn_wave_barrier();
    if (e >= 0) {
      perm[slot] = (int32_t)(p / top_k);
      if (topk_w) w_perm[slot] = topk_w[p];
    }
    if (slot_of != nullptr && p < n_pairs) slot_of[p] = e >= 0 ? slot : -1;
  }
}

__global__ void dense_tables_kernel(int64_t n, int n_experts, int tile_m, int max_tiles,
                                    int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                    int32_t* __restrict__ tile_offset, int32_t* __restrict__ tile_expert) {
  const int tiles_per = (int)((n + tile_m - 1) / tile_m);
  for (int e = threadIdx.x; e <= n_experts; e += blockDim.x) {
    if (e < n_experts) counts[e] = (int32_t)n;
    offsets[e] = (int32_t)(e * n);
    tile_offset[e] = e * tiles_per;
  }
  for (int t = threadIdx.x; t < n_experts * tiles_per && t < max_tiles; t += blockDim.x)
    tile_expert[t] = t / tiles_per;
}

}  // namespace

hipError_t launch_bucket(hipStream_t stream, const int32_t* topk_idx, const float* topk_w, int64_t n, int top_k,
                         int n_experts, int tile_m, int max_tiles, const BucketTables& t) {
  const int64_t n_pairs = n * top_k;
  const int n_blocks = (int)bucket_blocks(n_pairs);
  if (n_blocks > 0)
    hipLaunchKernelGGL(bucket_count_kernel, dim3(n_blocks), dim3(kThreads), 0, stream, topk_idx, n_pairs, n_experts,
                       t.block_hist);
  hipLaunchKernelGGL(bucket_scan_kernel, dim3(1), dim3(CAMERA_MAX_EXPERTS), 0, stream, t.block_hist, n_blocks,
                     n_experts, tile_m, max_tiles, t.counts, t.offsets, t.tile_offset, t.tile_expert);
  if (n_blocks > 0)
    hipLaunchKernelGGL(bucket_scatter_kernel, dim3(n_blocks), dim3(kThreads), 0, stream, topk_idx, topk_w, n_pairs,
                       top_k, n_experts, t.block_hist, t.offsets, t.perm, t.w_perm, t.slot_of);
  return hipGetLastError();
}

hipError_t launch_dense_tables(hipStream_t stream, int64_t n, int n_experts, int tile_m, int max_tiles,
                               const BucketTables& t) {
  hipLaunchKernelGGL(dense_tables_kernel, dim3(1), dim3(256), 0, stream, n, n_experts, tile_m, max_tiles, t.counts,
                     t.offsets, t.tile_offset, t.tile_expert);
  return hipGetLastError();
}

}  // namespace camera

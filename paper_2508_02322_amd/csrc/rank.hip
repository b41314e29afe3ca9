// Ranking decisions on a layer's energies (Algorithm 1 line 11, Algorithm 2
// line 9, Algorithm 3 lines 5-8).  All integer work on float32 bit patterns.
//
// The order is the stable ascending order of (energy, index).  A cut at rank t
// separates the t lowest-ranked micro-experts from the rest; CAMERA-P needs one
// cut (t = n_prune), CAMERA-Q one per class boundary.  No sort is needed for
// that: a radix select (11 + 11 + 10 bits) finds, for every cut, the key K of the
// element of rank t and how many elements equal to K lie below the cut (r);
// element i is below the cut iff key_i < K, or key_i == K and fewer than r equal
// keys precede it.  The "equal keys that precede" count comes from an ordered
// walk: every wave owns a contiguous index range, ballots + popcounts give the
// order inside 256-element steps.
//
// classify_kernel: one workgroup of 16 waves does the select passes and the
// walk for all cuts at once (<= 184 320 keys per layer in the paper's models:
// the pass is latency-bound, not bandwidth-bound).
// segment_kernel: one workgroup per expert: class sizes and the stable
// partition of its micro-experts by class.
// full rank: LSD radix sort (4 x 8 bits) of (key, index) built from a stable
// counting sort whose in-wave order again comes from ballots.
#include "camera_internal.h"

namespace camera {
namespace {

constexpr int kMaxCuts = CAMERA_MAX_LEVELS - 1;

__device__ __forceinline__ uint32_t key_of(float v) {
  uint32_t u = __float_as_uint(v);
  if (u == 0x80000000u) u = 0u;  // -0.0 ranks as +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// 4 consecutive keys starting at i (i is a multiple of 4); keys past n are 0xffffffff with valid = false
struct Keys4 {
  uint32_t k[4];
  bool valid[4];
};
__device__ __forceinline__ Keys4 load_keys4(const float* __restrict__ E, int64_t i, int64_t n) {
  Keys4 out;
  if (i + 3 < n) {
    const float4 v = *reinterpret_cast<const float4*>(E + i);
    out.k[0] = key_of(v.x);
    out.k[1] = key_of(v.y);
    out.k[2] = key_of(v.z);
    out.k[3] = key_of(v.w);
    out.valid[0] = out.valid[1] = out.valid[2] = out.valid[3] = true;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      out.valid[j] = i + j < n;
      out.k[j] = out.valid[j] ? key_of(E[i + j]) : 0xffffffffu;
    }
  }
  return out;
}

// ---------------------------------------------------------------------------
// classify
// ---------------------------------------------------------------------------
constexpr int kClsThreads = 1024;
constexpr int kClsWaves = kClsThreads / kWave;
constexpr int kBins = 2048;
constexpr int kReplicas = kMaxCuts;  // pass 0 spreads one histogram over the per-cut slots
constexpr int kInFlight = 4;         // independent 16-byte loads a thread keeps in flight

__device__ __forceinline__ Keys4 keys_of(float4 v) {
  Keys4 k;
  k.k[0] = key_of(v.x);
  k.k[1] = key_of(v.y);
  k.k[2] = key_of(v.z);
  k.k[3] = key_of(v.w);
  k.valid[0] = k.valid[1] = k.valid[2] = k.valid[3] = true;
  return k;
}

// Every thread of the block visits groups of 4 keys, block-strided; the order does not matter.
// One workgroup cannot hide memory latency with occupancy, so kInFlight loads are issued before
// the first is used.
template <class F>
__device__ __forceinline__ void sweep_block(const float* __restrict__ E, int64_t n, F&& f) {
  constexpr int64_t step = (int64_t)kClsThreads * 4;
  int64_t i = (int64_t)threadIdx.x * 4;
  for (; i + (kInFlight - 1) * step + 3 < n; i += kInFlight * step) {
    float4 v[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) v[u] = *reinterpret_cast<const float4*>(E + i + u * step);
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) f(keys_of(v[u]));
  }
  for (; i < n; i += step) f(load_keys4(E, i, n));
}

// A wave visits its contiguous index range [begin, end) in order, 256 indices per step (lane l
// holds 4 l .. 4 l + 3 of the step); f(keys, first index of the lane) runs on whole waves, so it
// may ballot.  Loads of kInFlight steps are issued together.
template <class F>
__device__ __forceinline__ void walk_wave(const float* __restrict__ E, int64_t begin, int64_t end, int lane, F&& f) {
  int64_t i0 = begin;
  for (; i0 + kInFlight * 256 <= end; i0 += kInFlight * 256) {
    float4 v[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) v[u] = *reinterpret_cast<const float4*>(E + i0 + u * 256 + lane * 4);
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) f(keys_of(v[u]), i0 + u * 256 + lane * 4);
  }
  for (; i0 < end; i0 += 256) f(load_keys4(E, i0 + lane * 4, end), i0 + lane * 4);
}

// exclusive prefix of v over the block (thread order); s_wave is [kClsWaves + 1] scratch
__device__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* s_wave) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  uint32_t inc = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const uint32_t o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == kWave - 1) s_wave[wave] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += s_wave[w];
  __syncthreads();
  return base + inc - v;
}

__global__ __launch_bounds__(kClsThreads) void classify_kernel(const float* __restrict__ E, int64_t n,
                                                               RankCuts cuts, uint8_t* __restrict__ class_out,
                                                               uint8_t* __restrict__ byte_out,
                                                               int32_t* __restrict__ kept_idx) {
  __shared__ uint32_t hist[kMaxCuts][kBins];
  __shared__ uint32_t s_wave[kClsWaves + 1];
  __shared__ uint32_t s_prefix[kMaxCuts];  // key bits fixed so far (right-aligned)
  __shared__ uint32_t s_rem[kMaxCuts];     // rank of the cut among the keys that share the prefix
  __shared__ int s_mode[kMaxCuts];         // 0 select, 1 nothing below, 2 everything below
  __shared__ uint32_t s_tie[kMaxCuts][kClsWaves];
  __shared__ uint32_t s_kept[kClsWaves];

  const int tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  const int n_cuts = cuts.n_cuts;
  if (tid < kMaxCuts) {
    int mode = 1;
    uint32_t rem = 0;
    if (tid < n_cuts) {
      const int64_t t = cuts.cut_rank[tid];
      mode = t <= 0 ? 1 : (t >= n ? 2 : 0);
      rem = mode == 0 ? (uint32_t)t : 0u;
    }
    s_mode[tid] = mode;
    s_rem[tid] = rem;
    s_prefix[tid] = 0u;
  }
  __syncthreads();
  bool any_select = false;
  for (int q = 0; q < n_cuts; ++q) any_select |= s_mode[q] == 0;

  if (any_select) {
    const int shift_of[3] = {21, 10, 0};
    const int bits_of[3] = {11, 11, 10};
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = shift_of[pass];
      const uint32_t mask = (1u << bits_of[pass]) - 1u;
      for (int i = tid; i < kMaxCuts * kBins; i += kClsThreads) (&hist[0][0])[i] = 0u;
      __syncthreads();
      if (pass == 0) {
        // no prefix yet: one histogram serves every cut; lanes spread over replicas to
        // thin out same-address LDS atomics (energies share their top bits)
        uint32_t* my_hist = hist[lane % kReplicas];
        sweep_block(E, n, [&](const Keys4& k) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (k.valid[j]) atomicAdd(&my_hist[k.k[j] >> shift], 1u);
        });
        __syncthreads();
        for (int b = tid; b < kBins; b += kClsThreads) {
          uint32_t sum = 0;
#pragma unroll
          for (int r = 0; r < kReplicas; ++r) sum += hist[r][b];
          for (int r = 0; r < kReplicas; ++r) hist[r][b] = sum;  // bin b is touched by this thread only
        }
        __syncthreads();
      } else {
        const int prev_shift = shift + bits_of[pass];
        uint32_t want[kMaxCuts];
#pragma unroll
        for (int q = 0; q < kMaxCuts; ++q) want[q] = (q < n_cuts && s_mode[q] == 0) ? s_prefix[q] : 0xffffffffu;
        sweep_block(E, n, [&](const Keys4& k) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (!k.valid[j]) continue;
            const uint32_t top = k.k[j] >> prev_shift;  // at most 22 bits: never 0xffffffff
#pragma unroll
            for (int q = 0; q < kMaxCuts; ++q)
              if (top == want[q]) atomicAdd(&hist[q][(k.k[j] >> shift) & mask], 1u);
          }
        });
        __syncthreads();
      }
      // locate, for every cut, the bin that holds rank s_rem[q]
      for (int q = 0; q < n_cuts; ++q) {
        if (s_mode[q] != 0) continue;  // block-uniform
        const uint32_t h0 = hist[q][2 * tid], h1 = hist[q][2 * tid + 1];
        const uint32_t before = block_exclusive_scan(h0 + h1, s_wave);
        const uint32_t rem = s_rem[q];
        __syncthreads();
        if (rem >= before && rem < before + h0) {
          s_prefix[q] = (s_prefix[q] << bits_of[pass]) | (uint32_t)(2 * tid);
          s_rem[q] = rem - before;
        } else if (rem >= before + h0 && rem < before + h0 + h1) {
          s_prefix[q] = (s_prefix[q] << bits_of[pass]) | (uint32_t)(2 * tid + 1);
          s_rem[q] = rem - before - h0;
        }
        __syncthreads();
      }
    }
  }
  // s_prefix[q] is now the full key K_q, s_rem[q] the number of keys equal to K_q below the cut.

  // Ordered walk.  Wave w owns indices [w*span, (w+1)*span).
  const int64_t span = ((n + kClsWaves * 256 - 1) / (kClsWaves * 256)) * 256;
  const int64_t w_begin = min(n, (int64_t)wave * span);
  const int64_t w_end = min(n, w_begin + span);
  const uint64_t lower = (1ull << lane) - 1ull;

  uint32_t K[kMaxCuts], R[kMaxCuts];
  int mode[kMaxCuts];
  bool ties_split = false;  // some cut runs through a group of equal keys: their index order matters
#pragma unroll
  for (int q = 0; q < kMaxCuts; ++q) {
    K[q] = s_prefix[q];
    R[q] = s_rem[q];
    mode[q] = q < n_cuts ? s_mode[q] : 1;
    ties_split |= mode[q] == 0 && R[q] > 0;
  }

  if (ties_split) {  // equal-key counts per wave, then their exclusive prefix over the waves
    uint32_t cnt[kMaxCuts];
#pragma unroll
    for (int q = 0; q < kMaxCuts; ++q) cnt[q] = 0;
    walk_wave(E, w_begin, w_end, lane, [&](const Keys4& k, int64_t) {
#pragma unroll
      for (int q = 0; q < kMaxCuts; ++q) {
        if (mode[q] != 0 || R[q] == 0) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) cnt[q] += __popcll(__ballot(k.valid[j] && k.k[j] == K[q]));
      }
    });
    if (lane == 0) {
#pragma unroll
      for (int q = 0; q < kMaxCuts; ++q) s_tie[q][wave] = cnt[q];
    }
    __syncthreads();
    if (tid < kMaxCuts) {
      uint32_t run = 0;
      for (int w = 0; w < kClsWaves; ++w) {
        const uint32_t c = s_tie[tid][w];
        s_tie[tid][w] = run;
        run += c;
      }
    }
    __syncthreads();
  }

  uint32_t tie_base[kMaxCuts];
#pragma unroll
  for (int q = 0; q < kMaxCuts; ++q) tie_base[q] = ties_split ? s_tie[q][wave] : 0u;
  uint32_t kept = 0;
  walk_wave(E, w_begin, w_end, lane, [&](const Keys4& k, int64_t i) {
    int below[4] = {0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < kMaxCuts; ++q) {
      if (mode[q] == 1) continue;
      if (mode[q] == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) below[j] += 1;
        continue;
      }
      if (R[q] == 0) {  // no key equal to K is below this cut
#pragma unroll
        for (int j = 0; j < 4; ++j) below[j] += k.k[j] < K[q] ? 1 : 0;
        continue;
      }
      bool eq[4];
      uint32_t lanes_before = 0, total = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        eq[j] = k.valid[j] && k.k[j] == K[q];
        const uint64_t b = __ballot(eq[j]);
        lanes_before += __popcll(b & lower);
        total += __popcll(b);
      }
      uint32_t tie_rank = tie_base[q] + lanes_before;  // equal keys at lower indices
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (k.k[j] < K[q] || (eq[j] && tie_rank < R[q])) below[j] += 1;
        tie_rank += eq[j] ? 1u : 0u;
      }
      tie_base[q] += total;
    }
    if (k.valid[3]) {  // whole group inside: one 4-byte store per output
      const uint32_t cls4 = (uint32_t)below[0] | ((uint32_t)below[1] << 8) | ((uint32_t)below[2] << 16) |
                            ((uint32_t)below[3] << 24);
      const uint32_t out4 = (uint32_t)cuts.out_of_below[below[0]] | ((uint32_t)cuts.out_of_below[below[1]] << 8) |
                            ((uint32_t)cuts.out_of_below[below[2]] << 16) |
                            ((uint32_t)cuts.out_of_below[below[3]] << 24);
      *reinterpret_cast<uint32_t*>(class_out + i) = cls4;
      *reinterpret_cast<uint32_t*>(byte_out + i) = out4;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (k.valid[j]) {
          class_out[i + j] = (uint8_t)below[j];
          byte_out[i + j] = cuts.out_of_below[below[j]];
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) kept += __popcll(__ballot(k.valid[j] && below[j] == 0));
  });
  if (kept_idx == nullptr) return;  // block-uniform

  if (lane == 0) s_kept[wave] = kept;
  __syncthreads();
  uint32_t pos = 0;
  for (int w = 0; w < wave; ++w) pos += s_kept[w];
  // ascending list of the kept indices: re-derive "kept" from the keys instead of re-reading class_out
  // (same arithmetic as above restricted to "below no cut")
  for (int64_t i0 = w_begin; i0 < w_end; i0 += 256) {
    const int64_t i = i0 + lane * 4;
    bool is_kept[4];
    uint32_t lanes_before = 0, total = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      is_kept[j] = i + j < w_end && class_out[i + j] == 0;  // written by this same lane above
      const uint64_t b = __ballot(is_kept[j]);
      lanes_before += __popcll(b & lower);
      total += __popcll(b);
    }
    uint32_t p = pos + lanes_before;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (is_kept[j]) kept_idx[p++] = (int32_t)(i + j);
    pos += total;
  }
}

// ---------------------------------------------------------------------------
// per-segment class sizes and stable partition
// ---------------------------------------------------------------------------
constexpr int kSegThreads = 256;
constexpr int kSegWaves = kSegThreads / kWave;

__global__ __launch_bounds__(kSegThreads) void segment_kernel(const uint8_t* __restrict__ class_in, SegTable seg,
                                                              int n_classes, int kept_only,
                                                              int32_t* __restrict__ counts,
                                                              int32_t* __restrict__ perm) {
  __shared__ uint32_t s_cnt[kSegWaves][CAMERA_MAX_LEVELS];
  const int s = blockIdx.x;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int begin = seg.off[s], end = seg.off[s + 1];
  const int span = ((end - begin + kSegWaves * kWave - 1) / (kSegWaves * kWave)) * kWave;
  const int w_begin = min(end, begin + wave * span);
  const int w_end = min(end, w_begin + span);
  const uint64_t lower = (1ull << lane) - 1ull;

  uint32_t cnt[CAMERA_MAX_LEVELS];
#pragma unroll
  for (int m = 0; m < CAMERA_MAX_LEVELS; ++m) cnt[m] = 0;
  for (int i0 = w_begin; i0 < w_end; i0 += 4 * kWave) {  // four independent byte loads in flight
    int c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kWave + lane;
      c[u] = i < w_end ? (int)class_in[i] : -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int m = 0; m < CAMERA_MAX_LEVELS; ++m)
        if (m < n_classes) cnt[m] += __popcll(__ballot(c[u] == m));
  }
  if (lane == 0) {
#pragma unroll
    for (int m = 0; m < CAMERA_MAX_LEVELS; ++m) s_cnt[wave][m] = cnt[m];
  }
  __syncthreads();
  if (threadIdx.x < n_classes) {
    uint32_t total = 0;
    for (int w = 0; w < kSegWaves; ++w) total += s_cnt[w][threadIdx.x];
    if (kept_only) {
      if (threadIdx.x == 0) counts[s] = (int32_t)total;
    } else {
      counts[s * n_classes + threadIdx.x] = (int32_t)total;
    }
  }
  if (perm == nullptr) return;  // block-uniform

  // first slot of class m for this wave: segment start + all earlier classes + earlier waves
  uint32_t slot[CAMERA_MAX_LEVELS];
  uint32_t run = (uint32_t)begin;
#pragma unroll
  for (int m = 0; m < CAMERA_MAX_LEVELS; ++m) {
    slot[m] = 0;
    if (m < n_classes) {
      for (int w = 0; w < kSegWaves; ++w) {
        if (w == wave) slot[m] = run;
        run += s_cnt[w][m];
      }
    }
  }
  for (int i0 = w_begin; i0 < w_end; i0 += 4 * kWave) {
    int c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kWave + lane;
      c[u] = i < w_end ? (int)class_in[i] : -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kWave + lane;
#pragma unroll
      for (int m = 0; m < CAMERA_MAX_LEVELS; ++m) {
        if (m < n_classes) {
          const uint64_t b = __ballot(c[u] == m);
          if (c[u] == m) perm[slot[m] + __popcll(b & lower)] = i;
          slot[m] += __popcll(b);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// full rank: LSD radix sort of (key, index), 8 bits per pass
// ---------------------------------------------------------------------------
constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortChunk = 2048;                          // keys per block
constexpr int kSortPerWave = kSortChunk / kSortWaves;     // 512 consecutive keys per wave
constexpr int kDigits = 256;

__global__ __launch_bounds__(kSortThreads) void sort_init_kernel(const float* __restrict__ E, int64_t n,
                                                                 uint32_t* __restrict__ keys,
                                                                 uint32_t* __restrict__ idx) {
  const int64_t i = (int64_t)blockIdx.x * kSortThreads + threadIdx.x;
  if (i < n) {
    keys[i] = key_of(E[i]);
    idx[i] = (uint32_t)i;
  }
}

__global__ __launch_bounds__(kSortThreads) void sort_count_kernel(const uint32_t* __restrict__ keys, int64_t n,
                                                                  int shift, int32_t* __restrict__ block_hist) {
  __shared__ int32_t hist[kDigits];
  hist[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortChunk;
  for (int i = threadIdx.x; i < kSortChunk; i += kSortThreads)
    if (base + i < n) atomicAdd(&hist[(keys[base + i] >> shift) & 0xff], 1);
  __syncthreads();
  block_hist[(int64_t)blockIdx.x * kDigits + threadIdx.x] = hist[threadIdx.x];
}

// one block; thread d owns digit d: exclusive bases over (digit, block)
__global__ __launch_bounds__(kDigits) void sort_scan_kernel(int32_t* __restrict__ block_hist, int n_blocks) {
  __shared__ int32_t s_total[kDigits];
  __shared__ int32_t s_base[kDigits];
  const int d = threadIdx.x;
  int32_t total = 0;
  for (int b = 0; b < n_blocks; ++b) {
    const int32_t c = block_hist[(int64_t)b * kDigits + d];
    block_hist[(int64_t)b * kDigits + d] = total;
    total += c;
  }
  s_total[d] = total;
  __syncthreads();
  if (d == 0) {
    int32_t run = 0;
    for (int i = 0; i < kDigits; ++i) {
      s_base[i] = run;
      run += s_total[i];
    }
  }
  __syncthreads();
  const int32_t base = s_base[d];
  for (int b = 0; b < n_blocks; ++b) block_hist[(int64_t)b * kDigits + d] += base;
}

// stable scatter; in the last pass the destination position is written to rank[idx]
__global__ __launch_bounds__(kSortThreads) void sort_scatter_kernel(const uint32_t* __restrict__ keys_in,
                                                                    const uint32_t* __restrict__ idx_in, int64_t n,
                                                                    int shift, const int32_t* __restrict__ block_base,
                                                                    uint32_t* __restrict__ keys_out,
                                                                    uint32_t* __restrict__ idx_out,
                                                                    uint32_t* __restrict__ rank_out) {
  __shared__ int32_t next[kSortWaves][kDigits];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t wave_first = (int64_t)blockIdx.x * kSortChunk + (int64_t)wave * kSortPerWave;
  for (int i = threadIdx.x; i < kSortWaves * kDigits; i += kSortThreads) (&next[0][0])[i] = 0;
  __syncthreads();
  for (int it = 0; it < kSortPerWave / kWave; ++it) {
    const int64_t p = wave_first + it * kWave + lane;
    if (p < n) atomicAdd(&next[wave][(keys_in[p] >> shift) & 0xff], 1);
  }
  __syncthreads();
  {
    const int d = threadIdx.x;  // kSortThreads == kDigits
    int32_t run = block_base[(int64_t)blockIdx.x * kDigits + d];
    for (int w = 0; w < kSortWaves; ++w) {
      const int32_t c = next[w][d];
      next[w][d] = run;
      run += c;
    }
  }
  __syncthreads();
  const uint64_t lower = (1ull << lane) - 1ull;
  for (int it = 0; it < kSortPerWave / kWave; ++it) {
    const int64_t p = wave_first + it * kWave + lane;
    int digit = -1;
    uint32_t key = 0, id = 0;
    if (p < n) {
      key = keys_in[p];
      id = idx_in[p];
      digit = (int)((key >> shift) & 0xff);
    }
    uint64_t waiting = __ballot(digit >= 0);
    int dst = -1;
    while (waiting) {
      const int leader = __ffsll((unsigned long long)waiting) - 1;
      const int ld = __shfl(digit, leader);
      const uint64_t same = __ballot(digit == ld);
      if (digit == ld) dst = next[wave][ld] + __popcll(same & lower);
      __builtin_amdgcn_wave_barrier();
      if (lane == leader) next[wave][ld] += __popcll(same);
      __builtin_amdgcn_wave_barrier();
      waiting &= ~same;
    }
    if (digit >= 0) {
      if (rank_out) {
        rank_out[id] = (uint32_t)dst;
      } else {
        keys_out[dst] = key;
        idx_out[dst] = id;
      }
    }
  }
}

static_assert(kSortThreads == kDigits, "one thread per digit in the scatter prologue");

}  // namespace

int64_t rank_workspace_words(int64_t n_micro, int want_rank) {
  int64_t words = n_micro / 4 + 64;  // class bytes
  if (want_rank) {
    const int64_t n_blocks = (n_micro + kSortChunk - 1) / kSortChunk;
    words += 4 * (n_micro + 64) + n_blocks * kDigits;
  }
  return words;
}

hipError_t launch_classify(hipStream_t stream, const float* energy, int64_t n_micro, const RankCuts& cuts,
                           uint8_t* class_out, uint8_t* byte_out, int32_t* kept_idx, int32_t* ws) {
  (void)ws;
  if (n_micro <= 0) return hipSuccess;
  hipLaunchKernelGGL(classify_kernel, dim3(1), dim3(kClsThreads), 0, stream, energy, n_micro, cuts, class_out,
                     byte_out, kept_idx);
  return hipGetLastError();
}

hipError_t launch_segment_counts(hipStream_t stream, const uint8_t* class_out, const SegTable& seg, int n_classes,
                                 int kept_only, int32_t* counts, int32_t* perm) {
  if (seg.n_seg <= 0) return hipSuccess;
  hipLaunchKernelGGL(segment_kernel, dim3((unsigned)seg.n_seg), dim3(kSegThreads), 0, stream, class_out, seg,
                     n_classes, kept_only, counts, perm);
  return hipGetLastError();
}

hipError_t launch_full_rank(hipStream_t stream, const float* energy, int64_t n_micro, uint32_t* rank,
                            int32_t* ws) {
  if (n_micro <= 0) return hipSuccess;
  const int64_t padded = n_micro + 64;
  uint32_t* keys_a = reinterpret_cast<uint32_t*>(ws);
  uint32_t* keys_b = keys_a + padded;
  uint32_t* idx_a = keys_b + padded;
  uint32_t* idx_b = idx_a + padded;
  int32_t* block_hist = reinterpret_cast<int32_t*>(idx_b + padded);
  const int n_blocks = (int)((n_micro + kSortChunk - 1) / kSortChunk);
  hipLaunchKernelGGL(sort_init_kernel, dim3((unsigned)((n_micro + kSortThreads - 1) / kSortThreads)),
                     dim3(kSortThreads), 0, stream, energy, n_micro, keys_a, idx_a);
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = pass * 8;
    hipLaunchKernelGGL(sort_count_kernel, dim3((unsigned)n_blocks), dim3(kSortThreads), 0, stream, keys_a, n_micro,
                       shift, block_hist);
    hipLaunchKernelGGL(sort_scan_kernel, dim3(1), dim3(kDigits), 0, stream, block_hist, n_blocks);
    hipLaunchKernelGGL(sort_scatter_kernel, dim3((unsigned)n_blocks), dim3(kSortThreads), 0, stream, keys_a, idx_a,
                       n_micro, shift, block_hist, keys_b, idx_b, pass == 3 ? rank : nullptr);
    uint32_t* t = keys_a; keys_a = keys_b; keys_b = t;
    t = idx_a; idx_a = idx_b; idx_b = t;
  }
  return hipGetLastError();
}

}  // namespace camera

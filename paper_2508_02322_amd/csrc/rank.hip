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
// rank_* kernels: the select passes and the walk for all cuts at once (the
// CAMERA-P cuts of several ratios and the CAMERA-Q class boundaries of a layer
// are cuts on the same order, so one set of passes serves both decisions), one
// workgroup per 4096 keys (<= 184 320 keys per layer in the paper's models:
// latency- and launch-bound, not bandwidth-bound).
// segment_kernel: one workgroup per expert: class sizes, from them the kept
// counts per ratio and the level sizes, and the stable partition of its
// micro-experts by precision level.
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
// classify: radix select for every cut, then the ordered classification walk.
//
// A layer has at most a few hundred thousand keys, so every pass is latency- and launch-bound:
// the work is spread over one workgroup per 4096 keys (each thread has its 16 keys in flight at
// once) and chained as short kernels on the stream.  After each histogram pass the workgroup
// that finishes last (a ticket from an atomic counter after a __threadfence; nobody waits for
// anybody) picks, for every cut, the bin that holds the cut element and publishes prefix / rest.
//   hist<P>   P = 0, 1, 2: 11 + 11 + 10 key bits; keys that share the cut's prefix so far
//   label     ordered walk: class byte, up to two output bytes, kept counts per workgroup
//   compact   (optional) ascending list of the kept indices
// The select state is self-cleaning: it starts as zeros (the library clears it when it makes it), pass 0
// seeds the per-cut fields from the call's cuts, and the last workgroup of every pass clears the histograms
// and the ticket it has just used.  A call therefore needs no clearing launch and leaves the state as it
// found it.  Equal keys that a cut runs through (rare: energies of experts without tokens) are ordered by
// index inside the label kernel, each workgroup counting the equal keys that precede it.
// ---------------------------------------------------------------------------
constexpr int kRankThreads = 256;
constexpr int kRankWaves = kRankThreads / kWave;
constexpr int kKeysPerBlock = kRankThreads * 16;  // 4096
constexpr int kKeysPerWave = kKeysPerBlock / kRankWaves;  // 1024 consecutive keys
constexpr int kBins = 2048;

struct RankState {  // persistent, see above
  uint32_t hist[3][kMaxCuts][kBins];
  uint32_t ticket[4];
  uint32_t prefix[kMaxCuts];  // key bits fixed so far (right-aligned); after pass 2 the key K of the cut element
  uint32_t rest[kMaxCuts];    // rank of the cut among keys sharing the prefix; after pass 2: equal keys below the cut
  int32_t mode[kMaxCuts];     // 0 select, 1 nothing below, 2 everything below
  uint32_t ties_split;        // some cut runs through a group of equal keys
};

__device__ __forceinline__ Keys4 keys_of(float4 v) {
  Keys4 k;
  k.k[0] = key_of(v.x);
  k.k[1] = key_of(v.y);
  k.k[2] = key_of(v.z);
  k.k[3] = key_of(v.w);
  k.valid[0] = k.valid[1] = k.valid[2] = k.valid[3] = true;
  return k;
}

// The 16 keys of this thread: wave w of the block owns 1024 consecutive keys, step u of the wave
// 256 of them, lane l keys 4 l .. 4 l + 3 of the step.  All four loads are issued together.
struct Keys16 {
  Keys4 g[4];
  int64_t first[4];
};
__device__ __forceinline__ Keys16 load_keys16(const float* __restrict__ E, int64_t n) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t base = (int64_t)blockIdx.x * kKeysPerBlock + (int64_t)wave * kKeysPerWave + lane * 4;
  Keys16 out;
  if ((int64_t)blockIdx.x * kKeysPerBlock + kKeysPerBlock <= n) {  // block-uniform: whole block inside
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(E + base + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) out.g[u] = keys_of(v[u]);
  } else {
#pragma unroll
    for (int u = 0; u < 4; ++u) out.g[u] = load_keys4(E, base + u * 256, n);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) out.first[u] = base + u * 256;
  return out;
}

// What another workgroup wrote before it took its ticket: read past this CU's vector cache.
__device__ __forceinline__ uint32_t load_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int cut_mode(const RankCuts& cuts, int q, int64_t n) {
  if (q >= cuts.n_cuts) return 1;
  const int64_t t = cuts.cut_rank[q];
  return t <= 0 ? 1 : (t >= n ? 2 : 0);
}

// Histogram pass P over the keys that share each cut's prefix, then (last workgroup) the pick.
template <int P>
__global__ __launch_bounds__(kRankThreads) void rank_hist_kernel(const float* __restrict__ E, int64_t n, RankCuts cuts,
                                                                RankState* __restrict__ st) {
  constexpr int kShift = P == 0 ? 21 : (P == 1 ? 10 : 0);
  constexpr int kBits = P == 2 ? 10 : 11;
  constexpr int kPrevShift = kShift + kBits;
  constexpr uint32_t kMask = (1u << kBits) - 1u;
  constexpr int kHists = P == 0 ? 1 : kMaxCuts;  // pass 0 has no prefix yet: one histogram serves every cut
  __shared__ uint32_t hist[kHists][kBins];
  __shared__ uint32_t s_last;
  const int tid = threadIdx.x;
  const int n_cuts = cuts.n_cuts;

  uint32_t want[kMaxCuts];
  bool any = false;
#pragma unroll
  for (int q = 0; q < kMaxCuts; ++q) {
    const bool on = P == 0 ? cut_mode(cuts, q, n) == 0 : (q < n_cuts && st->mode[q] == 0);
    want[q] = on ? (P == 0 ? 0u : st->prefix[q]) : 0xffffffffu;  // a real prefix has at most 22 bits
    any |= on;
  }
  if (P == 0 && blockIdx.x == 0 && tid < kMaxCuts) {
    // The per-cut fields of this call.  Nobody else reads them during pass 0 (the pick below takes the cut
    // ranks from the kernel argument) and only the pick of this pass writes prefix / rest after them.
    st->mode[tid] = cut_mode(cuts, tid, n);
    if (cut_mode(cuts, tid, n) != 0) {
      st->prefix[tid] = 0u;
      st->rest[tid] = 0u;
    }
    if (tid == 0) st->ties_split = 0u;
  }
  if (!any) return;  // block-uniform: no cut needs a select
  const int n_hists = P == 0 ? 1 : n_cuts;
  for (int i = tid; i < n_hists * kBins; i += kRankThreads) (&hist[0][0])[i] = 0u;
  __syncthreads();
  const Keys16 keys = load_keys16(E, n);
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!keys.g[u].valid[j]) continue;
      const uint32_t k = keys.g[u].k[j];
      if constexpr (P == 0) {
        atomicAdd(&hist[0][k >> kShift], 1u);
      } else {
        const uint32_t top = k >> kPrevShift;
#pragma unroll
        for (int q = 0; q < kMaxCuts; ++q)
          if (top == want[q]) atomicAdd(&hist[q][(k >> kShift) & kMask], 1u);
      }
    }
  __syncthreads();
  for (int i = tid; i < n_hists * kBins; i += kRankThreads) {
    const uint32_t c = (&hist[0][0])[i];
    if (c) atomicAdd(&st->hist[P][0][0] + i, c);
  }
  // last workgroup to get here sees every other workgroup's additions
  __threadfence();
  __syncthreads();
  if (tid == 0) s_last = atomicAdd(&st->ticket[P], 1u) == gridDim.x - 1 ? 1u : 0u;
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  // The pick, for all cuts together (one round of loads, one scan): thread t owns bins kPer t .. kPer t + kPer - 1
  // of every cut's histogram (pass 0: the one histogram all cuts share).
  constexpr int kPer = kBins / kRankThreads;
  uint32_t c[kHists][kPer], before[kHists];
#pragma unroll
  for (int q = 0; q < kHists; ++q) {
    before[q] = 0u;
    const bool on = P == 0 || want[q] != 0xffffffffu;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      c[q][i] = on ? load_agent(&st->hist[P][q][tid * kPer + i]) : 0u;
      before[q] += c[q][i];
    }
  }
  {  // exclusive prefix over the threads, every histogram at once
    const int lane = tid % kWave, wave = tid / kWave;
    __shared__ uint32_t s_tot[kRankWaves][kHists];
    uint32_t inc[kHists];
#pragma unroll
    for (int q = 0; q < kHists; ++q) {
      inc[q] = before[q];
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t o = __shfl_up(inc[q], d);
        if (lane >= d) inc[q] += o;
      }
      if (lane == kWave - 1) s_tot[wave][q] = inc[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kHists; ++q) {
      uint32_t base = 0;
      for (int w = 0; w < wave; ++w) base += s_tot[w][q];
      before[q] = base + inc[q] - before[q];
    }
  }
#pragma unroll
  for (int q = 0; q < kMaxCuts; ++q) {
    if (q >= n_cuts || want[q] == 0xffffffffu) continue;  // block-uniform
    constexpr int kShared = P == 0 ? 1 : kMaxCuts;
    const int hq = q % kShared;  // pass 0: histogram 0 serves every cut
    const uint32_t rest = P == 0 ? (uint32_t)cuts.cut_rank[q] : st->rest[q];
    uint32_t run = before[hq];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      if (rest >= run && rest < run + c[hq][i]) {
        st->prefix[q] = (want[q] << kBits) | (uint32_t)(tid * kPer + i);
        st->rest[q] = rest - run;
        if (P == 2 && rest - run > 0) st->ties_split = 1u;
      }
      run += c[hq][i];
    }
  }
  __syncthreads();
  // leave the state as the next call needs it: this pass's histograms and ticket back to zero
  for (int i = tid; i < n_hists * kBins; i += kRankThreads) (&st->hist[P][0][0])[i] = 0u;
  if (tid == 0) st->ticket[P] = 0u;
}

// Ordered walk: an element is below cut q iff key < K_q, or key == K_q and fewer than rest_q equal
// keys precede it (by index).  Writes the class (number of cuts it is below) and the output bytes.
__global__ __launch_bounds__(kRankThreads) void rank_label_kernel(const float* __restrict__ E, int64_t n,
                                                                 RankCuts cuts, const RankState* __restrict__ st,
                                                                 uint8_t* __restrict__ class_out,
                                                                 uint8_t* __restrict__ byte_out,
                                                                 uint8_t* __restrict__ byte_out2 /*or NULL*/,
                                                                 uint32_t* __restrict__ kept_cnt /*[grid] or NULL*/) {
  __shared__ uint32_t s_tie[kMaxCuts][kRankWaves];
  __shared__ uint32_t s_before[kMaxCuts][kRankWaves];
  __shared__ uint32_t s_kept[kRankWaves];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint64_t lower = (1ull << lane) - 1ull;
  const bool ties_split = st->ties_split != 0;
  uint32_t K[kMaxCuts], R[kMaxCuts];
  int mode[kMaxCuts];
#pragma unroll
  for (int q = 0; q < kMaxCuts; ++q) {
    mode[q] = q < cuts.n_cuts ? st->mode[q] : 1;
    K[q] = st->prefix[q];
    R[q] = mode[q] == 0 ? st->rest[q] : 0u;
  }
  const Keys16 keys = load_keys16(E, n);

  uint32_t tie_base[kMaxCuts];
#pragma unroll
  for (int q = 0; q < kMaxCuts; ++q) tie_base[q] = 0u;
  if (ties_split) {  // block-uniform
    // equal keys before this wave: in the workgroups before this one (counted here, by all threads, over
    // keys [0, first key of this workgroup)) and in the earlier waves of this one
    uint32_t mine[kMaxCuts], before[kMaxCuts];
#pragma unroll
    for (int q = 0; q < kMaxCuts; ++q) {
      mine[q] = 0u;
      before[q] = 0u;
      if (mode[q] == 0 && R[q] > 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            mine[q] += __popcll(__ballot(keys.g[u].valid[j] && keys.g[u].k[j] == K[q]));
      }
    }
    const int64_t n_before = (int64_t)blockIdx.x * kKeysPerBlock;  // a multiple of 4, all inside [0, n)
    for (int64_t i = (int64_t)threadIdx.x * 4; i < n_before; i += kRankThreads * 4) {
      const Keys4 k = keys_of(*reinterpret_cast<const float4*>(E + i));
#pragma unroll
      for (int q = 0; q < kMaxCuts; ++q)
        if (mode[q] == 0 && R[q] > 0) {
#pragma unroll
          for (int j = 0; j < 4; ++j) before[q] += k.k[j] == K[q] ? 1u : 0u;
        }
    }
#pragma unroll
    for (int q = 0; q < kMaxCuts; ++q) {
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) before[q] += __shfl_xor(before[q], m);
    }
    if (lane == 0) {
#pragma unroll
      for (int q = 0; q < kMaxCuts; ++q) {
        s_tie[q][wave] = mine[q];
        s_before[q][wave] = before[q];
      }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kMaxCuts; ++q) {
      if (mode[q] == 0 && R[q] > 0) {
        uint32_t run = 0;
        for (int w = 0; w < kRankWaves; ++w) run += s_before[q][w];
        for (int w = 0; w < wave; ++w) run += s_tie[q][w];
        tie_base[q] = run;
      }
    }
  }

  uint32_t kept = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const Keys4& k = keys.g[u];
    const int64_t i = keys.first[u];
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
      if (byte_out2) {
        const uint32_t second4 = (uint32_t)cuts.out2_of_below[below[0]] | ((uint32_t)cuts.out2_of_below[below[1]] << 8) |
                                 ((uint32_t)cuts.out2_of_below[below[2]] << 16) |
                                 ((uint32_t)cuts.out2_of_below[below[3]] << 24);
        *reinterpret_cast<uint32_t*>(byte_out2 + i) = second4;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (k.valid[j]) {
          class_out[i + j] = (uint8_t)below[j];
          byte_out[i + j] = cuts.out_of_below[below[j]];
          if (byte_out2) byte_out2[i + j] = cuts.out2_of_below[below[j]];
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) kept += __popcll(__ballot(k.valid[j] && below[j] == 0));
  }
  if (kept_cnt == nullptr) return;  // block-uniform
  if (lane == 0) s_kept[wave] = kept;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t total = 0;
    for (int w = 0; w < kRankWaves; ++w) total += s_kept[w];
    kept_cnt[blockIdx.x] = total;
  }
}

// Ascending list of the indices of class 0 (below no cut).
__global__ __launch_bounds__(kRankThreads) void rank_compact_kernel(const uint8_t* __restrict__ class_in, int64_t n,
                                                                   const uint32_t* __restrict__ kept_cnt,
                                                                   int32_t* __restrict__ kept_idx) {
  __shared__ uint32_t s_kept[kRankWaves];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint64_t lower = (1ull << lane) - 1ull;
  const int64_t base = (int64_t)blockIdx.x * kKeysPerBlock + (int64_t)wave * kKeysPerWave + lane * 4;
  bool is_kept[4][4];
  uint32_t mine = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = base + u * 256;
    uint32_t c4 = 0x01010101u;
    if (i + 3 < n) {
      c4 = *reinterpret_cast<const uint32_t*>(class_in + i);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i + j < n) c4 = (c4 & ~(0xffu << (8 * j))) | ((uint32_t)class_in[i + j] << (8 * j));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      is_kept[u][j] = ((c4 >> (8 * j)) & 0xffu) == 0u;
      mine += __popcll(__ballot(is_kept[u][j]));
    }
  }
  if (lane == 0) s_kept[wave] = mine;
  __syncthreads();
  uint32_t pos = 0;
  for (int b = lane; b < (int)blockIdx.x; b += kWave) pos += kept_cnt[b];
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) pos += __shfl_xor(pos, m);
  for (int w = 0; w < wave; ++w) pos += s_kept[w];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    uint32_t lanes_before = 0, total = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint64_t b = __ballot(is_kept[u][j]);
      lanes_before += __popcll(b & lower);
      total += __popcll(b);
    }
    uint32_t p = pos + lanes_before;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (is_kept[u][j]) kept_idx[p++] = (int32_t)(base + u * 256 + j);
    pos += total;
  }
}

// ---------------------------------------------------------------------------
// per segment (expert): class sizes, from them the kept counts of every pruning ratio and the sizes of
// the precision levels, and the stable partition of the segment by level
// ---------------------------------------------------------------------------
constexpr int kSegThreads = 1024;  // a shared expert can be a 20 480-element segment: 16 waves walk it
constexpr int kSegWaves = kSegThreads / kWave;

__device__ __forceinline__ int nibble(uint32_t packed, int c) { return (int)((packed >> (4 * c)) & 15u); }

__global__ __launch_bounds__(kSegThreads) void segment_kernel(const uint8_t* __restrict__ class_in, SegTable seg,
                                                              SegOutputs out) {
  __shared__ uint32_t s_cnt[kSegWaves][CAMERA_MAX_LEVELS];   // per wave and class
  __shared__ uint32_t s_lvl[kSegWaves][CAMERA_MAX_LEVELS];   // per wave and level
  const int s = blockIdx.x;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int begin = seg.off[s], end = seg.off[s + 1];
  const int span = ((end - begin + kSegWaves * kWave - 1) / (kSegWaves * kWave)) * kWave;
  const int w_begin = min(end, begin + wave * span);
  const int w_end = min(end, w_begin + span);
  const uint64_t lower = (1ull << lane) - 1ull;
  const int n_classes = out.n_classes;

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
  if (threadIdx.x < kSegWaves * CAMERA_MAX_LEVELS) {  // (wave w, level m): members of level m in wave w's range
    const int w = threadIdx.x / CAMERA_MAX_LEVELS, m = threadIdx.x % CAMERA_MAX_LEVELS;
    uint32_t total = 0;
    for (int c = 0; c < n_classes; ++c)
      if (nibble(out.level_of_class, c) == m) total += s_cnt[w][c];
    s_lvl[w][m] = total;
  }
  if (threadIdx.x >= 512 && threadIdx.x < 512 + out.n_ratios) {
    // kept at ratio k: the members of the classes that lie below at most n_ratios - 1 - k of the pruning cuts
    const int k = threadIdx.x - 512;
    uint32_t total = 0;
    for (int c = 0; c < n_classes; ++c)
      if (nibble(out.prune_cuts_of_class, c) <= out.n_ratios - 1 - k)
        for (int w = 0; w < kSegWaves; ++w) total += s_cnt[w][c];
    out.kept[k * seg.n_seg + s] = (int32_t)total;
  }
  __syncthreads();
  if (threadIdx.x < out.n_levels) {
    uint32_t total = 0;
    for (int w = 0; w < kSegWaves; ++w) total += s_lvl[w][threadIdx.x];
    out.level_count[s * out.n_levels + threadIdx.x] = (int32_t)total;
  }
  if (out.perm == nullptr) return;  // block-uniform

  // first slot of level m for this wave: segment start + all earlier levels + earlier waves
  uint32_t slot[CAMERA_MAX_LEVELS];
  uint32_t run = (uint32_t)begin;
#pragma unroll
  for (int m = 0; m < CAMERA_MAX_LEVELS; ++m) {
    slot[m] = 0;
    if (m < out.n_levels) {
      for (int w = 0; w < kSegWaves; ++w) {
        if (w == wave) slot[m] = run;
        run += s_lvl[w][m];
      }
    }
  }
  for (int i0 = w_begin; i0 < w_end; i0 += 4 * kWave) {
    int lv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kWave + lane;
      lv[u] = i < w_end ? nibble(out.level_of_class, (int)class_in[i] & 7) : -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kWave + lane;
#pragma unroll
      for (int m = 0; m < CAMERA_MAX_LEVELS; ++m) {
        if (m < out.n_levels) {
          const uint64_t b = __ballot(lv[u] == m);
          if (lv[u] == m) out.perm[slot[m] + __popcll(b & lower)] = i;
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

int64_t rank_blocks(int64_t n_micro) { return (n_micro + kKeysPerBlock - 1) / kKeysPerBlock; }

size_t rank_state_bytes() { return sizeof(RankState); }

int64_t rank_workspace_words(int64_t n_micro, int want_rank) {
  const int64_t g = rank_blocks(n_micro);
  int64_t words = g + 64;  // kept counts per workgroup
  if (want_rank) {
    const int64_t n_blocks = (n_micro + kSortChunk - 1) / kSortChunk;
    words += 4 * (n_micro + 64) + n_blocks * kDigits;
  }
  return words;
}

hipError_t launch_classify(hipStream_t stream, const float* energy, int64_t n_micro, const RankCuts& cuts,
                           uint8_t* class_out, uint8_t* byte_out, uint8_t* byte_out2, int32_t* kept_idx, void* state,
                           int32_t* ws) {
  if (n_micro <= 0) return hipSuccess;
  const unsigned g = (unsigned)rank_blocks(n_micro);
  RankState* st = static_cast<RankState*>(state);
  uint32_t* kept_cnt = reinterpret_cast<uint32_t*>(ws);
  hipLaunchKernelGGL(rank_hist_kernel<0>, dim3(g), dim3(kRankThreads), 0, stream, energy, n_micro, cuts, st);
  hipLaunchKernelGGL(rank_hist_kernel<1>, dim3(g), dim3(kRankThreads), 0, stream, energy, n_micro, cuts, st);
  hipLaunchKernelGGL(rank_hist_kernel<2>, dim3(g), dim3(kRankThreads), 0, stream, energy, n_micro, cuts, st);
  hipLaunchKernelGGL(rank_label_kernel, dim3(g), dim3(kRankThreads), 0, stream, energy, n_micro, cuts, st, class_out,
                     byte_out, byte_out2, kept_idx ? kept_cnt : nullptr);
  if (kept_idx)
    hipLaunchKernelGGL(rank_compact_kernel, dim3(g), dim3(kRankThreads), 0, stream, class_out, n_micro, kept_cnt,
                       kept_idx);
  return hipGetLastError();
}

hipError_t launch_segment_outputs(hipStream_t stream, const uint8_t* class_out, const SegTable& seg,
                                  const SegOutputs& out) {
  if (seg.n_seg <= 0) return hipSuccess;
  hipLaunchKernelGGL(segment_kernel, dim3((unsigned)seg.n_seg), dim3(kSegThreads), 0, stream, class_out, seg, out);
  return hipGetLastError();
}

hipError_t launch_full_rank(hipStream_t stream, const float* energy, int64_t n_micro, uint32_t* rank,
                            int32_t* ws) {
  if (n_micro <= 0) return hipSuccess;
  const int64_t padded = n_micro + 64;
  ws += rank_workspace_words(n_micro, 0);  // behind the kept counts
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

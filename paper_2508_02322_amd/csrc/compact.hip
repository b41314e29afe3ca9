// The layer output from compacted weights (the result of Algorithm 2, lines
// 10-13: every expert keeps its own number of micro-experts), for the small
// token batches of decoding (the setting of the decoding-speed comparison of a
// pruned MoE layer, batch of 64 tokens).
//
// With a handful of tokens per expert the layer is bound by reading each
// activated expert's weights once, so no operand is tiled through LDS: a
// workgroup owns 32 weight rows and up to 32 tokens of one expert, its waves
// split the K extent between them and stream their share from HBM straight
// into MFMA operand registers (v_mfma_f32_32x32x16_bf16: the weight rows are
// the M side, the tokens the N side); the partial sums of the waves meet in
// LDS, added in wave order.  Work items are kept small and alike, so that a
// launch has several times more workgroups than the chip holds at once and its
// last round does not leave most compute units idle:
//   - the K extent of a workgroup is split between its waves;
//   - the 32-token groups of an expert go to different workgroups (grid y),
//     which read the same weights at about the same time (the second read is
//     served by the caches); the workgroups of groups an expert does not have
//     leave at once;
//   - in the second contraction an expert with many kept micro-experts (a
//     large shared expert) is cut into K chunks that go to different
//     workgroups, each writing its own partial product rows; the chunks are
//     added, in chunk order, when the token's experts are summed.
// Inside a 64-element K block lane (row, half) holds the 32 consecutive
// elements [32*half, 32*half + 32) of its row as four 16-byte loads, so the two
// lanes of a row read one full 128-byte line; the token operand uses the same
// K order, which a sum over K does not care about.  Experts that no token of
// the batch selected are skipped before any weight is read.
//
//   hidden  : Lambda[slot][c] = a silu(x w_gate,c) (x w_up,c), bf16, for the c < count[e] kept micro-experts
//   down    : partial[chunk][slot][r] = sum over the chunk's c of Lambda[slot][c] W_down_e[r][c], float32
//   combine : y_token (+)= the partial rows of its experts' slots, experts in k order, chunks in chunk order
// The rows of the compacted W_down block of an expert hold count[e] elements and
// then zeros up to the caller's row alignment.  Without alignment (rows of any
// length) its 16-byte loads are unaligned (2-byte aligned) and the chunk that
// straddles the end of a row is taken as the 16 bytes that end there, shifted
// down: correct, but a third slower than rows that start on 128-byte lines.
#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
typedef __attribute__((ext_vector_type(8))) int16_t i16x8;

// Waves of a workgroup, each with its share of the K blocks (1, 2 or 4: the four accumulator groups of a lane
// are dealt to them after the reduction).  The first contraction's K extent is d_model.
#ifndef CAMERA_COMPACT_KSPLIT_HIDDEN
#define CAMERA_COMPACT_KSPLIT_HIDDEN 4
#endif
constexpr int kSplitHidden = CAMERA_COMPACT_KSPLIT_HIDDEN;
static_assert(kSplitHidden == 1 || kSplitHidden == 2 || kSplitHidden == 4, "1, 2 or 4 waves");
// The second contraction's K extent is the expert's kept count, which shrinks with the pruning ratio: four
// waves while a K chunk gives each of them at least five K blocks, two below that (measured 3-8 % apart).
constexpr int kDownFourWavesFrom = 1280;
constexpr int kRows = 32;    // weight rows per workgroup (the MFMA's M)
constexpr int kTokens = 32;  // tokens per workgroup (the MFMA's N)
constexpr int kKBlock = 64;  // K elements per step: 4 MFMAs of K = 16

__device__ __forceinline__ float silu_f32(float g) {
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
  return z;
}

// 16 bytes from a 16-byte aligned address
__device__ __forceinline__ bf16x8 load8(const __bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
// 16 bytes from an address that is only element aligned
__device__ __forceinline__ bf16x8 load8_unaligned(const __bf16* p) {
  bf16x8 v;
  __builtin_memcpy(&v, p, sizeof(v));
  return v;
}

// One lane's share of a 64-element K block: chunk j covers elements [8j, 8j + 8) of the lane's 32.
struct Frag {
  bf16x8 c[4];
};

template <bool ALIGNED>
__device__ __forceinline__ void load_frag(Frag& f, const __bf16* p) {
#pragma unroll
  for (int j = 0; j < 4; ++j) f.c[j] = ALIGNED ? load8(p + 8 * j) : load8_unaligned(p + 8 * j);
}

// out[i] = w[i + d] for i + d < 8, else 0 (1 <= d <= 7, the same for the whole wave)
__device__ __forceinline__ bf16x8 shift_down(bf16x8 w, int d) {
  const u64x2 v = __builtin_bit_cast(u64x2, w);
  const int s = 16 * d;
  u64x2 o;
  if (s < 64) {
    o[0] = (v[0] >> s) | (v[1] << (64 - s));
    o[1] = v[1] >> s;
  } else {
    o[0] = v[1] >> (s - 64);
    o[1] = 0;
  }
  return __builtin_bit_cast(bf16x8, o);
}

// The last, partial K block of an operand row.  `k` is the K index (inside the block) of the lane's first element,
// `k_full` the end of the valid elements.  MODE says what lies behind k_full:
//   kWhole   k_full is a multiple of 8 (no partial chunk)
//   kPadded  the row is zero-filled and readable up to the next multiple of 8
//   kRagged  nothing at or beyond k_full may be touched: the chunk that straddles the end is taken as the 16 bytes
//            that end at k_full, shifted down (`row_k`, the valid elements of the whole row, must be >= 8 for
//            that; shorter rows are read element by element)
enum TailMode { kWhole, kPadded, kRagged };
template <bool ALIGNED, TailMode MODE>
__device__ __forceinline__ void load_frag_tail(Frag& f, const __bf16* p, int k, int k_full, int row_k) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int kj = k + 8 * j;
    if (kj + 8 <= k_full || (MODE == kPadded && kj < k_full)) {
      f.c[j] = ALIGNED ? load8(p + 8 * j) : load8_unaligned(p + 8 * j);
    } else if (MODE == kRagged && kj < k_full) {
      const int valid = k_full - kj;  // 1..7, the same for every lane that gets here
      if (row_k >= 8) {
        f.c[j] = shift_down(load8_unaligned(p + 8 * j + valid - 8), 8 - valid);
      } else {
        u64x2 o = {0, 0};
#pragma unroll 1
        for (int i = 0; i < valid; ++i) {
          const uint64_t x = __builtin_bit_cast(uint16_t, p[8 * j + i]);
          o[i >> 2] |= x << (16 * (i & 3));
        }
        f.c[j] = __builtin_bit_cast(bf16x8, o);
      }
    } else {
      f.c[j] = zero8();
    }
  }
}

__device__ __forceinline__ void mfma4(f32x16& acc, const Frag& a, const Frag& b) {
#pragma unroll
  for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.c[j], b.c[j], acc, 0, 0, 0);
}

// ---- partial sums of the waves ------------------------------------------------------------------------------
// red[wave][tile][i][lane]: accumulator element i of `lane`.  With one wave per workgroup nothing goes through LDS.
template <int KS, int TILES>
struct Reduce {
  float (*red)[TILES][16][kWave];
  __device__ __forceinline__ void put(int wave, int tile, const f32x16& acc, int lane) const {
#pragma unroll
    for (int i = 0; i < 16; ++i) red[wave][tile][i][lane] = acc[i];
  }
  __device__ __forceinline__ float get(int tile, int i, int lane) const {
    float s = red[0][tile][i][lane];
#pragma unroll
    for (int w = 1; w < KS; ++w) s += red[w][tile][i][lane];
    return s;
  }
};
// The groups of four accumulator elements (q = i / 4) that `wave` finishes after the reduction.
template <int KS>
__device__ __forceinline__ bool owns_group(int wave, int q) { return (q * KS) / 4 == wave; }

// K blocks [kb0, kb1) of a wave; the wave with `tail` also takes the partial block after the last full one.
struct KRange {
  int kb0, kb1;
  bool tail;
};
template <int KS>
__device__ __forceinline__ KRange k_range(int full_blocks, bool has_tail, int wave) {
  KRange k;
  k.kb0 = full_blocks * wave / KS;
  k.kb1 = full_blocks * (wave + 1) / KS;
  k.tail = has_tail && wave == KS - 1;
  return k;
}

// Last index e in [0, n) with off[e] <= x, for a rising table with off[0] <= x < off[n].
__device__ __forceinline__ int find_segment(const int32_t* off, int n, int x) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

// ---- Lambda = a silu(X W_gate^T) (X W_up^T) on the kept rows ----------------------------------------------
__device__ __forceinline__ void hidden_pass(const __bf16* __restrict__ wg, const __bf16* __restrict__ wu,
                                            const __bf16* __restrict__ x, int d_model, KRange kr, f32x16& g,
                                            f32x16& u) {
  Frag ag[2], au[2], b[2];
  auto fetch = [&](int buf, int kb) {
    const int off = kb * kKBlock;
    load_frag<true>(ag[buf], wg + off);
    load_frag<true>(au[buf], wu + off);
    load_frag<true>(b[buf], x + off);
  };
  auto multiply = [&](int buf) {
    mfma4(g, ag[buf], b[buf]);
    mfma4(u, au[buf], b[buf]);
  };
  int kb = kr.kb0;
  if (kb < kr.kb1) fetch(0, kb);
  for (; kb + 2 <= kr.kb1; kb += 2) {  // the loads of the next block are in flight while this one multiplies
    fetch(1, kb + 1);
    multiply(0);
    if (kb + 2 < kr.kb1) fetch(0, kb + 2);
    multiply(1);
  }
  if (kb < kr.kb1) multiply(0);
  if (kr.tail) {
    const int full = d_model / kKBlock;
    const int rem = d_model - full * kKBlock;         // a multiple of 8
    const int half_k = (threadIdx.x & 63) >> 5 << 5;  // K index of the lane's first element inside the block
    const int off = full * kKBlock;
    load_frag_tail<true, kWhole>(ag[0], wg + off, half_k, rem, d_model);
    load_frag_tail<true, kWhole>(au[0], wu + off, half_k, rem, d_model);
    load_frag_tail<true, kWhole>(b[0], x + off, half_k, rem, d_model);
    multiply(0);
  }
}

// grid: x = 32-row tiles of all experts (exactly tab.tile_off[tab.n_experts]), y = 32-token groups.  The
// workgroups of the last group also take any further groups of their expert (an expert can hold more tokens
// than the batch has only if a token names it twice).
template <int KS>
__global__ __launch_bounds__(kWave * KS) __attribute__((amdgpu_waves_per_eu(2))) void compact_hidden_kernel(
    const __bf16* __restrict__ X, int64_t ldx, int d_model, const __bf16* __restrict__ W_gate,
    const __bf16* __restrict__ W_up, CompactRows tab, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm, const float* __restrict__ w_perm,
    __bf16* __restrict__ H, int ldh) {
  __shared__ float red_mem[KS][2][16][kWave];  // gate and up
  const Reduce<KS, 2> red{red_mem};
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int tile = blockIdx.x;
  const int e = find_segment(tab.tile_off, tab.n_experts, tile);
  const int m = __builtin_amdgcn_readfirstlane(counts[e]);
  const int t_first = (int)blockIdx.y * kTokens;
  if (t_first >= m) return;  // no token (of this group) selected the expert: the whole workgroup leaves, nothing is read
  const bool last_group = blockIdx.y + 1 == gridDim.y;
  const int slot0 = __builtin_amdgcn_readfirstlane(offsets[e]);
  const int cnt = tab.row_off[e + 1] - tab.row_off[e];
  const int cnt8 = (cnt + 7) & ~7;
  const int c0 = (tile - tab.tile_off[e]) * kRows;
  const int r = lane & 31, h = lane >> 5;
  const int row = min(c0 + r, cnt - 1);  // rows past the expert's end repeat its last row; their results are dropped
  const int64_t w_off = ((int64_t)tab.row_off[e] + row) * d_model + h * 32;
  const __bf16* wg = W_gate + w_off;
  const __bf16* wu = W_up + w_off;
  const KRange kr = k_range<KS>(d_model / kKBlock, d_model % kKBlock != 0, wave);

  for (int t0 = t_first; t0 < m; t0 += kTokens) {
    const int t = t0 + r;
    const int tc = min(t, m - 1);  // clamped: columns past m are dropped
    const int64_t tok = perm ? perm[slot0 + tc] : tc;
    const __bf16* x = X + tok * ldx + h * 32;
    f32x16 g = {}, u = {};
    hidden_pass(wg, wu, x, d_model, kr, g, u);
    if constexpr (KS > 1) {
      red.put(wave, 0, g, lane);
      red.put(wave, 1, u, lane);
      __syncthreads();
    }
    // accumulator element i of a lane: weight row 8*(i/4) + 4*h + i%4, token column r
    if (t < m) {
      const int64_t slot = slot0 + t;
      const float a = w_perm ? w_perm[slot] : 1.0f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!owns_group<KS>(wave, q)) continue;
        const int c = c0 + 8 * q + 4 * h;
        if (c >= cnt8) continue;  // columns [cnt, cnt8) are written as zeros: the down kernel reads whole chunks
        bf16x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float gv = KS > 1 ? red.get(0, 4 * q + i, lane) : g[4 * q + i];
          const float uv = KS > 1 ? red.get(1, 4 * q + i, lane) : u[4 * q + i];
          const float lam = a * silu_f32(gv) * uv;
          out[i] = (__bf16)(c + i < cnt ? lam : 0.0f);
        }
        *reinterpret_cast<bf16x4*>(H + slot * ldh + c) = out;
      }
    }
    if (!last_group) break;
    if constexpr (KS > 1) __syncthreads();  // the next pass writes the same LDS
  }
}

// ---- partial = Lambda W_down_e^T over one K chunk ----------------------------------------------------------
// wd, hrow point at the first element of the chunk; k_len its length; row_k the valid length of the whole row.
__device__ __forceinline__ void down_pass(const __bf16* __restrict__ wd, const __bf16* __restrict__ hrow, int k_len,
                                          int row_k, KRange kr, f32x16& p) {
  Frag a[2], b[2];
  auto fetch = [&](int buf, int kb) {
    const int off = kb * kKBlock;
    load_frag<false>(a[buf], wd + off);
    load_frag<true>(b[buf], hrow + off);
  };
  int kb = kr.kb0;
  if (kb < kr.kb1) fetch(0, kb);
  for (; kb + 2 <= kr.kb1; kb += 2) {
    fetch(1, kb + 1);
    mfma4(p, a[0], b[0]);
    if (kb + 2 < kr.kb1) fetch(0, kb + 2);
    mfma4(p, a[1], b[1]);
  }
  if (kb < kr.kb1) mfma4(p, a[0], b[0]);
  if (kr.tail) {
    const int full = k_len / kKBlock;
    const int rem = k_len - full * kKBlock;
    const int half_k = (threadIdx.x & 63) >> 5 << 5;
    const int off = full * kKBlock;
    load_frag_tail<false, kRagged>(a[0], wd + off, half_k, rem, row_k);   // never past the end of the weight row
    load_frag_tail<true, kPadded>(b[0], hrow + off, half_k, rem, row_k);  // Lambda rows are zero-filled up to a multiple of 8
    mfma4(p, a[0], b[0]);
  }
}

// Length of the K chunks of an expert with cnt kept micro-experts cut into n_chunks (a multiple of 64).
__device__ __forceinline__ int chunk_length(int cnt, int n_chunks) {
  return ((cnt + n_chunks - 1) / n_chunks + kKBlock - 1) & ~(kKBlock - 1);
}

// grid: x = (K chunk of an expert, 32-row tile of d_model): tab.chunk_off[tab.n_experts] * row_tiles workgroups,
// y = 32-token groups.  partial is [chunk within the expert][n_slots][d_model].
template <int KS>
__global__ __launch_bounds__(kWave * KS) __attribute__((amdgpu_waves_per_eu(3))) void compact_down_kernel(
    const __bf16* __restrict__ H, int ldh, const __bf16* __restrict__ W_down, int d_model, CompactDown tab,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ offsets, int64_t n_slots,
    float* __restrict__ partial) {
  __shared__ float red_mem[KS][1][16][kWave];
  const Reduce<KS, 1> red{red_mem};
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int row_tiles = (d_model + kRows - 1) / kRows;
  const int chunk = blockIdx.x / row_tiles;
  const int r0 = ((int)blockIdx.x - chunk * row_tiles) * kRows;
  const int e = find_segment(tab.chunk_off, tab.n_experts, chunk);
  const int m = __builtin_amdgcn_readfirstlane(counts[e]);
  const int t_first = (int)blockIdx.y * kTokens;
  if (t_first >= m) return;
  const bool last_group = blockIdx.y + 1 == gridDim.y;
  const int slot0 = __builtin_amdgcn_readfirstlane(offsets[e]);
  const int cnt = tab.count[e];
  const int ld = tab.ld_off[e + 1] - tab.ld_off[e];  // row length of the expert's block (cnt and zero padding)
  const int chunk_in = chunk - tab.chunk_off[e];
  const int len = chunk_length(cnt, tab.chunk_off[e + 1] - tab.chunk_off[e]);
  const int k0 = min(chunk_in * len, cnt);
  const int k_len = min(len, cnt - k0);
  const int r = lane & 31, h = lane >> 5;
  const int row = min(r0 + r, d_model - 1);
  const __bf16* wd = W_down + (int64_t)tab.ld_off[e] * d_model + (int64_t)row * ld + k0 + h * 32;
  const KRange kr = k_range<KS>(k_len / kKBlock, k_len % kKBlock != 0, wave);
  float* out_chunk = partial + (int64_t)chunk_in * n_slots * d_model;

  for (int t0 = t_first; t0 < m; t0 += kTokens) {
    const int t = t0 + r;
    const __bf16* hrow = H + (int64_t)(slot0 + min(t, m - 1)) * ldh + k0 + h * 32;
    f32x16 p = {};
    down_pass(wd, hrow, k_len, cnt, kr, p);
    if constexpr (KS > 1) {
      red.put(wave, 0, p, lane);
      __syncthreads();
    }
    if (t < m) {
      float* out = out_chunk + (int64_t)(slot0 + t) * d_model;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!owns_group<KS>(wave, q)) continue;
        const int rr = r0 + 8 * q + 4 * h;
        if (rr >= d_model) continue;  // d_model is a multiple of 8: a group of four is inside or outside as a whole
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = KS > 1 ? red.get(0, 4 * q + i, lane) : p[4 * q + i];
        *reinterpret_cast<float4*>(out + rr) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
    if (!last_group) break;
    if constexpr (KS > 1) __syncthreads();
  }
}

// ---- y_token (+)= its partial rows -------------------------------------------------------------------------
// One thread per (token, four output columns).  Routed: the token's slots are slot_of[token * terms + k], the
// expert of a slot is found in `offsets`; dense (slot_of == nullptr): expert k, slot k * n + token.
__global__ __launch_bounds__(256) void compact_combine_kernel(const float4* __restrict__ partial,
                                                              const int32_t* __restrict__ slot_of,
                                                              const int32_t* __restrict__ offsets, CompactDown tab,
                                                              int64_t n, int terms, int vecs, int64_t n_slots,
                                                              int accumulate, float4* __restrict__ Y) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= n * vecs) return;
  const int64_t tok = id / vecs;
  const int v = (int)(id - tok * vecs);
  float4 s = accumulate ? Y[id] : make_float4(0.f, 0.f, 0.f, 0.f);
  for (int k = 0; k < terms; ++k) {
    int64_t slot;
    int e;
    if (slot_of) {
      slot = slot_of[tok * terms + k];
      if (slot < 0) continue;  // a pair with an expert id outside the group
      e = find_segment(offsets, tab.n_experts, (int)slot);
    } else {
      slot = (int64_t)k * n + tok;
      e = k;
    }
    const int chunks = tab.chunk_off[e + 1] - tab.chunk_off[e];
    for (int c = 0; c < chunks; ++c) {
      const float4 p = partial[((int64_t)c * n_slots + slot) * vecs + v];
      s.x += p.x;
      s.y += p.y;
      s.z += p.z;
      s.w += p.w;
    }
  }
  Y[id] = s;
}

// ---- bucket order of a decoding batch ----------------------------------------------------------------------
// Pair p = token * (top_k + n_shared) + k: for k < top_k the routed expert topk_idx[token][k] with weight
// topk_w[token][k], for k >= top_k the appended expert n_experts + k - top_k with weight 1.
//
// One workgroup does what the three launches of the general counting sort do, for at most kCompactSmallPairs
// pairs.  Four threads per expert, each with a quarter of the pair range: a thread counts the pairs of its
// expert in its quarter, an exclusive prefix over the threads (expert-major, quarter-minor: the stable order)
// gives its first slot, and it places its pairs in pair order.
constexpr int kQuarters = 4;
constexpr int kSmallThreads = CAMERA_MAX_EXPERTS * kQuarters;
static_assert(kSmallThreads <= 1024, "one workgroup");

__global__ __launch_bounds__(kSmallThreads) void compact_bucket_small_kernel(
    const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w, int n, int top_k, int n_experts,
    int n_shared, int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
    float* __restrict__ w_perm, int32_t* __restrict__ slot_of) {
  __shared__ __attribute__((aligned(16))) int16_t ids[kCompactSmallPairs];  // expert of every pair, -1: none
  __shared__ int16_t token[kCompactSmallPairs];                             // its token
  __shared__ float weight[kCompactSmallPairs];                              // and its weight
  __shared__ int32_t wave_total[kSmallThreads / kWave];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kk = top_k + n_shared, total = n_experts + n_shared, n_pairs = n * kk;
  const int padded = (n_pairs + 7) & ~7;
  for (int p = tid; p < padded; p += kSmallThreads) {
    int e = -1, j = 0;
    float a = 1.0f;
    if (p < n_pairs) {
      j = p / kk;
      const int k = p - j * kk;
      if (k < top_k) {
        e = topk_idx[j * top_k + k];
        a = topk_w[j * top_k + k];
        if (e < 0 || e >= n_experts) e = -1;
      } else {
        e = n_experts + k - top_k;
      }
      if (e < 0) slot_of[p] = -1;
    }
    ids[p] = (int16_t)e;
    token[p] = (int16_t)j;
    weight[p] = a;
  }
  __syncthreads();
  const int e = tid / kQuarters, quarter = tid % kQuarters;
  const int groups = padded / 8;
  const int p_begin = groups * quarter / kQuarters * 8, p_end = groups * (quarter + 1) / kQuarters * 8;
  int mine = 0;
  if (e < total) {
    for (int p = p_begin; p < p_end; p += 8) {
      const i16x8 v = *reinterpret_cast<const i16x8*>(&ids[p]);
#pragma unroll
      for (int i = 0; i < 8; ++i) mine += v[i] == e;
    }
  }
  // exclusive prefix of `mine` over the threads: inside the wave by shuffles, then the totals of the waves before
  int incl = mine;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  if (lane == kWave - 1) wave_total[wave] = incl;
  __syncthreads();
  int first = incl - mine;
  for (int w = 0; w < wave; ++w) first += wave_total[w];
  const int first_of_expert = __shfl(first, lane & ~(kQuarters - 1));  // the four threads of an expert are neighbours
  if (e < total) {
    if (quarter == 0) offsets[e] = first;
    if (quarter == kQuarters - 1) {
      counts[e] = first + mine - first_of_expert;
      if (e == total - 1) offsets[total] = first + mine;
    }
    int slot = first;
    for (int p = p_begin; p < p_end; p += 8) {
      const i16x8 v = *reinterpret_cast<const i16x8*>(&ids[p]);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (v[i] != e) continue;
        const int q = p + i;
        perm[slot] = token[q];
        w_perm[slot] = weight[q];
        slot_of[q] = slot;
        ++slot;
      }
    }
  }
}

// The same pairs written out, for the general counting sort: idx_aug / w_aug [n][top_k + n_shared].
__global__ void compact_append_shared_kernel(const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
                                             int64_t n, int top_k, int n_experts, int n_shared,
                                             int32_t* __restrict__ idx_aug, float* __restrict__ w_aug) {
  const int kk = top_k + n_shared;
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= n * kk) return;
  const int64_t j = p / kk;
  const int k = (int)(p - j * kk);
  if (k < top_k) {
    const int e = topk_idx[j * top_k + k];
    idx_aug[p] = (e < 0 || e >= n_experts) ? -1 : e;  // an id of the appended experts is not a routed choice
    w_aug[p] = topk_w[j * top_k + k];
  } else {
    idx_aug[p] = n_experts + k - top_k;
    w_aug[p] = 1.0f;
  }
}

}  // namespace

hipError_t launch_compact_bucket_small(hipStream_t stream, const int32_t* topk_idx, const float* topk_w, int64_t n,
                                       int top_k, int n_experts, int n_shared, const BucketTables& t) {
  compact_bucket_small_kernel<<<1, kSmallThreads, 0, stream>>>(topk_idx, topk_w, (int)n, top_k, n_experts, n_shared,
                                                               t.counts, t.offsets, t.perm, t.w_perm, t.slot_of);
  return hipGetLastError();
}

hipError_t launch_compact_append_shared(hipStream_t stream, const int32_t* topk_idx, const float* topk_w, int64_t n,
                                        int top_k, int n_experts, int n_shared, int32_t* idx_aug, float* w_aug) {
  const int64_t pairs = n * (top_k + n_shared);
  compact_append_shared_kernel<<<(int)((pairs + 255) / 256), 256, 0, stream>>>(topk_idx, topk_w, n, top_k, n_experts,
                                                                                n_shared, idx_aug, w_aug);
  return hipGetLastError();
}

hipError_t launch_compact_hidden(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model, const void* W_gate,
                                 const void* W_up, const CompactRows& tab, const BucketTables& t, int token_groups,
                                 void* hidden, int ldh) {
  const int tiles = tab.tile_off[tab.n_experts];
  if (tiles <= 0) return hipSuccess;
  compact_hidden_kernel<kSplitHidden><<<dim3(tiles, token_groups), kWave * kSplitHidden, 0, stream>>>(
      static_cast<const __bf16*>(X), ldx, (int)d_model, static_cast<const __bf16*>(W_gate),
      static_cast<const __bf16*>(W_up), tab, t.counts, t.offsets, t.perm, t.w_perm, static_cast<__bf16*>(hidden), ldh);
  return hipGetLastError();
}

hipError_t launch_compact_down(hipStream_t stream, const void* hidden, int ldh, const void* W_down, int64_t d_model,
                               const CompactDown& tab, const BucketTables& t, int token_groups, int64_t n_slots,
                               float* partial) {
  const int64_t blocks = (int64_t)tab.chunk_off[tab.n_experts] * ((d_model + kRows - 1) / kRows);
  if (blocks <= 0) return hipSuccess;
  int64_t kept = 0;
  for (int e = 0; e < tab.n_experts; ++e) kept += tab.count[e];
  const dim3 grid((unsigned)blocks, token_groups);
  if (kept >= (int64_t)kDownFourWavesFrom * tab.chunk_off[tab.n_experts])  // mean chunk length
    compact_down_kernel<4><<<grid, kWave * 4, 0, stream>>>(static_cast<const __bf16*>(hidden), ldh,
                                                           static_cast<const __bf16*>(W_down), (int)d_model, tab,
                                                           t.counts, t.offsets, n_slots, partial);
  else
    compact_down_kernel<2><<<grid, kWave * 2, 0, stream>>>(static_cast<const __bf16*>(hidden), ldh,
                                                           static_cast<const __bf16*>(W_down), (int)d_model, tab,
                                                           t.counts, t.offsets, n_slots, partial);
  return hipGetLastError();
}

hipError_t launch_compact_combine(hipStream_t stream, const float* partial, const CompactDown& tab,
                                  const BucketTables& t, int64_t n, int terms, int64_t d_model, int64_t n_slots,
                                  int accumulate, float* Y) {
  const int vecs = (int)(d_model / 4);
  const int64_t threads = n * vecs;
  compact_combine_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, stream>>>(
      reinterpret_cast<const float4*>(partial), t.slot_of, t.offsets, tab, n, terms, vecs, n_slots, accumulate,
      reinterpret_cast<float4*>(Y));
  return hipGetLastError();
}

}  // namespace camera

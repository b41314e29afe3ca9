// The layer output from compacted weights (the result of Algorithm 2, lines
// 10-13: every expert keeps its own number of micro-experts), for the small
// token batches of decoding (the setting of the decoding-speed comparison of a
// pruned MoE layer, batch of 64 tokens).
//
// With a handful of tokens per expert the layer is bound by reading each
// activated expert's weights once, so nothing is tiled through LDS: a wave owns
// 32 weight rows, streams them from HBM straight into MFMA operand registers
// (v_mfma_f32_32x32x16_bf16: the weight rows are the M side, up to 64 tokens of
// the expert the N side) and never shares data with another wave.  Inside a
// 64-element K block lane (row, half) holds the 32 consecutive elements
// [32*half, 32*half + 32) of its row as four 16-byte loads, so the two lanes of
// a row read one full 128-byte line; the token operand uses the same K order,
// which a sum over K does not care about.  Experts that no token of the batch
// selected are skipped before any weight is read.
//
//   hidden  : Lambda[slot][c] = a silu(x w_gate,c) (x w_up,c), bf16, for the c < count[e] kept micro-experts
//   down    : product[slot][r] = sum_c Lambda[slot][c] W_down_e[r][c], float32
// The rows of the compacted W_down block of an expert are count[e] elements
// long, which need not be a multiple of eight: its 16-byte loads are unaligned
// (2-byte aligned), and the ragged end of a row is read element by element.
#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kRows = 32;    // weight rows per wave (the MFMA's M)
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

// The last, partial K block.  `k` is the K index of the lane's first element, `k_full` the end of the valid
// elements, `k_pad` (a multiple of 8, >= k_full) the end of what may be read when PAD_READABLE (an operand whose
// rows are padded with zeros up to k_pad), else elements at and beyond k_full are never touched.
template <bool ALIGNED, bool PAD_READABLE>
__device__ __forceinline__ void load_frag_tail(Frag& f, const __bf16* p, int k, int k_full, int k_pad) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int kj = k + 8 * j;
    if (kj + 8 <= k_full || (PAD_READABLE && kj < k_pad)) {
      f.c[j] = ALIGNED ? load8(p + 8 * j) : load8_unaligned(p + 8 * j);
    } else if (kj < k_full) {
      bf16x8 v = zero8();
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (kj + i < k_full) v[i] = p[8 * j + i];
      f.c[j] = v;
    } else {
      f.c[j] = zero8();
    }
  }
}

__device__ __forceinline__ void mfma4(f32x16& acc, const Frag& a, const Frag& b) {
#pragma unroll
  for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.c[j], b.c[j], acc, 0, 0, 0);
}

// ---- Lambda = a silu(X W_gate^T) (X W_up^T) on the kept rows ----------------------------------------------
// One pass over the K extent for up to 64 tokens (TWO) or up to 32 (not TWO) of one expert.
template <bool TWO>
__device__ __forceinline__ void hidden_pass(const __bf16* __restrict__ wg, const __bf16* __restrict__ wu,
                                            const __bf16* __restrict__ x0, const __bf16* __restrict__ x1, int d_model,
                                            f32x16& g0, f32x16& u0, f32x16& g1, f32x16& u1) {
  const int full = d_model / kKBlock;
  Frag ag[2], au[2], b0[2], b1[2];
  auto fetch = [&](int buf, int kb) {
    const int off = kb * kKBlock;
    load_frag<true>(ag[buf], wg + off);
    load_frag<true>(au[buf], wu + off);
    load_frag<true>(b0[buf], x0 + off);
    if (TWO) load_frag<true>(b1[buf], x1 + off);
  };
  auto multiply = [&](int buf) {
    mfma4(g0, ag[buf], b0[buf]);
    mfma4(u0, au[buf], b0[buf]);
    if (TWO) {
      mfma4(g1, ag[buf], b1[buf]);
      mfma4(u1, au[buf], b1[buf]);
    }
  };
  if (full > 0) fetch(0, 0);
  int kb = 0;
  for (; kb + 2 <= full; kb += 2) {  // the loads of the next block are in flight while this one multiplies
    fetch(1, kb + 1);
    multiply(0);
    if (kb + 2 < full) fetch(0, kb + 2);
    multiply(1);
  }
  if (kb < full) multiply(0);
  const int rem = d_model - full * kKBlock;  // a multiple of 8
  if (rem > 0) {
    const int half_k = (threadIdx.x & 63) >> 5 << 5;  // K index of the lane's first element inside the block
    const int off = full * kKBlock;
    load_frag_tail<true, false>(ag[0], wg + off, half_k, rem, rem);
    load_frag_tail<true, false>(au[0], wu + off, half_k, rem, rem);
    load_frag_tail<true, false>(b0[0], x0 + off, half_k, rem, rem);
    if (TWO) load_frag_tail<true, false>(b1[0], x1 + off, half_k, rem, rem);
    multiply(0);
  }
}

// WIDE: the tokens of an expert are taken 64 at a time (two accumulator tiles), else 32 at a time.
template <bool WIDE>
__global__ __launch_bounds__(kThreads) void compact_hidden_kernel(
    const __bf16* __restrict__ X, int64_t ldx, int d_model, const __bf16* __restrict__ W_gate,
    const __bf16* __restrict__ W_up, CompactTable tab, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm, const float* __restrict__ w_perm,
    __bf16* __restrict__ H, int ldh) {
  const int lane = threadIdx.x & 63;
  const int tile = __builtin_amdgcn_readfirstlane((int)blockIdx.x * kWavesPerBlock + (int)(threadIdx.x >> 6));
  if (tile >= tab.tile_off[tab.n_experts]) return;
  int lo = 0, hi = tab.n_experts;  // tile_off[lo] <= tile < tile_off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tab.tile_off[mid] <= tile) lo = mid; else hi = mid;
  }
  const int e = lo;
  const int m = __builtin_amdgcn_readfirstlane(counts[e]);
  if (m <= 0) return;  // no token of the batch selected this expert: its weights are not read
  const int slot0 = __builtin_amdgcn_readfirstlane(offsets[e]);
  const int cnt = tab.row_off[e + 1] - tab.row_off[e];
  const int cnt8 = (cnt + 7) & ~7;
  const int c0 = (tile - tab.tile_off[e]) * kRows;
  const int r = lane & 31, h = lane >> 5;
  const int row = min(c0 + r, cnt - 1);  // rows past the expert's end repeat its last row; their results are dropped
  const int64_t w_off = ((int64_t)tab.row_off[e] + row) * d_model + h * 32;
  const __bf16* wg = W_gate + w_off;
  const __bf16* wu = W_up + w_off;

  for (int t0 = 0; t0 < m; t0 += WIDE ? 64 : 32) {
    const bool two = WIDE && m - t0 > 32;
    const int ta = min(t0 + r, m - 1), tb = min(t0 + 32 + r, m - 1);  // clamped: columns past m are dropped
    const int64_t tok_a = perm ? perm[slot0 + ta] : ta;
    const int64_t tok_b = perm ? perm[slot0 + tb] : tb;
    const __bf16* x0 = X + tok_a * ldx + h * 32;
    const __bf16* x1 = X + tok_b * ldx + h * 32;
    f32x16 g0 = {}, u0 = {}, g1 = {}, u1 = {};
    if constexpr (WIDE) {
      if (two)
        hidden_pass<true>(wg, wu, x0, x1, d_model, g0, u0, g1, u1);
      else
        hidden_pass<false>(wg, wu, x0, x1, d_model, g0, u0, g1, u1);
    } else {
      hidden_pass<false>(wg, wu, x0, x1, d_model, g0, u0, g1, u1);
    }
    // accumulator element i of a lane: weight row 8*(i/4) + 4*h + i%4, token column r
#pragma unroll
    for (int tile_n = 0; tile_n < 2; ++tile_n) {
      const int t = t0 + 32 * tile_n + r;
      if ((tile_n == 1 && !two) || t >= m) continue;
      const int64_t slot = slot0 + t;
      const float a = w_perm ? w_perm[slot] : 1.0f;
      const f32x16& g = tile_n ? g1 : g0;
      const f32x16& u = tile_n ? u1 : u0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = c0 + 8 * q + 4 * h;
        if (c >= cnt8) continue;  // columns [cnt, cnt8) are written as zeros: the down kernel reads whole chunks
        bf16x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float lam = a * silu_f32(g[4 * q + i]) * u[4 * q + i];
          out[i] = (__bf16)(c + i < cnt ? lam : 0.0f);
        }
        *reinterpret_cast<bf16x4*>(H + slot * ldh + c) = out;
      }
    }
  }
}

// ---- product = Lambda W_down_e^T ---------------------------------------------------------------------------
template <bool TWO>
__device__ __forceinline__ void down_pass(const __bf16* __restrict__ wd, const __bf16* __restrict__ h0,
                                          const __bf16* __restrict__ h1, int cnt, int cnt8, f32x16& p0, f32x16& p1) {
  const int full = cnt / kKBlock;
  Frag a[2], b0[2], b1[2];
  auto fetch = [&](int buf, int kb) {
    const int off = kb * kKBlock;
    load_frag<false>(a[buf], wd + off);
    load_frag<true>(b0[buf], h0 + off);
    if (TWO) load_frag<true>(b1[buf], h1 + off);
  };
  auto multiply = [&](int buf) {
    mfma4(p0, a[buf], b0[buf]);
    if (TWO) mfma4(p1, a[buf], b1[buf]);
  };
  if (full > 0) fetch(0, 0);
  int kb = 0;
  for (; kb + 2 <= full; kb += 2) {
    fetch(1, kb + 1);
    multiply(0);
    if (kb + 2 < full) fetch(0, kb + 2);
    multiply(1);
  }
  if (kb < full) multiply(0);
  const int rem = cnt - full * kKBlock;
  if (rem > 0) {
    const int half_k = (threadIdx.x & 63) >> 5 << 5;
    const int off = full * kKBlock;
    const int rem8 = cnt8 - off;
    load_frag_tail<false, false>(a[0], wd + off, half_k, rem, rem8);  // never past the end of the weight row
    load_frag_tail<true, true>(b0[0], h0 + off, half_k, rem, rem8);   // Lambda rows are zero-filled up to cnt8
    if (TWO) load_frag_tail<true, true>(b1[0], h1 + off, half_k, rem, rem8);
    multiply(0);
  }
}

template <bool WIDE>
__global__ __launch_bounds__(kThreads) void compact_down_kernel(const __bf16* __restrict__ H, int ldh,
                                                                const __bf16* __restrict__ W_down, int d_model,
                                                                CompactTable tab, const int32_t* __restrict__ counts,
                                                                const int32_t* __restrict__ offsets,
                                                                float* __restrict__ product) {
  const int lane = threadIdx.x & 63;
  const int row_tiles = (d_model + kRows - 1) / kRows;
  const int tile = __builtin_amdgcn_readfirstlane((int)blockIdx.x * kWavesPerBlock + (int)(threadIdx.x >> 6));
  if (tile >= tab.n_experts * row_tiles) return;
  const int e = tile / row_tiles;
  const int r0 = (tile - e * row_tiles) * kRows;
  const int m = __builtin_amdgcn_readfirstlane(counts[e]);
  if (m <= 0) return;
  const int slot0 = __builtin_amdgcn_readfirstlane(offsets[e]);
  const int cnt = tab.row_off[e + 1] - tab.row_off[e];  // 0: the product rows of this expert's tokens are zero
  const int cnt8 = (cnt + 7) & ~7;
  const int r = lane & 31, h = lane >> 5;
  const int row = min(r0 + r, d_model - 1);
  const __bf16* wd = W_down + (int64_t)tab.row_off[e] * d_model + (int64_t)row * cnt + h * 32;

  for (int t0 = 0; t0 < m; t0 += WIDE ? 64 : 32) {
    const bool two = WIDE && m - t0 > 32;
    const int ta = min(t0 + r, m - 1), tb = min(t0 + 32 + r, m - 1);
    const __bf16* h0 = H + (int64_t)(slot0 + ta) * ldh + h * 32;
    const __bf16* h1 = H + (int64_t)(slot0 + tb) * ldh + h * 32;
    f32x16 p0 = {}, p1 = {};
    if constexpr (WIDE) {
      if (two)
        down_pass<true>(wd, h0, h1, cnt, cnt8, p0, p1);
      else
        down_pass<false>(wd, h0, h1, cnt, cnt8, p0, p1);
    } else {
      down_pass<false>(wd, h0, h1, cnt, cnt8, p0, p1);
    }
#pragma unroll
    for (int tile_n = 0; tile_n < 2; ++tile_n) {
      const int t = t0 + 32 * tile_n + r;
      if ((tile_n == 1 && !two) || t >= m) continue;
      const f32x16& p = tile_n ? p1 : p0;
      float* out = product + (int64_t)(slot0 + t) * d_model;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int rr = r0 + 8 * q + 4 * h;
        if (rr >= d_model) continue;  // d_model is a multiple of 8: a group of four is inside or outside as a whole
        *reinterpret_cast<float4*>(out + rr) = make_float4(p[4 * q], p[4 * q + 1], p[4 * q + 2], p[4 * q + 3]);
      }
    }
  }
}

}  // namespace

hipError_t launch_compact_hidden(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model, const void* W_gate,
                                 const void* W_up, const CompactTable& tab, const BucketTables& t, void* hidden,
                                 int ldh, bool wide) {
  const int tiles = tab.tile_off[tab.n_experts];
  if (tiles <= 0) return hipSuccess;
  const int blocks = (tiles + kWavesPerBlock - 1) / kWavesPerBlock;
  auto kernel = wide ? compact_hidden_kernel<true> : compact_hidden_kernel<false>;
  kernel<<<blocks, kThreads, 0, stream>>>(static_cast<const __bf16*>(X), ldx, (int)d_model,
                                          static_cast<const __bf16*>(W_gate), static_cast<const __bf16*>(W_up), tab,
                                          t.counts, t.offsets, t.perm, t.w_perm, static_cast<__bf16*>(hidden), ldh);
  return hipGetLastError();
}

hipError_t launch_compact_down(hipStream_t stream, const void* hidden, int ldh, const void* W_down, int64_t d_model,
                               const CompactTable& tab, const BucketTables& t, float* product, bool wide) {
  const int64_t tiles = (int64_t)tab.n_experts * ((d_model + kRows - 1) / kRows);
  const int blocks = (int)((tiles + kWavesPerBlock - 1) / kWavesPerBlock);
  auto kernel = wide ? compact_down_kernel<true> : compact_down_kernel<false>;
  kernel<<<blocks, kThreads, 0, stream>>>(static_cast<const __bf16*>(hidden), ldh, static_cast<const __bf16*>(W_down),
                                          (int)d_model, tab, t.counts, t.offsets, product);
  return hipGetLastError();
}

}  // namespace camera

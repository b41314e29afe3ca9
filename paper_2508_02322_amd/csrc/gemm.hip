// Grouped gate/up contraction with the fused CAMERA epilogue.
//
// For every expert e and its routed tokens j (Algorithm 1, line 6; Eq. 1, 4):
//   G[j,c] = <x_j, w_gate_c>,  U[j,c] = <x_j, w_up_c>
//   Lambda[j,c] = a_j * silu(G[j,c]) * U[j,c]
// and per channel c the two column statistics of lines 7-8,
//   sum_j Lambda^2  and  max_j Lambda^2  ( = (max_j |Lambda|)^2 ).
// Lambda never leaves the registers.  A workgroup owns one (M-tile of tokens,
// N-tile of channels) of one expert and writes that tile's column statistics
// to part_phi2 / part_max [m_tile_slot][channel]; the finalize kernel adds the
// M-tiles of an expert in slot order, so the result is independent of launch
// order and uses no floating-point atomics.
//
// bf16: v_mfma_f32_32x32x16_bf16 (64-wide wavefront, fp32 accumulate).  Token
// rows (A operand, gathered through the bucket permutation) and weight rows (B
// operand) are both K-contiguous, so both fragments are 16-byte LDS reads; the
// LDS tiles are [row][8 chunks of 8 bf16] with the chunk index XOR-ed by
// ((row >> 1) & 7): the LDS has 64 four-byte banks, so two 128-byte tile rows
// fill one bank row and 16 consecutive rows reading the same K chunk (one
// quarter of a fragment read) then hit 16 different 16-byte bank groups.
// fp32: plain FMA tiles (used by the float32 configuration only).
#include <hip/hip_bf16.h>

#include <type_traits>

#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// silu(g) = g / (1 + exp(-g)); exp2 and rcp are single hardware instructions (about 1 ulp each)
__device__ __forceinline__ float silu_f32(float g) {
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.
//   A workgroup is WM x WN waves.  A wave owns TM 32-row blocks of tokens
//   (blocks wave_m, wave_m + WM, ... of the tile, so that a short last tile of an
//   expert is shared evenly and its empty blocks are skipped) by TN*32 channels,
//   for both the gate and the up product.  Block tile BM = 32*WM*TM tokens by
//   BN = 32*WN*TN channels; K advances KT = 64 elements per LDS stage, two
//   stages.  Schedule per K tile: global loads of the tile after next are issued
//   first (two register staging sets), the four 16-wide K steps run MFMAs on one
//   fragment set while the next set is read from LDS, the next tile is written
//   to the other stage, and the workgroup barrier sits before the last K step so
//   that the first fragments of the next tile are in flight while that step's
//   MFMAs run.
// ---------------------------------------------------------------------------
constexpr int KT = 64;
constexpr int kChunks = KT / 8;  // 16-byte chunks per tile row: one 128-byte LDS row
constexpr int kXcds = 8;         // accelerator dies, each with a private L2
constexpr int kPatchM = 4;       // M-tile slots per patch
constexpr int kPatchN = 8;       // N-tiles per patch

enum Sched { kSchedNone = 0, kSchedPhases = 1 };

template <int WM_, int WN_, int TM_, int TN_, int SCHED_>
struct GemmCfg {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_, SCHED = SCHED_;
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int BM = 32 * WM * TM;
  static constexpr int BN = 32 * WN * TN;
  static constexpr int kATileBytes = BM * KT * 2;
  static constexpr int kBTileBytes = BN * KT * 2;  // one of gate / up
  static constexpr int kStageBytes = kATileBytes + 2 * kBTileBytes;
  static constexpr int kRowsPerPass = kThreads / kChunks;  // tile rows one staging pass of the block covers
  static constexpr int kARows = BM / kRowsPerPass;         // 16-byte chunks of the A tile per thread
  static constexpr int kBRows = BN / kRowsPerPass;         // per matrix
  static constexpr int kSmemBytes = 2 * kStageBytes + BM * 8 + 2 * WM * BN * 4;
  static_assert(kRowsPerPass % 16 == 0 && BM % kRowsPerPass == 0 && BN % kRowsPerPass == 0, "staging shape");
};

// Everything a workgroup needs after its set-up, so that the K loop can be instantiated
// once per number of active row blocks (ACT) without run-time branches inside it.
template <class C>
struct TileState {
  unsigned char* smem;
  const float* s_a;
  float* s_red;
  // staging (global -> registers -> LDS)
  const __hip_bfloat16* a_src[C::kARows];
  const __hip_bfloat16* wg_src[C::kBRows];
  const __hip_bfloat16* wu_src[C::kBRows];
  int st_dst;  // byte offset of this thread's chunk in a tile (+ kRowsPerPass * 128 per further row)
  int st_k;    // first K element of this thread's chunk inside a K tile
  int d_model;
  // fragments
  int a_frag_base, b_frag_base;
  int k_swz[KT / 16];
  int wave_m, wave_n, frag_row, frag_half;
};

template <class C, int ACT, bool TAIL>
__device__ __forceinline__ void tile_body(const TileState<C>& st, int n0, int d_ff, int slot,
                                          float* __restrict__ part_phi2, float* __restrict__ part_max) {
  constexpr int BN = C::BN, TN = C::TN, WM = C::WM;
  constexpr int NA = ACT > 0 ? ACT : 1;
  constexpr int kPassBytes = C::kRowsPerPass * 128;
  unsigned char* const smem = st.smem;

  // Two register staging sets: tile kt+2 is on its way from HBM / L2 while tile kt+1 waits in the
  // other set to be written to LDS, so a load has two K tiles of MFMA time to arrive.
  struct Staging {
    u32x4 a[C::kARows], g[C::kBRows], u[C::kBRows];
  };
  // TAIL (d_model not a multiple of KT): chunks past d_model read as zero.  Without it no load is conditional.
  auto ld = [&](const __hip_bfloat16* p, int k0) -> u32x4 {
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    if constexpr (TAIL) return (k0 + st.st_k < st.d_model) ? *reinterpret_cast<const u32x4*>(p + k0) : zero4;
    else return *reinterpret_cast<const u32x4*>(p + k0);
  };
  auto load_global = [&](Staging& r, int k0) {
#pragma unroll
    for (int i = 0; i < C::kARows; ++i) r.a[i] = ld(st.a_src[i], k0);
#pragma unroll
    for (int i = 0; i < C::kBRows; ++i) {
      r.g[i] = ld(st.wg_src[i], k0);
      r.u[i] = ld(st.wu_src[i], k0);
    }
  };
  auto store_lds = [&](const Staging& r, int buf) {
    unsigned char* sA = smem + buf * C::kStageBytes + st.st_dst;
    unsigned char* sG = sA + C::kATileBytes;
    unsigned char* sU = sG + C::kBTileBytes;
#pragma unroll
    for (int i = 0; i < C::kARows; ++i) *reinterpret_cast<u32x4*>(sA + i * kPassBytes) = r.a[i];
#pragma unroll
    for (int i = 0; i < C::kBRows; ++i) {
      *reinterpret_cast<u32x4*>(sG + i * kPassBytes) = r.g[i];
      *reinterpret_cast<u32x4*>(sU + i * kPassBytes) = r.u[i];
    }
  };

  f32x16 acc_g[NA][TN], acc_u[NA][TN];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc_g[i][j][r] = 0.0f;
        acc_u[i][j][r] = 0.0f;
      }

  struct Frags {
    bf16x8 a[NA], g[TN], u[TN];
  };
  auto read_frags = [&](Frags& f, int buf, int ks) {
    if constexpr (ACT > 0) {
      const unsigned char* sA = smem + buf * C::kStageBytes + st.k_swz[ks];
      const unsigned char* sG = sA + C::kATileBytes + st.b_frag_base;
      const unsigned char* sU = sG + C::kBTileBytes;
#pragma unroll
      for (int i = 0; i < ACT; ++i)
        f.a[i] = *reinterpret_cast<const bf16x8*>(sA + st.a_frag_base + i * WM * 32 * 128);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        f.g[j] = *reinterpret_cast<const bf16x8*>(sG + j * 32 * 128);
        f.u[j] = *reinterpret_cast<const bf16x8*>(sU + j * 32 * 128);
      }
    }
  };
  auto mfma_step = [&](const Frags& f) {
#pragma unroll
    for (int i = 0; i < ACT; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        acc_g[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.g[j], acc_g[i][j], 0, 0, 0);
        acc_u[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.u[j], acc_u[i][j], 0, 0, 0);
      }
  };
  auto pin = [&]() {
    // keeps the compiler from sinking the global loads down to their LDS stores (which exposes
    // the memory latency every tile) and from folding the two fragment sets into one
    if constexpr (C::SCHED == kSchedPhases) __builtin_amdgcn_sched_barrier(0);
  };

  // One loop body for every K tile: tiles past the end are clamped to the last one (two redundant
  // tile loads per workgroup) instead of branching around the prefetch.
  const int n_k = (st.d_model + KT - 1) / KT;
  const int k_last = (n_k - 1) * KT;
  Frags f0, f1;
  Staging r0, r1;
  auto k_tile = [&](int kt, Staging& r_load, const Staging& r_store) {
    const int buf = kt & 1;
    load_global(r_load, min((kt + 2) * KT, k_last));  // tile kt + 2
    read_frags(f1, buf, 1);
    pin();
    mfma_step(f0);
    read_frags(f0, buf, 2);
    pin();
    mfma_step(f1);
    read_frags(f1, buf, 3);
    pin();
    mfma_step(f0);
    store_lds(r_store, buf ^ 1);  // tile kt + 1, loaded one iteration ago
    __syncthreads();              // the next stage is complete; every read of this stage has returned
    read_frags(f0, buf ^ 1, 0);
    pin();
    mfma_step(f1);
    pin();
  };
  load_global(r0, 0);
  load_global(r1, min(KT, k_last));
  store_lds(r0, 0);
  __syncthreads();
  read_frags(f0, 0, 0);
  int kt = 0;
  for (; kt + 1 < n_k; kt += 2) {
    k_tile(kt, r0, r1);
    k_tile(kt + 1, r1, r0);
  }
  if (kt < n_k) k_tile(kt, r0, r1);

  // Epilogue.  Accumulator register r of lane l is output row 8*(r/4) + 4*(l/32) + (r%4),
  // column l % 32 of its 32x32 tile: a lane owns one channel and 16 token rows per tile.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    float sum = 0.0f, mx = 0.0f;
#pragma unroll
    for (int i = 0; i < ACT; ++i) {
      const int band = (WM * i + st.wave_m) * 32 + st.frag_half * 4;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = band + (r / 4) * 8 + (r % 4);
        const float lam = st.s_a[row] * silu_f32(acc_g[i][j][r]) * acc_u[i][j][r];
        const float l2 = lam * lam;
        sum += l2;
        mx = fmaxf(mx, l2);
      }
    }
    sum += __shfl_xor(sum, 32);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (st.frag_half == 0) {
      const int col = st.wave_n * TN * 32 + j * 32 + st.frag_row;
      st.s_red[st.wave_m * BN + col] = sum;
      st.s_red[(WM + st.wave_m) * BN + col] = mx;
    }
  }
  __syncthreads();
  for (int col = threadIdx.x; col < BN; col += C::kThreads) {
    if (n0 + col < d_ff) {
      float sum = 0.0f, mx = 0.0f;
#pragma unroll
      for (int w = 0; w < WM; ++w) {  // fixed order
        sum += st.s_red[w * BN + col];
        mx = fmaxf(mx, st.s_red[(WM + w) * BN + col]);
      }
      part_phi2[(int64_t)slot * d_ff + n0 + col] = sum;
      part_max[(int64_t)slot * d_ff + n0 + col] = mx;
    }
  }
}

template <class C, bool TAIL>
__global__ __launch_bounds__(C::kThreads) void grouped_gemm_bf16_kernel(
    const __hip_bfloat16* __restrict__ X, int64_t ldx, int d_model, int d_ff,
    const __hip_bfloat16* __restrict__ Wg, const __hip_bfloat16* __restrict__ Wu, int64_t stride_gu,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tile_offset,
    const int32_t* __restrict__ tile_expert, const int32_t* __restrict__ perm, const float* __restrict__ w_perm,
    int n_experts, float* __restrict__ part_phi2, float* __restrict__ part_max) {
  constexpr int BM = C::BM, BN = C::BN, TM = C::TM, TN = C::TN, WM = C::WM;
  // Workgroup -> tile mapping.  The hardware deals consecutive workgroup ids round-robin to the 8
  // XCDs, each with its own L2.  Give every XCD a contiguous run of logical ids, and order logical
  // ids in patches of kPatchM M-tile slots x kPatchN N-tiles (= the 32 workgroups an XCD runs at a
  // time): a patch re-reads only kPatchM token tiles and kPatchN weight tiles through its L2.
  const int per_xcd = gridDim.x / kXcds;
  const int logical = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
  const int patch = logical / (kPatchM * kPatchN), in_patch = logical % (kPatchM * kPatchN);
  const int n_tiles_n = (d_ff + BN - 1) / BN;
  const int patches_n = (n_tiles_n + kPatchN - 1) / kPatchN;
  const int slot = (patch / patches_n) * kPatchM + in_patch % kPatchM;
  const int tile_n = (patch % patches_n) * kPatchN + in_patch / kPatchM;
  if (tile_n >= n_tiles_n || slot >= tile_offset[n_experts]) return;  // block-uniform: nothing here
  const int e = tile_expert[slot];
  const int tile_in_expert = slot - tile_offset[e];
  const int row_first = offsets[e] + tile_in_expert * BM;  // first bucket slot of this tile
  const int m_len = min(BM, offsets[e + 1] - row_first);   // >= 1
  const int n0 = tile_n * BN;

  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_tok = reinterpret_cast<int32_t*>(smem + 2 * C::kStageBytes);  // [BM] token id
  float* s_a = reinterpret_cast<float*>(s_tok + BM);                       // [BM] routing weight
  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;

  // Rows past the end of the expert's bucket read token row 0 of the tile again with weight 0:
  // their Lambda is exactly 0 (finite projections times a = 0), so no load in the K loop is conditional.
  for (int r = tid; r < BM; r += C::kThreads) {
    const int rr = r < m_len ? r : 0;
    s_tok[r] = perm ? perm[row_first + rr] : tile_in_expert * BM + rr;
    s_a[r] = r < m_len ? (w_perm ? w_perm[row_first + rr] : 1.0f) : 0.0f;
  }
  __syncthreads();

  TileState<C> st;
  st.smem = smem;
  st.s_a = s_a;
  st.s_red = s_a + BM;  // [2 stats][WM][BN]
  st.d_model = d_model;
  st.wave_m = wave % WM;
  st.wave_n = wave / WM;
  st.frag_row = lane % 32;
  st.frag_half = lane / 32;
  // Staging: thread t moves 16-byte chunk (t % 8) of tile rows t/8, t/8 + kRowsPerPass, ...
  const int st_row = tid / kChunks, st_ck = tid % kChunks;
  st.st_dst = st_row * 128 + ((st_ck ^ ((st_row >> 1) & 7)) << 4);  // the swizzle key repeats every 16 rows
  st.st_k = st_ck * 8;
#pragma unroll
  for (int i = 0; i < C::kARows; ++i)
    st.a_src[i] = X + (int64_t)s_tok[st_row + C::kRowsPerPass * i] * ldx + st_ck * 8;
#pragma unroll
  for (int i = 0; i < C::kBRows; ++i) {
    // channels past d_ff read the last channel again; their statistics are never written
    const int c = min(n0 + st_row + C::kRowsPerPass * i, d_ff - 1);
    const int64_t off = (int64_t)e * stride_gu + (int64_t)c * d_model + st_ck * 8;
    st.wg_src[i] = Wg + off;
    st.wu_src[i] = Wu + off;
  }
  // Fragments: lane l holds tile row (l % 32), K elements 8*(l / 32) .. +7 of a 16-wide K step.
  st.a_frag_base = (st.wave_m * 32 + st.frag_row) * 128;       // + i * WM * 32 * 128: row block WM*i + wave_m
  st.b_frag_base = (st.wave_n * TN * 32 + st.frag_row) * 128;  // + j * 32 * 128
#pragma unroll
  for (int ks = 0; ks < KT / 16; ++ks) st.k_swz[ks] = ((ks * 2 + st.frag_half) ^ ((st.frag_row >> 1) & 7)) << 4;

  // accumulator i of this wave covers row block WM*i + wave_m; blocks past m_len are skipped
  const int n_row_blocks = (m_len + 31) / 32;
  const int act = max(0, (n_row_blocks - st.wave_m + WM - 1) / WM);  // wave-uniform, 0 .. TM
  static_assert(TM == 4 || TM == 2 || TM == 1, "dispatch below covers TM = 1, 2 and 4");
  if (act >= TM) tile_body<C, TM, TAIL>(st, n0, d_ff, slot, part_phi2, part_max);
  else if (act == 3) tile_body<C, (TM > 3 ? 3 : 0), TAIL>(st, n0, d_ff, slot, part_phi2, part_max);
  else if (act == 2) tile_body<C, (TM > 2 ? 2 : 0), TAIL>(st, n0, d_ff, slot, part_phi2, part_max);
  else if (act == 1) tile_body<C, (TM > 1 ? 1 : 0), TAIL>(st, n0, d_ff, slot, part_phi2, part_max);
  else tile_body<C, 0, TAIL>(st, n0, d_ff, slot, part_phi2, part_max);
}

// ---------------------------------------------------------------------------
// fp32 FMA kernel: 64 tokens x 64 channels per block of 256 threads, K step 16,
// each thread 4 rows x 4 channels of gate and of up.
// ---------------------------------------------------------------------------
constexpr int F32_BM = 64, F32_BN = 64, F32_KT = 16;

__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(
    const float* __restrict__ X, int64_t ldx, int d_model, int d_ff, const float* __restrict__ Wg,
    const float* __restrict__ Wu, int64_t stride_gu, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ tile_offset, const int32_t* __restrict__ tile_expert,
    const int32_t* __restrict__ perm, const float* __restrict__ w_perm, int n_experts,
    float* __restrict__ part_phi2, float* __restrict__ part_max) {
  const int slot = blockIdx.y;
  if (slot >= tile_offset[n_experts]) return;
  const int e = tile_expert[slot];
  const int tile_in_expert = slot - tile_offset[e];
  const int row_first = offsets[e] + tile_in_expert * F32_BM;
  const int m_len = min(F32_BM, offsets[e + 1] - row_first);
  const int n0 = blockIdx.x * F32_BN;

  __shared__ float sX[F32_KT][F32_BM + 4];
  __shared__ float sG[F32_KT][F32_BN + 4];
  __shared__ float sU[F32_KT][F32_BN + 4];
  __shared__ int32_t s_tok[F32_BM];
  __shared__ float s_a[F32_BM];
  __shared__ float s_red[2][16][F32_BN];

  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  for (int r = tid; r < F32_BM; r += 256) {
    int tok = -1;
    float a = 0.0f;
    if (r < m_len) {
      tok = perm ? perm[row_first + r] : tile_in_expert * F32_BM + r;
      a = w_perm ? w_perm[row_first + r] : 1.0f;
    }
    s_tok[r] = tok;
    s_a[r] = a;
  }
  __syncthreads();

  // loader: thread -> (row = tid / 4, 4 consecutive K at (tid % 4) * 4)
  const int lrow = tid / 4, lk = (tid % 4) * 4;
  const int ltok = s_tok[lrow];
  const float* x_src = ltok >= 0 ? X + (int64_t)ltok * ldx + lk : nullptr;
  const int lc = n0 + lrow;
  const int64_t w_off = (int64_t)e * stride_gu + (int64_t)lc * d_model + lk;
  const float* g_src = lc < d_ff ? Wg + w_off : nullptr;
  const float* u_src = lc < d_ff ? Wu + w_off : nullptr;

  float acc_g[4][4] = {}, acc_u[4][4] = {};
  for (int k0 = 0; k0 < d_model; k0 += F32_KT) {
    const bool k_ok = k0 + lk < d_model;  // d_model is a multiple of 4
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 xv = (x_src && k_ok) ? *reinterpret_cast<const float4*>(x_src + k0) : z;
    const float4 gv = (g_src && k_ok) ? *reinterpret_cast<const float4*>(g_src + k0) : z;
    const float4 uv = (u_src && k_ok) ? *reinterpret_cast<const float4*>(u_src + k0) : z;
    __syncthreads();
    sX[lk + 0][lrow] = xv.x; sX[lk + 1][lrow] = xv.y; sX[lk + 2][lrow] = xv.z; sX[lk + 3][lrow] = xv.w;
    sG[lk + 0][lrow] = gv.x; sG[lk + 1][lrow] = gv.y; sG[lk + 2][lrow] = gv.z; sG[lk + 3][lrow] = gv.w;
    sU[lk + 0][lrow] = uv.x; sU[lk + 1][lrow] = uv.y; sU[lk + 2][lrow] = uv.z; sU[lk + 3][lrow] = uv.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < F32_KT; ++k) {
      float xr[4], gr[4], ur[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xr[i] = sX[k][ty * 4 + i];
        gr[i] = sG[k][tx * 4 + i];
        ur[i] = sU[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc_g[i][j] = fmaf(xr[i], gr[j], acc_g[i][j]);
          acc_u[i][j] = fmaf(xr[i], ur[j], acc_u[i][j]);
        }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float sum = 0.0f, mx = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lam = s_a[ty * 4 + i] * silu_f32(acc_g[i][j]) * acc_u[i][j];
      sum += lam * lam;
      mx = fmaxf(mx, lam * lam);
    }
    s_red[0][ty][tx * 4 + j] = sum;
    s_red[1][ty][tx * 4 + j] = mx;
  }
  __syncthreads();
  if (tid < F32_BN && n0 + tid < d_ff) {
    float sum = 0.0f, mx = 0.0f;
    for (int r = 0; r < 16; ++r) {  // fixed order
      sum += s_red[0][r][tid];
      mx = fmaxf(mx, s_red[1][r][tid]);
    }
    part_phi2[(int64_t)slot * d_ff + n0 + tid] = sum;
    part_max[(int64_t)slot * d_ff + n0 + tid] = mx;
  }
}

// Tile shape of the bf16 kernel (token rows x channels per workgroup, waves, schedule).
#ifndef CAMERA_GEMM_CFG
#define CAMERA_GEMM_CFG 4, 2, 2, 2, kSchedNone
#endif
using Bf16Cfg = GemmCfg<CAMERA_GEMM_CFG>;

}  // namespace

int gemm_tile_m(int dtype, int64_t d_ff) {
  (void)d_ff;
  return dtype == CAMERA_BF16 ? Bf16Cfg::BM : F32_BM;
}

hipError_t launch_grouped_gemm(hipStream_t stream, int dtype, const void* X, int64_t ldx, int64_t d_model,
                               int64_t d_ff, int n_experts, const void* W_gate, const void* W_up,
                               int64_t stride_gu, int max_tiles, const BucketTables& t, float* part_phi2,
                               float* part_max) {
  if (max_tiles <= 0) return hipSuccess;
  if (dtype == CAMERA_BF16) {
    using C = Bf16Cfg;
    const bool tail = d_model % KT != 0;
    auto kern = tail ? grouped_gemm_bf16_kernel<C, true> : grouped_gemm_bf16_kernel<C, false>;
    static bool attr_set[2] = {false, false};
    if (!attr_set[tail]) {
      hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kSmemBytes);
      if (err != hipSuccess) return err;
      attr_set[tail] = true;
    }
    const int64_t patches_n = ((d_ff + C::BN - 1) / C::BN + kPatchN - 1) / kPatchN;
    const int64_t patches_m = (max_tiles + kPatchM - 1) / kPatchM;
    const int64_t n_blocks = (patches_n * patches_m * kPatchM * kPatchN + kXcds - 1) / kXcds * kXcds;
    if (n_blocks >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    dim3 grid((unsigned)n_blocks);
    hipLaunchKernelGGL(kern, grid, dim3(C::kThreads), C::kSmemBytes, stream,
                       static_cast<const __hip_bfloat16*>(X), ldx, (int)d_model, (int)d_ff,
                       static_cast<const __hip_bfloat16*>(W_gate), static_cast<const __hip_bfloat16*>(W_up),
                       stride_gu, t.offsets, t.tile_offset, t.tile_expert, t.perm, t.w_perm, n_experts, part_phi2,
                       part_max);
  } else {
    dim3 grid((unsigned)((d_ff + F32_BN - 1) / F32_BN), (unsigned)max_tiles);
    hipLaunchKernelGGL(grouped_gemm_f32_kernel, grid, dim3(256), 0, stream, static_cast<const float*>(X), ldx,
                       (int)d_model, (int)d_ff, static_cast<const float*>(W_gate), static_cast<const float*>(W_up),
                       stride_gu, t.offsets, t.tile_offset, t.tile_expert, t.perm, t.w_perm, n_experts, part_phi2,
                       part_max);
  }
  return hipGetLastError();
}

}  // namespace camera

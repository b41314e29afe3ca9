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
// (row & 7), which spreads the rows a fragment read touches over all banks.
// fp32: plain FMA tiles (used by the float32 configuration only).
#include <hip/hip_bf16.h>

#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ float silu_f32(float g) { return g / (1.0f + __expf(-g)); }

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.
//   block = WM x WN waves; a wave owns (TM*32 tokens) x (TN*32 channels) of
//   both the gate and the up product; block tile BM = WM*TM*32 tokens by
//   BN = WN*TN*32 channels; K advances KT = 64 elements per stage.
// ---------------------------------------------------------------------------
constexpr int KT = 64;
constexpr int kChunks = KT / 8;  // 16-byte chunks per tile row: one 128-byte LDS row

template <int WM_, int WN_, int TM_, int TN_>
struct GemmCfg {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
  static constexpr int kWaves = WM * WN;
  static constexpr int kThreads = kWaves * kWave;
  static constexpr int BM = WM * TM * 32;
  static constexpr int BN = WN * TN * 32;
  static constexpr int kATileBytes = BM * KT * 2;
  static constexpr int kBTileBytes = BN * KT * 2;  // one of gate / up
  static constexpr int kStageBytes = kATileBytes + 2 * kBTileBytes;
  static constexpr int kAChunksPerThread = BM * kChunks / kThreads;
  static constexpr int kBChunksPerThread = BN * kChunks / kThreads;  // per matrix
  static constexpr int kSmemBytes = 2 * kStageBytes + BM * 8 + 2 * WM * BN * 4;
  static_assert((BM * kChunks) % kThreads == 0 && (BN * kChunks) % kThreads == 0, "whole chunks per thread");
};

__device__ __forceinline__ int swizzled(int row, int chunk) {
  // byte offset of 16-byte chunk `chunk` of tile row `row` (rows are 128 bytes)
  return row * 128 + ((chunk ^ (row & 7)) << 4);
}

template <class C>
__global__ __launch_bounds__(C::kThreads) void grouped_gemm_bf16_kernel(
    const __hip_bfloat16* __restrict__ X, int64_t ldx, int d_model, int d_ff,
    const __hip_bfloat16* __restrict__ Wg, const __hip_bfloat16* __restrict__ Wu, int64_t stride_gu,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tile_offset,
    const int32_t* __restrict__ tile_expert, const int32_t* __restrict__ perm, const float* __restrict__ w_perm,
    int n_experts, float* __restrict__ part_phi2, float* __restrict__ part_max) {
  constexpr int BM = C::BM, BN = C::BN, TM = C::TM, TN = C::TN, WM = C::WM;
  const int slot = blockIdx.y;
  if (slot >= tile_offset[n_experts]) return;  // block-uniform: unused M-tile slot
  const int e = tile_expert[slot];
  const int tile_in_expert = slot - tile_offset[e];
  const int row_first = offsets[e] + tile_in_expert * BM;  // first bucket slot of this tile
  const int m_len = min(BM, offsets[e + 1] - row_first);
  const int n0 = blockIdx.x * BN;

  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_tok = reinterpret_cast<int32_t*>(smem + 2 * C::kStageBytes);  // [BM] token id or -1
  float* s_a = reinterpret_cast<float*>(s_tok + BM);                       // [BM] routing weight
  float* s_red = s_a + BM;                                                 // [2][WM][BN]

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;
  const int wave_m = wave % WM;  // which TM*32-row band of the block tile
  const int wave_n = wave / WM;  // which TN*32-channel band

  for (int r = tid; r < BM; r += C::kThreads) {
    int tok = -1;
    float a = 0.0f;
    if (r < m_len) {
      tok = perm ? perm[row_first + r] : tile_in_expert * BM + r;
      a = w_perm ? w_perm[row_first + r] : 1.0f;
    }
    s_tok[r] = tok;
    s_a[r] = a;
  }
  __syncthreads();

  // Global -> register staging: this thread's chunks of the A tile and of the two B tiles.
  const __hip_bfloat16* a_src[C::kAChunksPerThread];
  int a_dst[C::kAChunksPerThread];
  int a_k[C::kAChunksPerThread];
#pragma unroll
  for (int i = 0; i < C::kAChunksPerThread; ++i) {
    const int q = tid + i * C::kThreads;
    const int row = q / kChunks, ck = q % kChunks;
    const int tok = s_tok[row];
    a_src[i] = tok >= 0 ? X + (int64_t)tok * ldx + ck * 8 : nullptr;
    a_dst[i] = swizzled(row, ck);
    a_k[i] = ck * 8;
  }
  const __hip_bfloat16* bg_src[C::kBChunksPerThread];
  const __hip_bfloat16* bu_src[C::kBChunksPerThread];
  int b_dst[C::kBChunksPerThread];
  int b_k[C::kBChunksPerThread];
#pragma unroll
  for (int i = 0; i < C::kBChunksPerThread; ++i) {
    const int q = tid + i * C::kThreads;
    const int row = q / kChunks, ck = q % kChunks;
    const int c = n0 + row;
    const int64_t off = (int64_t)e * stride_gu + (int64_t)c * d_model + ck * 8;
    bg_src[i] = c < d_ff ? Wg + off : nullptr;
    bu_src[i] = c < d_ff ? Wu + off : nullptr;
    b_dst[i] = swizzled(row, ck);
    b_k[i] = ck * 8;
  }

  u32x4 a_reg[C::kAChunksPerThread], bg_reg[C::kBChunksPerThread], bu_reg[C::kBChunksPerThread];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < C::kAChunksPerThread; ++i)
      a_reg[i] = (a_src[i] && k0 + a_k[i] < d_model) ? *reinterpret_cast<const u32x4*>(a_src[i] + k0) : zero4;
#pragma unroll
    for (int i = 0; i < C::kBChunksPerThread; ++i) {
      const bool ok = bg_src[i] && k0 + b_k[i] < d_model;
      bg_reg[i] = ok ? *reinterpret_cast<const u32x4*>(bg_src[i] + k0) : zero4;
      bu_reg[i] = ok ? *reinterpret_cast<const u32x4*>(bu_src[i] + k0) : zero4;
    }
  };
  auto store_lds = [&](int buf) {
    unsigned char* sA = smem + buf * C::kStageBytes;
    unsigned char* sBg = sA + C::kATileBytes;
    unsigned char* sBu = sBg + C::kBTileBytes;
#pragma unroll
    for (int i = 0; i < C::kAChunksPerThread; ++i) *reinterpret_cast<u32x4*>(sA + a_dst[i]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < C::kBChunksPerThread; ++i) {
      *reinterpret_cast<u32x4*>(sBg + b_dst[i]) = bg_reg[i];
      *reinterpret_cast<u32x4*>(sBu + b_dst[i]) = bu_reg[i];
    }
  };

  f32x16 acc_g[TM][TN], acc_u[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc_g[i][j][r] = 0.0f;
        acc_u[i][j][r] = 0.0f;
      }

  // Fragment addressing: lane l holds row (l % 32), K elements 8*(l / 32) .. +7 of a 16-wide K step.
  const int frag_row = lane % 32;
  const int frag_half = lane / 32;
  const int a_row0 = wave_m * TM * 32 + frag_row;
  const int b_row0 = wave_n * TN * 32 + frag_row;

  const int n_k = (d_model + KT - 1) / KT;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < n_k; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < n_k) load_global((kt + 1) * KT);
    const unsigned char* sA = smem + buf * C::kStageBytes;
    const unsigned char* sBg = sA + C::kATileBytes;
    const unsigned char* sBu = sBg + C::kBTileBytes;
#pragma unroll
    for (int ks = 0; ks < KT / 16; ++ks) {
      const int chunk = ks * 2 + frag_half;
      bf16x8 fa[TM], fg[TN], fu[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(sA + swizzled(a_row0 + i * 32, chunk));
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        fg[j] = *reinterpret_cast<const bf16x8*>(sBg + swizzled(b_row0 + j * 32, chunk));
        fu[j] = *reinterpret_cast<const bf16x8*>(sBu + swizzled(b_row0 + j * 32, chunk));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc_g[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fg[j], acc_g[i][j], 0, 0, 0);
          acc_u[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fu[j], acc_u[i][j], 0, 0, 0);
        }
    }
    if (kt + 1 < n_k) store_lds(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  Accumulator register r of lane l is output row 8*(r/4) + 4*(l/32) + (r%4),
  // column l % 32 of its 32x32 tile: a lane owns one channel and 16 token rows.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    float sum = 0.0f, mx = 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int band = wave_m * TM * 32 + i * 32 + frag_half * 4;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = band + (r / 4) * 8 + (r % 4);
        const float lam = s_a[row] * silu_f32(acc_g[i][j][r]) * acc_u[i][j][r];
        const float l2 = lam * lam;
        sum += l2;
        mx = fmaxf(mx, l2);
      }
    }
    sum += __shfl_xor(sum, 32);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (frag_half == 0) {
      const int col = wave_n * TN * 32 + j * 32 + frag_row;
      s_red[wave_m * BN + col] = sum;
      s_red[(WM + wave_m) * BN + col] = mx;
    }
  }
  __syncthreads();
  for (int col = tid; col < BN; col += C::kThreads) {
    if (n0 + col < d_ff) {
      float sum = 0.0f, mx = 0.0f;
#pragma unroll
      for (int w = 0; w < WM; ++w) {  // fixed order
        sum += s_red[w * BN + col];
        mx = fmaxf(mx, s_red[(WM + w) * BN + col]);
      }
      part_phi2[(int64_t)slot * d_ff + n0 + col] = sum;
      part_max[(int64_t)slot * d_ff + n0 + col] = mx;
    }
  }
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

// Tile shape of the bf16 kernel: 2x2 waves, each 64 tokens x 64 channels (gate and up).
using Bf16Cfg = GemmCfg<2, 2, 2, 2>;

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
    static bool attr_set = false;
    auto kern = grouped_gemm_bf16_kernel<C>;
    if (!attr_set) {
      hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kSmemBytes);
      if (err != hipSuccess) return err;
      attr_set = true;
    }
    dim3 grid((unsigned)((d_ff + C::BN - 1) / C::BN), (unsigned)max_tiles);
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

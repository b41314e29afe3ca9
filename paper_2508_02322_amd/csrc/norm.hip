// Squared column norms of W_down (Algorithm 1, line 5: omega^2 = ColumnSum(W_down o W_down))
// and the final combination of line 10 (energy with the balance coefficient alpha).
//
// down_norm: HBM-bound streaming pass.  W_down[e] is [d_model x d_ff] row-major, so column c
// (micro-expert c) is strided; a lane owns 8 consecutive columns (one 16-byte load per row),
// a wave owns 512 consecutive columns of a row (1 KiB, fully coalesced) and the four waves of
// a block take rows r, r+1, r+2, r+3 of the block's row split.  Row splits keep enough
// loads in flight to fill the chip; their partial sums are added in split order by the
// finalize kernel.
#include <hip/hip_bf16.h>

#include "camera_internal.h"

namespace camera {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

template <typename T>
struct Vec;
template <>
struct Vec<__hip_bfloat16> {
  static constexpr int kPerLane = 8;  // 16 bytes
  __device__ static void load_sq(const __hip_bfloat16* p, float (&acc)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lo = __uint_as_float(w[i] << 16);
      const float hi = __uint_as_float(w[i] & 0xffff0000u);
      acc[2 * i] = fmaf(lo, lo, acc[2 * i]);
      acc[2 * i + 1] = fmaf(hi, hi, acc[2 * i + 1]);
    }
  }
  __device__ static float to_float(__hip_bfloat16 v) { return __bfloat162float(v); }
};
template <>
struct Vec<float> {
  static constexpr int kPerLane = 4;  // 16 bytes
  __device__ static void load_sq(const float* p, float (&acc)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    acc[0] = fmaf(v.x, v.x, acc[0]);
    acc[1] = fmaf(v.y, v.y, acc[1]);
    acc[2] = fmaf(v.z, v.z, acc[2]);
    acc[3] = fmaf(v.w, v.w, acc[3]);
  }
  __device__ static float to_float(float v) { return v; }
};

// grid = (column blocks, row splits, experts)
template <typename T>
__global__ __launch_bounds__(kThreads) void down_norm_kernel(const T* __restrict__ W, int64_t stride_down,
                                                             int d_model, int d_ff, int rows_per_split,
                                                             int64_t n_micro, float* __restrict__ omega_part) {
  constexpr int V = Vec<T>::kPerLane;
  __shared__ float s_part[kWaves][kWave * V];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int e = blockIdx.z;
  const int c0 = (blockIdx.x * kWave + lane) * V;
  const int r_begin = blockIdx.y * rows_per_split;
  const int r_end = min(d_model, r_begin + rows_per_split);
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.0f;
  if (c0 < d_ff) {  // d_ff is a multiple of V here, so the whole vector is inside
    const T* col = W + (int64_t)e * stride_down + c0;
    int r = r_begin + wave;
    for (; r + 3 * kWaves < r_end; r += 4 * kWaves) {  // four independent loads in flight
      Vec<T>::load_sq(col + (int64_t)r * d_ff, acc);
      Vec<T>::load_sq(col + (int64_t)(r + kWaves) * d_ff, acc);
      Vec<T>::load_sq(col + (int64_t)(r + 2 * kWaves) * d_ff, acc);
      Vec<T>::load_sq(col + (int64_t)(r + 3 * kWaves) * d_ff, acc);
    }
    for (; r < r_end; r += kWaves) Vec<T>::load_sq(col + (int64_t)r * d_ff, acc);
  }
#pragma unroll
  for (int i = 0; i < V; ++i) s_part[wave][lane * V + i] = acc[i];
  __syncthreads();
  for (int i = threadIdx.x; i < kWave * V; i += kThreads) {
    const int c = blockIdx.x * kWave * V + i;
    if (c < d_ff) {
      float s = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) s += s_part[w][i];  // fixed order
      omega_part[(int64_t)blockIdx.y * n_micro + (int64_t)e * d_ff + c] = s;
    }
  }
}

// Any d_ff / alignment: one thread per column, rows streamed (consecutive threads read
// consecutive columns, so rows are still coalesced).
template <typename T>
__global__ __launch_bounds__(kThreads) void down_norm_generic_kernel(const T* __restrict__ W, int64_t stride_down,
                                                                     int d_model, int d_ff, int rows_per_split,
                                                                     int64_t n_micro,
                                                                     float* __restrict__ omega_part) {
  const int e = blockIdx.z;
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= d_ff) return;
  const int r_begin = blockIdx.y * rows_per_split;
  const int r_end = min(d_model, r_begin + rows_per_split);
  const T* col = W + (int64_t)e * stride_down + c;
  float s = 0.0f;
  for (int r = r_begin; r < r_end; ++r) {
    const float v = Vec<T>::to_float(col[(int64_t)r * d_ff]);
    s = fmaf(v, v, s);
  }
  omega_part[(int64_t)blockIdx.y * n_micro + (int64_t)e * d_ff + c] = s;
}

// Input-channel energies h[e][c] = sum over the tokens routed to expert e of X[token][c]^2 (the diagonal of
// X_e^T X_e).  Same streaming shape as down_norm, with the rows found through the bucket permutation:
// grid = (column blocks, row splits, experts); split s of expert e takes an equal share of its bucket.
template <typename T>
__global__ __launch_bounds__(kThreads) void input_energy_kernel(const T* __restrict__ X, int64_t ldx, int d_model,
                                                                const int32_t* __restrict__ offsets,
                                                                const int32_t* __restrict__ perm, int64_t n_cols,
                                                                float* __restrict__ part) {
  constexpr int V = Vec<T>::kPerLane;
  __shared__ float s_part[kWaves][kWave * V];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int e = blockIdx.z;
  const int c0 = (blockIdx.x * kWave + lane) * V;
  const int first = offsets[e], count = offsets[e + 1] - first;
  const int r_begin = (int)((int64_t)count * blockIdx.y / gridDim.y);
  const int r_end = (int)((int64_t)count * (blockIdx.y + 1) / gridDim.y);
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.0f;
  if (c0 < d_model) {  // d_model is a multiple of V, so the whole vector is inside
    auto row = [&](int r) { return X + (int64_t)(perm ? perm[first + r] : r) * ldx + c0; };
    int r = r_begin + wave;
    for (; r + 3 * kWaves < r_end; r += 4 * kWaves) {  // four independent loads in flight
      const T* p0 = row(r);
      const T* p1 = row(r + kWaves);
      const T* p2 = row(r + 2 * kWaves);
      const T* p3 = row(r + 3 * kWaves);
      Vec<T>::load_sq(p0, acc);
      Vec<T>::load_sq(p1, acc);
      Vec<T>::load_sq(p2, acc);
      Vec<T>::load_sq(p3, acc);
    }
    for (; r < r_end; r += kWaves) Vec<T>::load_sq(row(r), acc);
  }
#pragma unroll
  for (int i = 0; i < V; ++i) s_part[wave][lane * V + i] = acc[i];
  __syncthreads();
  for (int i = threadIdx.x; i < kWave * V; i += kThreads) {
    const int c = blockIdx.x * kWave * V + i;
    if (c < d_model) {
      float s = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) s += s_part[w][i];  // fixed order
      part[(int64_t)blockIdx.y * n_cols + (int64_t)e * d_model + c] = s;
    }
  }
}

// out[i] = part[0][i] + part[1][i] + ... in split order
__global__ __launch_bounds__(kThreads) void sum_splits_kernel(const float* __restrict__ part, int splits, int64_t n_cols,
                                                              float* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n_cols) return;
  float s = 0.0f;
  for (int k = 0; k < splits; ++k) s += part[(int64_t)k * n_cols + i];
  out[i] = s;
}

__global__ __launch_bounds__(kThreads) void finalize_kernel(int n_experts, int d_ff,
                                                            const int32_t* __restrict__ tile_offset,
                                                            const float* __restrict__ part_phi2,
                                                            const float* __restrict__ part_max,
                                                            const float* __restrict__ omega_part, int splits,
                                                            float alpha, int accumulate, int finalize,
                                                            float* __restrict__ phi2, float* __restrict__ phi_inf,
                                                            float* __restrict__ omega2, float* __restrict__ energy) {
  const int e = blockIdx.y;
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= d_ff) return;
  const int64_t i = (int64_t)e * d_ff + c;
  const int64_t n_micro = (int64_t)n_experts * d_ff;
  // M-tiles of this expert, added in tile order.  Eight loads are in flight at a time (a thread that waits for
  // each tile in turn spends the kernel waiting); tiles past the end re-read the last one and contribute nothing.
  float sum = 0.0f, mx = 0.0f;
  const int t_begin = tile_offset[e], t_end = tile_offset[e + 1];
  for (int t0 = t_begin; t0 < t_end; t0 += 8) {
    float p2[8], pm[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = min(t0 + u, t_end - 1);
      p2[u] = part_phi2[(int64_t)t * d_ff + c];
      pm[u] = part_max[(int64_t)t * d_ff + c];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (t0 + u < t_end) {
        sum += p2[u];
        mx = fmaxf(mx, pm[u]);
      }
    }
  }
  if (accumulate) {
    sum += phi2[i];
    mx = fmaxf(mx, phi_inf[i]);
  }
  phi2[i] = sum;
  phi_inf[i] = mx;
  if (finalize) {
    float w2 = 0.0f;
    for (int s0 = 0; s0 < splits; s0 += 8) {  // row splits of omega^2, in split order, eight loads at a time
      float part[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) part[u] = omega_part[(int64_t)min(s0 + u, splits - 1) * n_micro + i];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (s0 + u < splits) w2 += part[u];
    }
    omega2[i] = w2;
    energy[i] = ((1.0f - alpha) * sum + alpha * mx) * w2;
  }
}

}  // namespace

int down_norm_splits(int n_experts, int64_t d_model, int64_t d_ff) {
  // aim at >= 2048 blocks, at least 64 rows per split, at most 64 splits (one wide expert -- a shared expert of
  // 20480 channels is 40 column blocks -- needs many row splits to fill the chip)
  const int64_t col_blocks = (d_ff + 511) / 512;
  int64_t want = (2048 + n_experts * col_blocks - 1) / (n_experts * col_blocks);
  const int64_t by_rows = d_model / 64 > 0 ? d_model / 64 : 1;
  if (want > by_rows) want = by_rows;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  return (int)want;
}

hipError_t launch_down_norm(hipStream_t stream, int dtype, const void* W_down, int64_t stride_down,
                            int n_experts, int64_t d_model, int64_t d_ff, int splits, float* omega_part) {
  const int rows_per_split = (int)((d_model + splits - 1) / splits);
  const int64_t n_micro = (int64_t)n_experts * d_ff;
  const int v = dtype == CAMERA_BF16 ? 8 : 4;
  const bool vector_ok = d_ff % v == 0 && stride_down % v == 0;
  if (vector_ok) {
    dim3 grid((unsigned)((d_ff + kWave * v - 1) / (kWave * v)), (unsigned)splits, (unsigned)n_experts);
    if (dtype == CAMERA_BF16)
      hipLaunchKernelGGL(down_norm_kernel<__hip_bfloat16>, grid, dim3(kThreads), 0, stream,
                         static_cast<const __hip_bfloat16*>(W_down), stride_down, (int)d_model, (int)d_ff,
                         rows_per_split, n_micro, omega_part);
    else
      hipLaunchKernelGGL(down_norm_kernel<float>, grid, dim3(kThreads), 0, stream,
                         static_cast<const float*>(W_down), stride_down, (int)d_model, (int)d_ff, rows_per_split,
                         n_micro, omega_part);
  } else {
    dim3 grid((unsigned)((d_ff + kThreads - 1) / kThreads), (unsigned)splits, (unsigned)n_experts);
    if (dtype == CAMERA_BF16)
      hipLaunchKernelGGL(down_norm_generic_kernel<__hip_bfloat16>, grid, dim3(kThreads), 0, stream,
                         static_cast<const __hip_bfloat16*>(W_down), stride_down, (int)d_model, (int)d_ff,
                         rows_per_split, n_micro, omega_part);
    else
      hipLaunchKernelGGL(down_norm_generic_kernel<float>, grid, dim3(kThreads), 0, stream,
                         static_cast<const float*>(W_down), stride_down, (int)d_model, (int)d_ff, rows_per_split,
                         n_micro, omega_part);
  }
  return hipGetLastError();
}

int input_energy_splits(int n_experts, int64_t d_model, int dtype) {
  // aim at >= 1024 blocks, at most 16 splits
  const int v = dtype == CAMERA_BF16 ? 8 : 4;
  const int64_t col_blocks = (d_model + kWave * v - 1) / (kWave * v);
  int64_t want = (1024 + n_experts * col_blocks - 1) / (n_experts * col_blocks);
  return (int)(want < 1 ? 1 : (want > 16 ? 16 : want));
}

hipError_t launch_input_energy(hipStream_t stream, int dtype, const void* X, int64_t ldx, int n_experts,
                               int64_t d_model, const BucketTables& t, int splits, float* part, float* h) {
  const int v = dtype == CAMERA_BF16 ? 8 : 4;
  const int64_t n_cols = (int64_t)n_experts * d_model;
  dim3 grid((unsigned)((d_model + kWave * v - 1) / (kWave * v)), (unsigned)splits, (unsigned)n_experts);
  if (dtype == CAMERA_BF16)
    hipLaunchKernelGGL(input_energy_kernel<__hip_bfloat16>, grid, dim3(kThreads), 0, stream,
                       static_cast<const __hip_bfloat16*>(X), ldx, (int)d_model, t.offsets, t.perm, n_cols, part);
  else
    hipLaunchKernelGGL(input_energy_kernel<float>, grid, dim3(kThreads), 0, stream, static_cast<const float*>(X), ldx,
                       (int)d_model, t.offsets, t.perm, n_cols, part);
  hipLaunchKernelGGL(sum_splits_kernel, dim3((unsigned)((n_cols + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                     part, splits, n_cols, h);
  return hipGetLastError();
}

hipError_t launch_finalize(hipStream_t stream, int n_experts, int64_t d_ff, const BucketTables& t,
                           const float* part_phi2, const float* part_max, const float* omega_part, int splits,
                           float alpha, int accumulate, int finalize, float* phi2, float* phi_inf,
                           float* omega2, float* energy) {
  dim3 grid((unsigned)((d_ff + kThreads - 1) / kThreads), (unsigned)n_experts);
  hipLaunchKernelGGL(finalize_kernel, grid, dim3(kThreads), 0, stream, n_experts, (int)d_ff, t.tile_offset,
                     part_phi2, part_max, omega_part, splits, alpha, accumulate, finalize, phi2, phi_inf, omega2,
                     energy);
  return hipGetLastError();
}

}  // namespace camera

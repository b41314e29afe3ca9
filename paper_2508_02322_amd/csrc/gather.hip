// Applying a selection: W_up, W_gate, W_down <- W_up[S,:], W_gate[S,:], W_down[:,S]
// (Algorithm 2, lines 10-13), per expert and packed; with the permutation of
// the bit allocation as the index list it is the reordering that colocates
// micro-experts of equal precision inside an expert (Section "Mixed-precision
// Strategy CAMERA-Q").  Pure data movement, bound by HBM bandwidth:
//   offsets : exclusive prefix of the per-expert entry counts (one small block)
//   rows    : a wave copies one kept gate row and the matching up row, 16 bytes
//             per lane and step -- fully coalesced on both sides
//   columns : a workgroup owns one expert and a few rows of its W_down; it
//             keeps the expert's column list in LDS, streams each row through
//             LDS with 16-byte loads (the kept columns touch nearly every 64-byte
//             sector of the row anyway) and writes the kept elements side by side,
//             then zeros up to the block's row length (the count rounded up to the
//             caller's row alignment).
// Entries that do not lie inside their expert give zero rows / columns: no
// address is ever formed from an unchecked index.
#include <hip/hip_bf16.h>

#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = kThreads / kWave;  // gather_rows: one wave per output row
constexpr int kDownRows = 8;                     // gather_cols: W_down rows per workgroup
constexpr uint16_t kNoColumn = 0xffffu;

// off [n_experts + 1]: prefix of the entry counts; off_ld [n_experts + 1]: prefix of the counts rounded up to
// a multiple of row_align (the row lengths of the W_down blocks).
__global__ __launch_bounds__(CAMERA_MAX_EXPERTS) void gather_offsets_kernel(const int32_t* __restrict__ count,
                                                                            int n_experts, int d_ff, int row_align,
                                                                            int32_t* __restrict__ off,
                                                                            int32_t* __restrict__ off_ld) {
  __shared__ int32_t s_cnt[CAMERA_MAX_EXPERTS];
  const int e = threadIdx.x;
  if (e < n_experts) s_cnt[e] = count ? min(max(count[e], 0), d_ff) : d_ff;
  __syncthreads();
  if (e == 0) {
    int32_t run = 0, run_ld = 0;
    for (int i = 0; i < n_experts; ++i) {
      off[i] = run;
      off_ld[i] = run_ld;
      run += s_cnt[i];
      run_ld += (s_cnt[i] + row_align - 1) / row_align * row_align;
    }
    off[n_experts] = run;
    off_ld[n_experts] = run_ld;
  }
}

// expert that owns output position r: the last e with off[e] <= r (off is non-decreasing, off[0] = 0)
__device__ __forceinline__ int owner_of(const int32_t* s_off, int n_experts, int64_t r) {
  int lo = 0, hi = n_experts;  // invariant: off[lo] <= r < off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) / 2;
    if (s_off[mid] <= r) lo = mid;
    else hi = mid;
  }
  return lo;
}

// row_vecs = d_model * element size / 16.  Output row r of gate_out / up_out <- row index[r] of its expert.
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(
    const u32x4* __restrict__ Wg, const u32x4* __restrict__ Wu, int64_t stride_gu_vecs, int n_experts, int d_ff,
    int row_vecs, const int32_t* __restrict__ index, int64_t n_index, int64_t index_base,
    const int32_t* __restrict__ off, u32x4* __restrict__ gate_out, u32x4* __restrict__ up_out) {
  __shared__ int32_t s_off[CAMERA_MAX_EXPERTS + 1];
  for (int i = threadIdx.x; i <= n_experts; i += kThreads) s_off[i] = off[i];
  __syncthreads();
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int64_t r = (int64_t)blockIdx.x * kRowsPerBlock + wave;
  if (r >= n_index || r >= s_off[n_experts]) return;  // wave-uniform
  const int e = owner_of(s_off, n_experts, r);
  const int64_t c = (int64_t)index[r] - index_base - (int64_t)e * d_ff;
  const bool ok = c >= 0 && c < d_ff;
  const int64_t src = (int64_t)e * stride_gu_vecs + (ok ? c : 0) * row_vecs;
  const int64_t dst = r * row_vecs;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int k = lane; k < row_vecs; k += kWave) {
    if (gate_out) gate_out[dst + k] = ok ? Wg[src + k] : zero;
    if (up_out) up_out[dst + k] = ok ? Wu[src + k] : zero;
  }
}

// T: element type by size (uint16_t for bf16, uint32_t for float32).  VEC: rows of W_down start on 16-byte
// boundaries and are whole 16-byte vectors long.  Dynamic LDS: d_ff elements of T, then cnt_max uint16 columns.
template <class T, bool VEC>
__global__ __launch_bounds__(kThreads) void gather_cols_kernel(const T* __restrict__ Wd, int64_t stride_down,
                                                               int d_ff, int d_model,
                                                               const int32_t* __restrict__ index, int64_t n_index,
                                                               int64_t index_base, const int32_t* __restrict__ off,
                                                               const int32_t* __restrict__ off_ld,
                                                               T* __restrict__ down_out) {
  extern __shared__ __align__(16) unsigned char smem[];
  T* s_row = reinterpret_cast<T*>(smem);
  uint16_t* s_col = reinterpret_cast<uint16_t*>(smem + (((size_t)d_ff * sizeof(T) + 15) & ~size_t(15)));
  const int e = blockIdx.x;
  const int64_t first = off[e];
  const int cnt = (int)min((int64_t)(off[e + 1] - off[e]), max((int64_t)0, n_index - first));  // entries that exist
  if (cnt <= 0) return;  // block-uniform
  for (int j = threadIdx.x; j < cnt; j += kThreads) {
    const int64_t c = (int64_t)index[first + j] - index_base - (int64_t)e * d_ff;
    s_col[j] = (c >= 0 && c < d_ff) ? (uint16_t)c : kNoColumn;  // d_ff <= 32768 (checked by the caller), so no clash
  }
  const T* src_expert = Wd + (int64_t)e * stride_down;
  const int ld = off_ld[e + 1] - off_ld[e];  // row length of the block: the count rounded up, the rest zero
  T* dst_expert = down_out + off_ld[e] * (int64_t)d_model;
  const int r_begin = blockIdx.y * kDownRows, r_end = min(d_model, r_begin + kDownRows);
  for (int r = r_begin; r < r_end; ++r) {
    __syncthreads();  // the column list is complete; the previous row has been read out
    const T* src_row = src_expert + (int64_t)r * d_ff;
    if (VEC) {
      const int n_vec = d_ff * (int)sizeof(T) / 16;
      for (int k = threadIdx.x; k < n_vec; k += kThreads)
        reinterpret_cast<u32x4*>(s_row)[k] = reinterpret_cast<const u32x4*>(src_row)[k];
    } else {
      for (int k = threadIdx.x; k < d_ff; k += kThreads) s_row[k] = src_row[k];
    }
    __syncthreads();
    T* dst_row = dst_expert + (int64_t)r * ld;
    for (int j = threadIdx.x; j < ld; j += kThreads) {
      const uint16_t c = j < cnt ? s_col[j] : kNoColumn;
      dst_row[j] = c == kNoColumn ? T(0) : s_row[c];
    }
  }
}

}  // namespace

hipError_t launch_gather_offsets(hipStream_t stream, const int32_t* count, int n_experts, int64_t d_ff,
                                 int row_align, int32_t* off, int32_t* off_ld) {
  hipLaunchKernelGGL(gather_offsets_kernel, dim3(1), dim3(CAMERA_MAX_EXPERTS), 0, stream, count, n_experts, (int)d_ff,
                     row_align, off, off_ld);
  return hipGetLastError();
}

hipError_t launch_gather_rows(hipStream_t stream, int dtype, const void* W_gate, const void* W_up, int64_t stride_gu,
                              int n_experts, int64_t d_ff, int64_t d_model, const int32_t* index, int64_t n_index,
                              int64_t index_base, const int32_t* off, void* gate_out, void* up_out) {
  if (n_index <= 0 || (gate_out == nullptr && up_out == nullptr)) return hipSuccess;
  const int es = dtype == CAMERA_BF16 ? 2 : 4;
  const int64_t blocks = (n_index + kRowsPerBlock - 1) / kRowsPerBlock;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                     static_cast<const u32x4*>(W_gate), static_cast<const u32x4*>(W_up), stride_gu * es / 16, n_experts,
                     (int)d_ff, (int)(d_model * es / 16), index, n_index, index_base, off,
                     static_cast<u32x4*>(gate_out), static_cast<u32x4*>(up_out));
  return hipGetLastError();
}

template <class T>
static hipError_t launch_cols(hipStream_t stream, const void* W_down, int64_t stride_down, int n_experts, int64_t d_ff,
                              int64_t d_model, const int32_t* index, int64_t n_index, int64_t index_base,
                              const int32_t* off, const int32_t* off_ld, void* down_out) {
  const bool vec = (d_ff * sizeof(T)) % 16 == 0 && (stride_down * sizeof(T)) % 16 == 0 &&
                   (reinterpret_cast<uintptr_t>(W_down) & 15u) == 0;
  auto kern = vec ? gather_cols_kernel<T, true> : gather_cols_kernel<T, false>;
  const size_t smem = (((size_t)d_ff * sizeof(T) + 15) & ~size_t(15)) + (size_t)d_ff * sizeof(uint16_t);
  hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
  if (err != hipSuccess) return err;
  dim3 grid((unsigned)n_experts, (unsigned)((d_model + kDownRows - 1) / kDownRows));
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, stream, static_cast<const T*>(W_down), stride_down, (int)d_ff,
                     (int)d_model, index, n_index, index_base, off, off_ld, static_cast<T*>(down_out));
  return hipGetLastError();
}

hipError_t launch_gather_cols(hipStream_t stream, int dtype, const void* W_down, int64_t stride_down, int n_experts,
                              int64_t d_ff, int64_t d_model, const int32_t* index, int64_t n_index,
                              int64_t index_base, const int32_t* off, const int32_t* off_ld, void* down_out) {
  if (n_index <= 0 || down_out == nullptr) return hipSuccess;
  if (dtype == CAMERA_BF16)
    return launch_cols<uint16_t>(stream, W_down, stride_down, n_experts, d_ff, d_model, index, n_index, index_base, off,
                                 off_ld, down_out);
  return launch_cols<uint32_t>(stream, W_down, stride_down, n_experts, d_ff, d_model, index, n_index, index_base, off,
                               off_ld, down_out);
}

}  // namespace camera

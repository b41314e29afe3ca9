// The layer output over the kept micro-experts (Eq. 1-2; the recomputed output
// of Algorithm 2, line 14) and its distance from the original output (the
// Lemma's decoding error; the L2 / cosine comparison of hidden states).
//
// The two contractions run in the grouped MFMA kernel (gemm.hip): first
// Lambda = a silu(X W_gate^T) (X W_up^T), masked and stored as bf16 per bucket
// slot, then Lambda W_down^T per slot in float32.  What is here:
//   combine : y_token (+)= the rows of its top-k slots, added in k order (a
//             token's experts are summed in a fixed order, no float atomics)
//   error   : per token ||y - y_hat||^2, ||y||^2, ||y_hat||^2, <y, y_hat>
#include "camera_internal.h"

namespace camera {
namespace {

constexpr int kThreads = 256;
constexpr int kTokensPerBlock = kThreads / kWave;  // one wave per token

// rows: product [pairs][d_model] float32.  Routed: slot_of[token * top_k + k]; dense: slot = e * n + token.
__global__ __launch_bounds__(kThreads) void combine_kernel(const float4* __restrict__ product,
                                                           const int32_t* __restrict__ slot_of, int64_t n, int top_k,
                                                           int n_experts, int vecs, int accumulate,
                                                           float4* __restrict__ Y) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int64_t tok = (int64_t)blockIdx.x * kTokensPerBlock + wave;
  if (tok >= n) return;
  const int terms = slot_of ? top_k : n_experts;
  for (int v = lane; v < vecs; v += kWave) {
    float4 s = accumulate ? Y[tok * vecs + v] : make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = 0; k < terms; ++k) {
      const int64_t row = slot_of ? (int64_t)slot_of[tok * top_k + k] : (int64_t)k * n + tok;
      if (row < 0) continue;  // a pair with an expert id outside the group
      const float4 p = product[row * vecs + v];
      s.x += p.x;
      s.y += p.y;
      s.z += p.z;
      s.w += p.w;
    }
    Y[tok * vecs + v] = s;
  }
}

__global__ __launch_bounds__(kThreads) void output_error_kernel(const float* __restrict__ Y,
                                                                const float* __restrict__ Y_hat, int64_t n,
                                                                int64_t d_model, int64_t ldy, int64_t ldh,
                                                                float* __restrict__ per_token) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int64_t tok = (int64_t)blockIdx.x * kTokensPerBlock + wave;
  if (tok >= n) return;
  const float* y = Y + tok * ldy;
  const float* h = Y_hat + tok * ldh;
  float d2 = 0.f, yy = 0.f, hh = 0.f, yh = 0.f;
  for (int64_t c = lane; c < d_model; c += kWave) {
    const float a = y[c], b = h[c], d = a - b;
    d2 = fmaf(d, d, d2);
    yy = fmaf(a, a, yy);
    hh = fmaf(b, b, hh);
    yh = fmaf(a, b, yh);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    d2 += __shfl_xor(d2, m);
    yy += __shfl_xor(yy, m);
    hh += __shfl_xor(hh, m);
    yh += __shfl_xor(yh, m);
  }
  if (lane == 0) {
    per_token[tok * 4 + 0] = d2;
    per_token[tok * 4 + 1] = yy;
    per_token[tok * 4 + 2] = hh;
    per_token[tok * 4 + 3] = yh;
  }
}

}  // namespace

hipError_t launch_combine(hipStream_t stream, const float* product, const int32_t* slot_of, int64_t n, int top_k,
                          int n_experts, int64_t d_model, int accumulate, float* Y) {
  if (n <= 0) return hipSuccess;
  const int64_t blocks = (n + kTokensPerBlock - 1) / kTokensPerBlock;
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                     reinterpret_cast<const float4*>(product), slot_of, n, top_k, n_experts, (int)(d_model / 4),
                     accumulate, reinterpret_cast<float4*>(Y));
  return hipGetLastError();
}

hipError_t launch_output_error(hipStream_t stream, const float* Y, const float* Y_hat, int64_t n, int64_t d_model,
                               int64_t ldy, int64_t ldh, float* per_token) {
  if (n <= 0) return hipSuccess;
  const int64_t blocks = (n + kTokensPerBlock - 1) / kTokensPerBlock;
  hipLaunchKernelGGL(output_error_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, Y, Y_hat, n, d_model, ldy,
                     ldh, per_token);
  return hipGetLastError();
}

}  // namespace camera

// A = Top&Norm(R X): router logits, softmax, top-k and renormalisation
// (Algorithm 1, line 2; the weights A_i(x) of Eq. 2).
//
// Logits L[j, e] = <x_j, R_e> (+ bias_e) are accumulated in float32: for bf16 on
// v_mfma_f32_32x32x16_bf16 (a block = 32 tokens x all experts, its four waves
// split d_model, fragments read straight from global memory -- R is small and
// stays in L2), for float32 with FMA and a wave reduction.  The logits of a
// block's tokens go through LDS so that eight lanes can walk the experts of
// one token: top_k rounds of "largest remaining logit, lower index on ties".
// Selection is on the logits (softmax is increasing, so this is the top-k of
// the probabilities); the kept weights are exp(L - max) over the softmax
// denominator, renormalised over the kept ones.
#include <hip/hip_bf16.h>

#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kTokens = 32;  // tokens per block
constexpr int kSub = 8;      // lanes that share one token in the top-k stage

// Top-k of one token by kSub consecutive lanes: lane `sub` scans experts sub, sub + kSub, ...; each
// round takes the largest logit not yet taken (ties: lower index) and the lanes agree on it with
// three xor-shuffles.  s_row[0 .. n_experts) are the token's logits.
__device__ void topk_of_token(const float* s_row, int n_experts, int top_k, int renorm, int sub,
                              int32_t* idx_out, float* w_out) {
  float row_max = -INFINITY;
  for (int e = sub; e < n_experts; e += kSub) row_max = fmaxf(row_max, s_row[e]);
#pragma unroll
  for (int m = kSub / 2; m >= 1; m >>= 1) row_max = fmaxf(row_max, __shfl_xor(row_max, m));
  float denom = 0.0f;
  if (!renorm) {
    for (int e = sub; e < n_experts; e += kSub) denom += __expf(s_row[e] - row_max);
#pragma unroll
    for (int m = kSub / 2; m >= 1; m >>= 1) denom += __shfl_xor(denom, m);
  }
  float prev_v = INFINITY;
  int prev_i = -1;
  float kept_sum = 0.0f;
  for (int r = 0; r < top_k; ++r) {
    float best_v = -INFINITY;
    int best_i = 0x7fffffff;
    for (int e = sub; e < n_experts; e += kSub) {
      const float v = s_row[e];
      const bool not_taken = v < prev_v || (v == prev_v && e > prev_i);
      if (not_taken && (v > best_v || (v == best_v && e < best_i))) {
        best_v = v;
        best_i = e;
      }
    }
#pragma unroll
    for (int m = kSub / 2; m >= 1; m >>= 1) {
      const float ov = __shfl_xor(best_v, m);
      const int oi = __shfl_xor(best_i, m);
      if (ov > best_v || (ov == best_v && oi < best_i)) {
        best_v = ov;
        best_i = oi;
      }
    }
    const float p = __expf(best_v - row_max);
    if (sub == 0) {
      idx_out[r] = best_i;
      w_out[r] = p;
    }
    kept_sum += p;
    prev_v = best_v;
    prev_i = best_i;
  }
  if (sub == 0) {
    const float inv = 1.0f / (renorm ? kept_sum : denom);
    for (int r = 0; r < top_k; ++r) w_out[r] *= inv;
  }
}

// bf16: 32 tokens per block, NT tiles of 32 experts.  The block's NG * 4 waves split d_model between them (a
// lone wave per 32 tokens leaves the chip idle and waits for every load in turn) and keep kUnroll K steps of
// loads in flight.  No load is conditional: a lane whose token, expert or K position lies outside reads a
// valid address all the same (row 0, or a page of zeros for the K tail), so the compiler can issue a whole
// batch before the first wait; what such lanes accumulate is never used.  Partial logits are added through
// LDS in a fixed order: the four waves of a group one after the other, then the groups.
template <int NT, int NG>
__global__ __launch_bounds__(256 * NG) void route_bf16_kernel(const __hip_bfloat16* __restrict__ X, int64_t n,
                                                              int d_model, int64_t ldx,
                                                              const __hip_bfloat16* __restrict__ R, int64_t ldr,
                                                              const float* __restrict__ bias, int n_experts,
                                                              int top_k, int renorm,
                                                              const __hip_bfloat16* __restrict__ zeros,
                                                              int32_t* __restrict__ topk_idx,
                                                              float* __restrict__ topk_w) {
  constexpr int kUnroll = NT <= 2 ? 8 : (NT == 4 ? 4 : 2);
  constexpr int kWaves = 4 * NG;
  __shared__ float s_logit[NG][kTokens][NT * 32 + 1];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int group = wave / 4, turn = wave % 4;
  const int frag_row = lane % 32, frag_half = lane / 32;
  const int64_t tok0 = (int64_t)blockIdx.x * kTokens;
  const int64_t tok = tok0 + frag_row;
  const __hip_bfloat16* x_src = X + (tok < n ? tok : 0) * ldx + frag_half * 8;
  const __hip_bfloat16* r_src[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int e = t * 32 + frag_row;
    r_src[t] = R + (int64_t)(e < n_experts ? e : 0) * ldr + frag_half * 8;
  }
  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

  // this wave's share of the K steps (16 elements each)
  const int n_steps = (d_model + 15) / 16;
  const int per_wave = (n_steps + kWaves - 1) / kWaves;
  const int k_begin = min(d_model, wave * per_wave * 16);
  const int k_end = min(d_model, (wave + 1) * per_wave * 16);
  for (int k0 = k_begin; k0 < k_end; k0 += 16 * kUnroll) {
    u32x4 av[kUnroll], bv[kUnroll][NT];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int k = k0 + 16 * u;
      const bool k_ok = k + frag_half * 8 < k_end;  // d_model and the wave shares are multiples of 8
      av[u] = *reinterpret_cast<const u32x4*>(k_ok ? x_src + k : zeros);
#pragma unroll
      for (int t = 0; t < NT; ++t) bv[u][t] = *reinterpret_cast<const u32x4*>(k_ok ? r_src[t] + k : zeros);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[u]),
                                                          __builtin_bit_cast(bf16x8, bv[u][t]), acc[t], 0, 0, 0);
  }
  // accumulator register r of lane l: token row 8*(r/4) + 4*(l/32) + (r%4), expert column l % 32
  for (int w = 0; w < 4; ++w) {  // fixed order inside a group: its first wave stores, the others add
    if (turn == w) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int e = t * 32 + frag_row;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float* dst = &s_logit[group][(r / 4) * 8 + frag_half * 4 + (r % 4)][e];
          *dst = (w == 0 ? 0.0f : *dst) + acc[t][r];
        }
      }
    }
    __syncthreads();
  }
  // groups in order, then the bias
  for (int i = threadIdx.x; i < kTokens * NT * 32; i += 256 * NG) {
    const int t_row = i / (NT * 32), e = i % (NT * 32);
    float v = s_logit[0][t_row][e];
#pragma unroll
    for (int g = 1; g < NG; ++g) v += s_logit[g][t_row][e];
    if (bias && e < n_experts) v += bias[e];
    s_logit[0][t_row][e] = v;
  }
  __syncthreads();
  if (threadIdx.x >= kTokens * kSub) return;
  const int t_local = threadIdx.x / kSub, sub = threadIdx.x % kSub;  // 32 tokens x 8 lanes
  if (tok0 + t_local < n)
    topk_of_token(s_logit[0][t_local], n_experts, top_k, renorm, sub, topk_idx + (tok0 + t_local) * top_k,
                  topk_w + (tok0 + t_local) * top_k);
}

// float32: four waves per block, 32 tokens, each wave 8 tokens; lanes stride over d_model.
__global__ __launch_bounds__(256) void route_f32_kernel(const float* __restrict__ X, int64_t n, int d_model,
                                                        int64_t ldx, const float* __restrict__ R, int64_t ldr,
                                                        const float* __restrict__ bias, int n_experts, int top_k,
                                                        int renorm, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w) {
  __shared__ float s_logit[kTokens][CAMERA_MAX_EXPERTS + 1];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t tok0 = (int64_t)blockIdx.x * kTokens;
  for (int t = 0; t < 8; ++t) {
    const int64_t tok = tok0 + wave * 8 + t;
    if (tok >= n) break;  // wave-uniform
    const float* x = X + tok * ldx;
    for (int e = 0; e < n_experts; ++e) {
      const float* rr = R + (int64_t)e * ldr;
      float s = 0.0f;
      for (int c = lane * 4; c < d_model; c += kWave * 4) {  // d_model is a multiple of 4
        const float4 xv = *reinterpret_cast<const float4*>(x + c);
        const float4 rv = *reinterpret_cast<const float4*>(rr + c);
        s = fmaf(xv.x, rv.x, s);
        s = fmaf(xv.y, rv.y, s);
        s = fmaf(xv.z, rv.z, s);
        s = fmaf(xv.w, rv.w, s);
      }
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
      if (lane == 0) s_logit[wave * 8 + t][e] = s + (bias ? bias[e] : 0.0f);
    }
  }
  __syncthreads();
  const int t_local = threadIdx.x / kSub, sub = threadIdx.x % kSub;  // 256 threads = 32 tokens x 8 lanes
  if (tok0 + t_local < n)
    topk_of_token(s_logit[t_local], n_experts, top_k, renorm, sub, topk_idx + (tok0 + t_local) * top_k,
                  topk_w + (tok0 + t_local) * top_k);
}

template <int NT, int NG>
void launch_bf16(hipStream_t stream, int64_t n_blocks, const void* X, int64_t n, int64_t d_model, int64_t ldx,
                 const void* W_r, int64_t ldr, const float* bias, int n_experts, int top_k, int renorm,
                 const void* zeros, int32_t* topk_idx, float* topk_w) {
  hipLaunchKernelGGL((route_bf16_kernel<NT, NG>), dim3((unsigned)n_blocks), dim3(256 * NG), 0, stream,
                     static_cast<const __hip_bfloat16*>(X), n, (int)d_model, ldx,
                     static_cast<const __hip_bfloat16*>(W_r), ldr, bias, n_experts, top_k, renorm,
                     static_cast<const __hip_bfloat16*>(zeros), topk_idx, topk_w);
}

}  // namespace

hipError_t launch_route_topk(hipStream_t stream, const void* X, int dtype, int64_t n, int64_t d_model,
                             int64_t ldx, const void* W_r, int64_t ldr, const float* bias, int n_experts,
                             int top_k, int renorm, const void* zeros, int32_t* topk_idx, float* topk_w) {
  if (n <= 0) return hipSuccess;
  const int64_t n_blocks = (n + kTokens - 1) / kTokens;
  if (dtype == CAMERA_BF16) {
    const int nt = (n_experts + 31) / 32;
    // two groups of four waves where the logits of both fit the 64 KiB of static LDS; a short d_model is not
    // worth splitting eight ways
    const bool wide = d_model >= 1024;
#define CAMERA_ROUTE_CASE(NT, NG)                                                                                     \
  launch_bf16<NT, NG>(stream, n_blocks, X, n, d_model, ldx, W_r, ldr, bias, n_experts, top_k, renorm, zeros, topk_idx, \
                      topk_w)
    if (nt <= 1) { if (wide) CAMERA_ROUTE_CASE(1, 2); else CAMERA_ROUTE_CASE(1, 1); }
    else if (nt <= 2) { if (wide) CAMERA_ROUTE_CASE(2, 2); else CAMERA_ROUTE_CASE(2, 1); }
    else if (nt <= 4) { if (wide) CAMERA_ROUTE_CASE(4, 2); else CAMERA_ROUTE_CASE(4, 1); }
    else CAMERA_ROUTE_CASE(8, 1);
#undef CAMERA_ROUTE_CASE
  } else {
    hipLaunchKernelGGL(route_f32_kernel, dim3((unsigned)n_blocks), dim3(256), 0, stream,
                       static_cast<const float*>(X), n, (int)d_model, ldx, static_cast<const float*>(W_r), ldr,
                       bias, n_experts, top_k, renorm, topk_idx, topk_w);
  }
  return hipGetLastError();
}

}  // namespace camera

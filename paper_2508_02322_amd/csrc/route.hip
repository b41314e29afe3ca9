// A = Top&Norm(R X): router logits, softmax, top-k and renormalisation
// (Algorithm 1, line 2; the weights A_i(x) of Eq. 2).
//
// Logits L[j, e] = <x_j, R_e> (+ bias_e) are accumulated in float32: for bf16 on
// v_mfma_f32_32x32x16_bf16 (a block = 32 tokens x all experts, K chunks staged
// through LDS, its four waves split each chunk -- R is small and stays in L2),
// for float32 with FMA and a wave reduction.  The logits of a
// block's tokens go through LDS so that eight lanes can walk the experts of
// one token: top_k rounds of "largest remaining logit, lower index on ties".
// Selection is on the logits (softmax is increasing, so this is the top-k of
// the probabilities); the kept weights are exp(L - max) over the softmax
// denominator, renormalised over the kept ones.
#include <hip/hip_bf16.h>

#include <type_traits>

#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// f(integral_constant<int, LO>), ..., f(integral_constant<int, HI - 1>)
template <int LO, int HI, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (LO < HI) {
    f(std::integral_constant<int, LO>{});
    static_for<LO + 1, HI>(f);
  }
}

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

// bf16: 32 tokens per block, NT tiles of 32 experts, K in chunks of KC elements that go through LDS.
// The MFMA operand layout (lane = row, 8 consecutive K elements) makes neighbouring lanes read different rows, i.e.
// a different cache line per lane; fetched that way from global memory a wave instruction costs four times the
// address cycles of a coalesced one.  So the block fetches each chunk coalesced (a row's KC elements by KC / 8
// neighbouring threads, 16 bytes each), PF chunks ahead in registers (a block is alone on its CU for most sizes:
// what hides the latency of HBM is the number of its own loads in flight), stores it to LDS with rows padded by
// 16 bytes (conflict-free fragment reads), and the four waves split the chunk's K steps.
// No load is conditional: a thread whose token, expert or K position lies outside reads a valid address all the
// same (row 0, or a page of zeros for the K tail); what it brings in is never used.  Partial logits of the four
// waves are added through LDS in wave order.
template <int NT>
__global__ __launch_bounds__(256) void route_bf16_kernel(const __hip_bfloat16* __restrict__ X, int64_t n,
                                                         int d_model, int64_t ldx,
                                                         const __hip_bfloat16* __restrict__ R, int64_t ldr,
                                                         const float* __restrict__ bias, int n_experts,
                                                         int top_k, int renorm,
                                                         const __hip_bfloat16* __restrict__ zeros,
                                                         int32_t* __restrict__ topk_idx,
                                                         float* __restrict__ topk_w) {
  constexpr int KC = NT <= 4 ? 128 : 64;            // K elements per chunk
  constexpr int kRowB = KC * 2 + 16;                // bytes of a padded LDS row
  constexpr int kVecs = KC / 8;                     // 16-byte vectors per row
  constexpr int kRowsPerPass = 256 / kVecs;         // rows the block fetches per pass
  constexpr int kXPasses = kTokens / kRowsPerPass;
  constexpr int kRPasses = NT * 32 / kRowsPerPass;
  constexpr int kStepsPerWave = KC / 16 / 4;        // MFMA K steps of a chunk per wave
  constexpr int kTileBytes = (kTokens + NT * 32) * kRowB;
  constexpr int kLogitBytes = kTokens * (NT * 32 + 1) * 4;
  // the logits of the block's tokens lie over the chunk buffers: they are written after the last chunk was read
  __shared__ __align__(16) unsigned char s_raw[kTileBytes > kLogitBytes ? kTileBytes : kLogitBytes];
  unsigned char* s_x = s_raw;
  unsigned char* s_r = s_raw + kTokens * kRowB;
  float (*s_logit)[NT * 32 + 1] = reinterpret_cast<float (*)[NT * 32 + 1]>(s_raw);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int frag_row = lane % 32, frag_half = lane / 32;
  const int64_t tok0 = (int64_t)blockIdx.x * kTokens;

  // fetch side: this thread's vector of every row it brings in
  const int vec = threadIdx.x % kVecs, row0 = threadIdx.x / kVecs;
  const __hip_bfloat16* x_src[kXPasses];
  const __hip_bfloat16* r_src[kRPasses];
#pragma unroll
  for (int p = 0; p < kXPasses; ++p) {
    const int64_t tok = tok0 + row0 + p * kRowsPerPass;
    x_src[p] = X + (tok < n ? tok : 0) * ldx + vec * 8;
  }
#pragma unroll
  for (int p = 0; p < kRPasses; ++p) {
    const int e = row0 + p * kRowsPerPass;
    r_src[p] = R + (int64_t)(e < n_experts ? e : 0) * ldr + vec * 8;
  }
  constexpr int PF = NT <= 2 ? 4 : 2;               // chunks in flight
  u32x4 xv[PF][kXPasses], rv[PF][kRPasses];
  auto fetch = [&](auto slot, int k0) {              // chunks past the end read the zero page
    constexpr int u = decltype(slot)::value;
    const bool k_ok = k0 + vec * 8 < d_model;        // d_model is a multiple of 8
#pragma unroll
    for (int p = 0; p < kXPasses; ++p) xv[u][p] = *reinterpret_cast<const u32x4*>(k_ok ? x_src[p] + k0 : zeros);
#pragma unroll
    for (int p = 0; p < kRPasses; ++p) rv[u][p] = *reinterpret_cast<const u32x4*>(k_ok ? r_src[p] + k0 : zeros);
  };
  auto stage = [&](auto slot) {
    constexpr int u = decltype(slot)::value;
#pragma unroll
    for (int p = 0; p < kXPasses; ++p)
      *reinterpret_cast<u32x4*>(s_x + (row0 + p * kRowsPerPass) * kRowB + vec * 16) = xv[u][p];
#pragma unroll
    for (int p = 0; p < kRPasses; ++p)
      *reinterpret_cast<u32x4*>(s_r + (row0 + p * kRowsPerPass) * kRowB + vec * 16) = rv[u][p];
  };

  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

  const int n_chunks = (d_model + KC - 1) / KC;
  static_for<0, PF>([&](auto u) { fetch(u, decltype(u)::value * KC); });
  for (int c0 = 0; c0 < n_chunks; c0 += PF) {
    static_for<0, PF>([&](auto u) {
      const int c = c0 + decltype(u)::value;
      if (c < n_chunks) {  // block-uniform
        stage(u);          // waits for this slot's loads only: the younger chunks stay in flight
        __syncthreads();
        fetch(u, (c + PF) * KC);
#pragma unroll
        for (int i = 0; i < kStepsPerWave; ++i) {
          const int col = ((wave * kStepsPerWave + i) * 16 + frag_half * 8) * 2;  // byte column of this lane's K elements
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(s_x + frag_row * kRowB + col);
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(s_r + (t * 32 + frag_row) * kRowB + col);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
          }
        }
        __syncthreads();  // every wave has read the chunk (after the last one: the logits may overwrite it)
      }
    });
  }
  // accumulator register r of lane l: token row 8*(r/4) + 4*(l/32) + (r%4), expert column l % 32
  for (int w = 0; w < 4; ++w) {  // fixed order: wave 0 stores (with the bias), waves 1..3 add
    if (wave == w) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int e = t * 32 + frag_row;
        const float b = (w == 0 && bias && e < n_experts) ? bias[e] : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float* dst = &s_logit[(r / 4) * 8 + frag_half * 4 + (r % 4)][e];
          *dst = (w == 0 ? 0.0f : *dst) + acc[t][r] + b;
        }
      }
    }
    __syncthreads();
  }
  const int t_local = threadIdx.x / kSub, sub = threadIdx.x % kSub;  // 256 threads = 32 tokens x 8 lanes
  if (tok0 + t_local < n)
    topk_of_token(s_logit[t_local], n_experts, top_k, renorm, sub, topk_idx + (tok0 + t_local) * top_k,
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

template <int NT>
void launch_bf16(hipStream_t stream, int64_t n_blocks, const void* X, int64_t n, int64_t d_model, int64_t ldx,
                 const void* W_r, int64_t ldr, const float* bias, int n_experts, int top_k, int renorm,
                 const void* zeros, int32_t* topk_idx, float* topk_w) {
  hipLaunchKernelGGL(route_bf16_kernel<NT>, dim3((unsigned)n_blocks), dim3(256), 0, stream,
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
#define CAMERA_ROUTE_CASE(NT)                                                                                        \
  launch_bf16<NT>(stream, n_blocks, X, n, d_model, ldx, W_r, ldr, bias, n_experts, top_k, renorm, zeros, topk_idx, \
                  topk_w)
    if (nt <= 1) CAMERA_ROUTE_CASE(1);
    else if (nt <= 2) CAMERA_ROUTE_CASE(2);
    else if (nt <= 4) CAMERA_ROUTE_CASE(4);
    else CAMERA_ROUTE_CASE(8);
#undef CAMERA_ROUTE_CASE
  } else {
    hipLaunchKernelGGL(route_f32_kernel, dim3((unsigned)n_blocks), dim3(256), 0, stream,
                       static_cast<const float*>(X), n, (int)d_model, ldx, static_cast<const float*>(W_r), ldr,
                       bias, n_experts, top_k, renorm, topk_idx, topk_w);
  }
  return hipGetLastError();
}

}  // namespace camera

// C ABI of libcamera_hip: argument checks on the host, workspace carving and
// the launch sequence of each entry point.  Declarations and the meaning of
// every argument are in include/camera.h.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "camera_internal.h"

struct camera_ctx {
  int device = 0;
  char err[512] = {0};
  void* ws = nullptr;
  size_t ws_bytes = 0;
  void* zeros = nullptr;                         // 256 zero bytes, made on first use
  void* rank_state = nullptr;                    // persistent select state of the ranking kernels (zero when made, self-cleaning)
  bool rank_dirty = false;                       // a ranking call failed between its passes: clear the state before the next
  bool profiling = false;
  struct Span {
    hipEvent_t begin, end;
  };
  std::vector<Span> spans[CAMERA_K_COUNT];       // recorded, not yet read
  std::vector<Span> free_spans;                  // reusable event pairs
};

// Scratch of camera_select_prune_noalloc: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; the device address it yields (one per device) is what the
// kernels and every other HIP call are given.
constexpr size_t kScratchBytes = 1536 * 1024;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
bool g_scratch_dirty[kMaxDevices] = {false};

char g_create_error[256] = {0};

int fail(camera_ctx* ctx, int code, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_create_error;
  const size_t cap = ctx ? sizeof(ctx->err) : sizeof(g_create_error);
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, cap, fmt, ap);
  va_end(ap);
  return code;
}

int fail_hip(camera_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, CAMERA_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define CAMERA_HIP(call, what)                          \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, what); \
  } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Makes ctx->device current for the duration of a call and restores the caller's device.
struct DeviceGuard {
  int prev = -1;
  bool changed = false;
  hipError_t enter(int device) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != device) {
      e = hipSetDevice(device);
      changed = e == hipSuccess;
    }
    return e;
  }
  ~DeviceGuard() {
    if (changed) (void)hipSetDevice(prev);
  }
};

// Bump allocator over the context workspace; sizes are rounded up to 256 bytes.
struct Carver {
  size_t used = 0;
  size_t take(size_t bytes) {
    const size_t at = used;
    used += (bytes + 255) & ~size_t(255);
    return at;
  }
};

// Workspace offsets of the bucket tables of one call, taken from a Carver, and the tables once the workspace exists.
struct BucketPlan {
  bool dense = false, slots = false;
  size_t counts = 0, offsets = 0, tile_off = 0, tile_exp = 0, perm = 0, wperm = 0, slot = 0, hist = 0;
  // n_experts groups of pairs; dense: no permutation (every expert sees tokens 0..n-1); slots: also the slot of
  // every pair (the layer output needs it to sum a token's experts)
  void take(Carver& cv, bool dense_, bool slots_, int n_experts, int64_t n_pairs, int max_tiles, int64_t n_blocks) {
    dense = dense_;
    slots = slots_ && !dense_;
    counts = cv.take(sizeof(int32_t) * n_experts);
    offsets = cv.take(sizeof(int32_t) * (n_experts + 1));
    tile_off = cv.take(sizeof(int32_t) * (n_experts + 1));
    tile_exp = cv.take(sizeof(int32_t) * (max_tiles + 1));
    perm = cv.take(dense ? 0 : sizeof(int32_t) * n_pairs);
    wperm = cv.take(dense ? 0 : sizeof(float) * n_pairs);
    slot = cv.take(slots ? sizeof(int32_t) * n_pairs : 0);
    hist = cv.take(sizeof(int32_t) * n_blocks * n_experts);
  }
  camera::BucketTables bind(char* ws, const void* zeros) const {
    camera::BucketTables t;
    t.counts = reinterpret_cast<int32_t*>(ws + counts);
    t.offsets = reinterpret_cast<int32_t*>(ws + offsets);
    t.tile_offset = reinterpret_cast<int32_t*>(ws + tile_off);
    t.tile_expert = reinterpret_cast<int32_t*>(ws + tile_exp);
    t.perm = dense ? nullptr : reinterpret_cast<int32_t*>(ws + perm);
    t.w_perm = dense ? nullptr : reinterpret_cast<float*>(ws + wperm);
    t.slot_of = slots ? reinterpret_cast<int32_t*>(ws + slot) : nullptr;
    t.block_hist = reinterpret_cast<int32_t*>(ws + hist);
    t.zeros = zeros;
    return t;
  }
};

int ensure_workspace(camera_ctx* ctx, size_t bytes) {
  if (ctx->zeros == nullptr) {
    hipError_t e = hipMalloc(&ctx->zeros, 256);
    if (e == hipSuccess) e = hipMemset(ctx->zeros, 0, 256);
    if (e == hipSuccess) e = hipDeviceSynchronize();  // once: visible to every stream from here on
    if (e != hipSuccess) {
      if (ctx->zeros) (void)hipFree(ctx->zeros);
      ctx->zeros = nullptr;
      (void)hipGetLastError();
      return fail(ctx, CAMERA_EWORKSPACE, "zero page: %s", hipGetErrorString(e));
    }
  }
  if (bytes <= ctx->ws_bytes) return CAMERA_OK;
  if (ctx->ws) {
    hipError_t e = hipFree(ctx->ws);  // waits for the device: earlier calls are done with it
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    if (e != hipSuccess) return fail_hip(ctx, e, "hipFree(workspace)");
  }
  const size_t want = bytes + bytes / 4 + (1u << 20);
  hipError_t e = hipMalloc(&ctx->ws, want);
  if (e != hipSuccess) {
    ctx->ws = nullptr;
    (void)hipGetLastError();
    return fail(ctx, CAMERA_EWORKSPACE, "workspace of %zu bytes: %s", want, hipGetErrorString(e));
  }
  ctx->ws_bytes = want;
  return CAMERA_OK;
}

int ensure_rank_state(camera_ctx* ctx) {
  if (ctx->rank_state != nullptr) return CAMERA_OK;
  const size_t bytes = camera::rank_state_bytes();
  hipError_t e = hipMalloc(&ctx->rank_state, bytes);
  if (e == hipSuccess) e = hipMemset(ctx->rank_state, 0, bytes);
  if (e == hipSuccess) e = hipDeviceSynchronize();  // once: visible to every stream from here on
  if (e != hipSuccess) {
    if (ctx->rank_state) (void)hipFree(ctx->rank_state);
    ctx->rank_state = nullptr;
    (void)hipGetLastError();
    return fail(ctx, CAMERA_EWORKSPACE, "select state: %s", hipGetErrorString(e));
  }
  return CAMERA_OK;
}

// Event bracket around one launch group when profiling is on.
struct Bracket {
  camera_ctx* ctx;
  hipStream_t stream;
  int id;
  camera_ctx::Span span{};
  bool live = false;
  Bracket(camera_ctx* c, hipStream_t s, int kernel_id) : ctx(c), stream(s), id(kernel_id) {
    if (!ctx->profiling) return;
    if (!ctx->free_spans.empty()) {
      span = ctx->free_spans.back();
      ctx->free_spans.pop_back();
    } else if (hipEventCreate(&span.begin) != hipSuccess || hipEventCreate(&span.end) != hipSuccess) {
      return;
    }
    live = hipEventRecord(span.begin, stream) == hipSuccess;
  }
  ~Bracket() {
    if (!live) return;
    if (hipEventRecord(span.end, stream) == hipSuccess) ctx->spans[id].push_back(span);
  }
};

int check_common(camera_ctx* ctx, const void* X, int dtype, int64_t n, int64_t d_model, int64_t ldx) {
  if (dtype != CAMERA_F32 && dtype != CAMERA_BF16) return fail(ctx, CAMERA_EDTYPE, "dtype: unknown code %d", dtype);
  if (n < 0) return fail(ctx, CAMERA_EINVAL, "n: negative");
  if (d_model <= 0) return fail(ctx, CAMERA_EINVAL, "d_model: must be positive");
  const int v = dtype == CAMERA_BF16 ? 8 : 4;
  if (d_model % v != 0) return fail(ctx, CAMERA_ESHAPE, "d_model: must be a multiple of %d for this dtype", v);
  if (ldx < d_model || ldx % v != 0) return fail(ctx, CAMERA_ESHAPE, "ldx: must be >= d_model and a multiple of %d", v);
  if (d_model > (1 << 24)) return fail(ctx, CAMERA_ESHAPE, "d_model: too large");
  if (n > 0 && X == nullptr) return fail(ctx, CAMERA_EINVAL, "X: NULL");
  if (!aligned16(X)) return fail(ctx, CAMERA_ESHAPE, "X: not 16-byte aligned");
  return CAMERA_OK;
}

int64_t floor_count(double fraction, int64_t n) { return (int64_t)std::floor(fraction * (double)n + 1e-6); }

int check_segments(camera_ctx* ctx, const int64_t* seg_offsets, int n_seg, int64_t n_micro, camera::SegTable* out) {
  if (n_seg < 1 || n_seg > CAMERA_MAX_SEGMENTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_seg: must be in [1, %d]", CAMERA_MAX_SEGMENTS);
  if (seg_offsets == nullptr) return fail(ctx, CAMERA_EINVAL, "seg_offsets: NULL");
  if (seg_offsets[0] != 0 || seg_offsets[n_seg] != n_micro)
    return fail(ctx, CAMERA_EINVAL, "seg_offsets: must start at 0 and end at n_micro");
  out->n_seg = n_seg;
  for (int s = 0; s <= n_seg; ++s) {
    if (s > 0 && seg_offsets[s] < seg_offsets[s - 1]) return fail(ctx, CAMERA_EINVAL, "seg_offsets: not rising");
    out->off[s] = (int32_t)seg_offsets[s];
  }
  return CAMERA_OK;
}

int check_energy(camera_ctx* ctx, const float* energy, int64_t n_micro) {
  if (n_micro < 0) return fail(ctx, CAMERA_EINVAL, "n_micro: negative");
  if (n_micro >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "n_micro: too large");
  if (n_micro > 0 && energy == nullptr) return fail(ctx, CAMERA_EINVAL, "energy: NULL");
  if (!aligned16(energy)) return fail(ctx, CAMERA_ESHAPE, "energy: not 16-byte aligned");
  return CAMERA_OK;
}

}  // namespace

extern "C" {

int camera_version(void) { return 1; }

int camera_create(camera_ctx** out, int device) {
  if (out == nullptr) return fail(nullptr, CAMERA_EINVAL, "out: NULL");
  *out = nullptr;
  if (device < 0) return fail(nullptr, CAMERA_EINVAL, "device: negative");
  camera_ctx* ctx = new (std::nothrow) camera_ctx();
  if (!ctx) return fail(nullptr, CAMERA_EWORKSPACE, "out of host memory");
  ctx->device = device;
  *out = ctx;
  return CAMERA_OK;
}

int camera_destroy(camera_ctx* ctx) {
  if (ctx == nullptr) return CAMERA_OK;
  int rc = CAMERA_OK;
  if (ctx->ws || ctx->zeros || ctx->rank_state || !ctx->free_spans.empty()) {
    DeviceGuard guard;
    (void)guard.enter(ctx->device);
    for (auto& v : ctx->spans)
      for (auto& s : v) ctx->free_spans.push_back(s);
    for (auto& s : ctx->free_spans) {
      (void)hipEventDestroy(s.begin);
      (void)hipEventDestroy(s.end);
    }
    if (ctx->ws && hipFree(ctx->ws) != hipSuccess) rc = CAMERA_EHIP;
    if (ctx->zeros && hipFree(ctx->zeros) != hipSuccess) rc = CAMERA_EHIP;
    if (ctx->rank_state && hipFree(ctx->rank_state) != hipSuccess) rc = CAMERA_EHIP;
  }
  delete ctx;
  return rc;
}

const char* camera_last_error(const camera_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

int camera_profile_enable(camera_ctx* ctx, int on) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  ctx->profiling = on != 0;
  return CAMERA_OK;
}

int camera_profile_read(camera_ctx* ctx, int kernel_id, double* total_ms, int64_t* launches) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (kernel_id < 0 || kernel_id >= CAMERA_K_COUNT) return fail(ctx, CAMERA_EINVAL, "kernel_id: out of range");
  if (total_ms == nullptr || launches == nullptr) return fail(ctx, CAMERA_EINVAL, "total_ms / launches: NULL");
  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  double sum = 0.0;
  int64_t count = 0;
  for (auto& s : ctx->spans[kernel_id]) {
    CAMERA_HIP(hipEventSynchronize(s.end), "hipEventSynchronize");
    float ms = 0.0f;
    CAMERA_HIP(hipEventElapsedTime(&ms, s.begin, s.end), "hipEventElapsedTime");
    sum += ms;
    ++count;
    ctx->free_spans.push_back(s);
  }
  ctx->spans[kernel_id].clear();
  *total_ms = sum;
  *launches = count;
  return CAMERA_OK;
}

int camera_gather_micro_experts(camera_ctx* ctx, void* stream_, int dtype, int n_experts, int64_t d_ff,
                                int64_t d_model, const void* W_gate, const void* W_up, int64_t stride_gu,
                                const void* W_down, int64_t stride_down, const int32_t* index, int64_t n_index,
                                int64_t index_base, const int32_t* count, int down_row_align, void* W_gate_out,
                                void* W_up_out, void* W_down_out) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (dtype != CAMERA_F32 && dtype != CAMERA_BF16) return fail(ctx, CAMERA_EDTYPE, "dtype: unknown code %d", dtype);
  if (down_row_align < 1 || down_row_align > CAMERA_MAX_ROW_ALIGN)
    return fail(ctx, CAMERA_EINVAL, "down_row_align: must be in [1, %d]", CAMERA_MAX_ROW_ALIGN);
  const int es = dtype == CAMERA_BF16 ? 2 : 4;
  if (n_experts < 1 || n_experts > CAMERA_MAX_EXPERTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_experts: must be in [1, %d]", CAMERA_MAX_EXPERTS);
  if (d_ff < 1 || d_model < 1) return fail(ctx, CAMERA_ESHAPE, "d_ff / d_model: must be positive");
  if (d_ff * es > 65536) return fail(ctx, CAMERA_EUNSUPPORTED, "d_ff: a W_down row must not exceed 65536 bytes");
  if ((d_model * es) % 16 != 0) return fail(ctx, CAMERA_ESHAPE, "d_model: rows must be whole 16-byte vectors");
  if (n_index < 0 || n_index > (int64_t)n_experts * d_ff)
    return fail(ctx, CAMERA_EINVAL, "n_index: must be in [0, n_experts * d_ff]");
  if (count == nullptr && n_index != (int64_t)n_experts * d_ff)
    return fail(ctx, CAMERA_EINVAL, "count: NULL needs n_index == n_experts * d_ff");
  if ((n_index + (int64_t)n_experts * down_row_align) * d_model >= (int64_t(1) << 40))
    return fail(ctx, CAMERA_ESHAPE, "n_index * d_model: too large");
  if (index_base < 0 || index_base > (int64_t(1) << 31) - (int64_t)n_experts * d_ff)
    return fail(ctx, CAMERA_EINVAL, "index_base: indices must fit 32 bits");
  const bool rows = W_gate_out != nullptr || W_up_out != nullptr;
  if (W_gate_out != nullptr && W_gate == nullptr) return fail(ctx, CAMERA_EINVAL, "W_gate: NULL");
  if (W_up_out != nullptr && W_up == nullptr) return fail(ctx, CAMERA_EINVAL, "W_up: NULL");
  if (W_down_out != nullptr && W_down == nullptr) return fail(ctx, CAMERA_EINVAL, "W_down: NULL");
  if (rows && (stride_gu < d_ff * d_model || (stride_gu * es) % 16 != 0))
    return fail(ctx, CAMERA_ESHAPE, "stride_gu: must be >= d_ff * d_model and a whole number of 16-byte vectors");
  if (W_down_out != nullptr && stride_down < d_ff * d_model)
    return fail(ctx, CAMERA_ESHAPE, "stride_down: must be >= d_model * d_ff");
  if ((W_gate_out && (!aligned16(W_gate) || !aligned16(W_gate_out))) || (W_up_out && (!aligned16(W_up) || !aligned16(W_up_out))))
    return fail(ctx, CAMERA_ESHAPE, "W_gate / W_up / their outputs: not 16-byte aligned");
  if (n_index == 0 || (!rows && W_down_out == nullptr)) return CAMERA_OK;
  if (index == nullptr) return fail(ctx, CAMERA_EINVAL, "index: NULL");

  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  Carver cv;
  const size_t o_off = cv.take(sizeof(int32_t) * (CAMERA_MAX_EXPERTS + 1));
  const size_t o_off_ld = cv.take(sizeof(int32_t) * (CAMERA_MAX_EXPERTS + 1));
  if (int rc = ensure_workspace(ctx, cv.used)) return rc;
  int32_t* off = reinterpret_cast<int32_t*>(static_cast<char*>(ctx->ws) + o_off);
  int32_t* off_ld = reinterpret_cast<int32_t*>(static_cast<char*>(ctx->ws) + o_off_ld);
  Bracket bracket(ctx, stream, CAMERA_K_GATHER);
  CAMERA_HIP(camera::launch_gather_offsets(stream, count, n_experts, d_ff, down_row_align, off, off_ld),
             "gather offsets");
  CAMERA_HIP(camera::launch_gather_rows(stream, dtype, W_gate, W_up, stride_gu, n_experts, d_ff, d_model, index, n_index,
                                        index_base, off, W_gate_out, W_up_out),
             "gather rows");
  CAMERA_HIP(camera::launch_gather_cols(stream, dtype, W_down, stride_down, n_experts, d_ff, d_model, index, n_index,
                                        index_base, off, off_ld, W_down_out),
             "gather columns");
  return CAMERA_OK;
}

int camera_route_topk(camera_ctx* ctx, void* stream_, const void* X, int dtype, int64_t n, int64_t d_model,
                      int64_t ldx, const void* W_r, int64_t ldr, const float* bias, int n_experts, int top_k,
                      int renorm, int32_t* topk_idx, float* topk_w) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (int rc = check_common(ctx, X, dtype, n, d_model, ldx)) return rc;
  if (n_experts < 1 || n_experts > CAMERA_MAX_EXPERTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_experts: must be in [1, %d]", CAMERA_MAX_EXPERTS);
  if (top_k < 1 || top_k > n_experts) return fail(ctx, CAMERA_EINVAL, "top_k: must be in [1, n_experts]");
  if (W_r == nullptr) return fail(ctx, CAMERA_EINVAL, "W_r: NULL");
  const int v = dtype == CAMERA_BF16 ? 8 : 4;
  if (ldr < d_model || ldr % v != 0) return fail(ctx, CAMERA_ESHAPE, "ldr: must be >= d_model and a multiple of %d", v);
  if (!aligned16(W_r)) return fail(ctx, CAMERA_ESHAPE, "W_r: not 16-byte aligned");
  if (n > 0 && (topk_idx == nullptr || topk_w == nullptr)) return fail(ctx, CAMERA_EINVAL, "topk_idx / topk_w: NULL");
  if (n * (int64_t)top_k >= (int64_t(1) << 31)) return fail(ctx, CAMERA_ESHAPE, "n * top_k: must be below 2^31");
  if (n == 0) return CAMERA_OK;

  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  if (int rc = ensure_workspace(ctx, 0)) return rc;  // the zero page
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  Bracket b(ctx, stream, CAMERA_K_ROUTE);
  CAMERA_HIP(camera::launch_route_topk(stream, X, dtype, n, d_model, ldx, W_r, ldr, bias, n_experts, top_k, renorm,
                                       ctx->zeros, topk_idx, topk_w),
             "route_topk launch");
  return CAMERA_OK;
}

int camera_score_layer(camera_ctx* ctx, void* stream_, const void* X, int dtype, int64_t n, int64_t d_model,
                       int64_t ldx, const int32_t* topk_idx, const float* topk_w, int top_k, int n_experts,
                       int64_t d_ff, const void* W_gate, const void* W_up, int64_t stride_gu, const void* W_down,
                       int64_t stride_down, float alpha, int flags, float* phi2, float* phi_inf, float* omega2,
                       float* energy) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (int rc = check_common(ctx, X, dtype, n, d_model, ldx)) return rc;
  const bool dense = topk_idx == nullptr && topk_w == nullptr;
  if (!dense && (topk_idx == nullptr || topk_w == nullptr))
    return fail(ctx, CAMERA_EINVAL, "topk_idx / topk_w: give both or neither");
  if (n_experts < 1 || n_experts > CAMERA_MAX_EXPERTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_experts: must be in [1, %d]", CAMERA_MAX_EXPERTS);
  if (!dense && (top_k < 1 || top_k > n_experts)) return fail(ctx, CAMERA_EINVAL, "top_k: must be in [1, n_experts]");
  if (d_ff <= 0) return fail(ctx, CAMERA_EINVAL, "d_ff: must be positive");
  if (flags & ~(CAMERA_ACCUMULATE | CAMERA_NO_FINALIZE)) return fail(ctx, CAMERA_EINVAL, "flags: unknown bits");
  if (!(alpha >= 0.0f && alpha <= 1.0f)) return fail(ctx, CAMERA_EINVAL, "alpha: must be in [0, 1]");
  const bool finalize = !(flags & CAMERA_NO_FINALIZE);
  const bool accumulate = (flags & CAMERA_ACCUMULATE) != 0;
  if (W_gate == nullptr || W_up == nullptr) return fail(ctx, CAMERA_EINVAL, "W_gate / W_up: NULL");
  if (finalize && W_down == nullptr) return fail(ctx, CAMERA_EINVAL, "W_down: NULL");
  if (phi2 == nullptr || phi_inf == nullptr) return fail(ctx, CAMERA_EINVAL, "phi2 / phi_inf: NULL");
  if (finalize && (omega2 == nullptr || energy == nullptr)) return fail(ctx, CAMERA_EINVAL, "omega2 / energy: NULL");
  const int v = dtype == CAMERA_BF16 ? 8 : 4;
  if (stride_gu < d_ff * d_model || stride_gu % v != 0)
    return fail(ctx, CAMERA_ESHAPE, "stride_gu: must be >= d_ff*d_model and a multiple of %d", v);
  if (finalize && stride_down < d_ff * d_model) return fail(ctx, CAMERA_ESHAPE, "stride_down: must be >= d_model*d_ff");
  if (!aligned16(W_gate) || !aligned16(W_up) || !aligned16(W_down))
    return fail(ctx, CAMERA_ESHAPE, "W_gate / W_up / W_down: not 16-byte aligned");
  const int64_t n_micro = (int64_t)n_experts * d_ff;
  if (n_micro >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "n_experts * d_ff: too large");
  const int64_t n_pairs = dense ? n * n_experts : n * (int64_t)top_k;
  if (n_pairs >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "routed pairs: must be below 2^31");

  const int tile_m = camera::gemm_tile_m(dtype, d_ff);
  const int64_t max_tiles64 = n == 0 ? 0 : (dense ? n_experts * ((n + tile_m - 1) / tile_m) : n_pairs / tile_m + n_experts);
  if (max_tiles64 > 65535)
    return fail(ctx, CAMERA_EUNSUPPORTED, "too many token tiles (%lld) for one call: feed the tokens in chunks with CAMERA_ACCUMULATE",
                (long long)max_tiles64);
  const int max_tiles = (int)max_tiles64;
  const int splits = finalize ? camera::down_norm_splits(n_experts, d_model, d_ff) : 0;
  const int64_t n_blocks = dense ? 0 : camera::bucket_blocks(n_pairs);

  Carver cv;
  BucketPlan plan;
  plan.take(cv, dense, false, n_experts, n_pairs, max_tiles, n_blocks);
  const size_t o_p2 = cv.take(sizeof(float) * (size_t)max_tiles * d_ff);
  const size_t o_pm = cv.take(sizeof(float) * (size_t)max_tiles * d_ff);
  const size_t o_omega = cv.take(sizeof(float) * (size_t)splits * n_micro);

  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  if (int rc = ensure_workspace(ctx, cv.used)) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  const camera::BucketTables t = plan.bind(ws, ctx->zeros);
  float* part_phi2 = reinterpret_cast<float*>(ws + o_p2);
  float* part_max = reinterpret_cast<float*>(ws + o_pm);
  float* omega_part = reinterpret_cast<float*>(ws + o_omega);

  hipStream_t stream = static_cast<hipStream_t>(stream_);
  {
    Bracket b(ctx, stream, CAMERA_K_BUCKET);
    if (dense || n == 0)
      CAMERA_HIP(camera::launch_dense_tables(stream, n, n_experts, tile_m, max_tiles, t), "dense tables launch");
    else
      CAMERA_HIP(camera::launch_bucket(stream, topk_idx, topk_w, n, top_k, n_experts, tile_m, max_tiles, t),
                 "bucket launch");
  }
  if (n > 0) {
    Bracket b(ctx, stream, CAMERA_K_GEMM);
    camera::GemmEpilogue ep;
    ep.part_phi2 = part_phi2;
    ep.part_max = part_max;
    CAMERA_HIP(camera::launch_grouped_gemm(stream, dtype, X, ldx, d_model, d_ff, n_experts, W_gate, W_up, stride_gu,
                                           max_tiles, t, ep),
               "grouped gemm launch");
  }
  if (finalize) {
    Bracket b(ctx, stream, CAMERA_K_DOWN_NORM);
    CAMERA_HIP(camera::launch_down_norm(stream, dtype, W_down, stride_down, n_experts, d_model, d_ff, splits,
                                        omega_part),
               "down norm launch");
  }
  {
    Bracket b(ctx, stream, CAMERA_K_FINALIZE);
    CAMERA_HIP(camera::launch_finalize(stream, n_experts, d_ff, t, part_phi2, part_max, omega_part, splits, alpha,
                                       accumulate ? 1 : 0, finalize ? 1 : 0, phi2, phi_inf, omega2, energy),
               "finalize launch");
  }
  return CAMERA_OK;
}

int camera_input_channel_energy(camera_ctx* ctx, void* stream_, const void* X, int dtype, int64_t n, int64_t d_model,
                                int64_t ldx, const int32_t* topk_idx, int top_k, int n_experts, float* h) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (int rc = check_common(ctx, X, dtype, n, d_model, ldx)) return rc;
  const bool dense = topk_idx == nullptr;
  if (n_experts < 1 || n_experts > CAMERA_MAX_EXPERTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_experts: must be in [1, %d]", CAMERA_MAX_EXPERTS);
  if (!dense && (top_k < 1 || top_k > n_experts)) return fail(ctx, CAMERA_EINVAL, "top_k: must be in [1, n_experts]");
  if (h == nullptr) return fail(ctx, CAMERA_EINVAL, "h: NULL");
  const int64_t n_pairs = dense ? n * n_experts : n * (int64_t)top_k;
  if (n_pairs >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "routed pairs: must be below 2^31");
  const int64_t n_cols = (int64_t)n_experts * d_model;
  if (n_cols >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "n_experts * d_model: too large");
  const int splits = camera::input_energy_splits(n_experts, d_model, dtype);
  const int64_t n_blocks = dense ? 0 : camera::bucket_blocks(n_pairs);
  const int tile_m = 256;                         // the M-tile tables are made but not used here
  const int max_tiles = (int)std::min<int64_t>(65535, n == 0 ? 0 : (dense ? n_experts * ((n + tile_m - 1) / tile_m)
                                                                          : n_pairs / tile_m + n_experts));
  Carver cv;
  BucketPlan plan;
  plan.take(cv, dense, false, n_experts, n_pairs, max_tiles, n_blocks);
  const size_t o_part = cv.take(sizeof(float) * (size_t)splits * n_cols);
  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  if (int rc = ensure_workspace(ctx, cv.used)) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  const camera::BucketTables t = plan.bind(ws, ctx->zeros);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  {
    Bracket b(ctx, stream, CAMERA_K_BUCKET);
    if (dense || n == 0)
      CAMERA_HIP(camera::launch_dense_tables(stream, n, n_experts, tile_m, max_tiles, t), "dense tables launch");
    else
      CAMERA_HIP(camera::launch_bucket(stream, topk_idx, nullptr, n, top_k, n_experts, tile_m, max_tiles, t),
                 "bucket launch");
  }
  Bracket b(ctx, stream, CAMERA_K_DOWN_NORM);
  CAMERA_HIP(camera::launch_input_energy(stream, dtype, X, ldx, n_experts, d_model, t, splits,
                                         reinterpret_cast<float*>(ws + o_part), h),
             "input energy launch");
  return CAMERA_OK;
}

int camera_layer_forward(camera_ctx* ctx, void* stream_, const void* X, int dtype, int64_t n, int64_t d_model,
                         int64_t ldx, const int32_t* topk_idx, const float* topk_w, int top_k, int n_experts,
                         int64_t d_ff, const void* W_gate, const void* W_up, int64_t stride_gu, const void* W_down,
                         int64_t stride_down, const uint8_t* keep_mask, int flags, float* Y) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (int rc = check_common(ctx, X, dtype, n, d_model, ldx)) return rc;
  const bool dense = topk_idx == nullptr && topk_w == nullptr;
  if (!dense && (topk_idx == nullptr || topk_w == nullptr))
    return fail(ctx, CAMERA_EINVAL, "topk_idx / topk_w: give both or neither");
  if (n_experts < 1 || n_experts > CAMERA_MAX_EXPERTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_experts: must be in [1, %d]", CAMERA_MAX_EXPERTS);
  if (!dense && (top_k < 1 || top_k > n_experts)) return fail(ctx, CAMERA_EINVAL, "top_k: must be in [1, n_experts]");
  const int v = dtype == CAMERA_BF16 ? 8 : 4;  // elements per 16 bytes: d_ff is the K extent of the second contraction
  if (d_ff <= 0 || d_ff % v != 0) return fail(ctx, CAMERA_ESHAPE, "d_ff: must be a positive multiple of %d", v);
  if (flags & ~CAMERA_ACCUMULATE) return fail(ctx, CAMERA_EINVAL, "flags: only CAMERA_ACCUMULATE is accepted");
  if (W_gate == nullptr || W_up == nullptr || W_down == nullptr)
    return fail(ctx, CAMERA_EINVAL, "W_gate / W_up / W_down: NULL");
  if (n > 0 && Y == nullptr) return fail(ctx, CAMERA_EINVAL, "Y: NULL");
  if (stride_gu < d_ff * d_model || stride_gu % v != 0)
    return fail(ctx, CAMERA_ESHAPE, "stride_gu: must be >= d_ff*d_model and a multiple of %d", v);
  if (stride_down < d_ff * d_model || stride_down % v != 0)
    return fail(ctx, CAMERA_ESHAPE, "stride_down: must be >= d_model*d_ff and a multiple of %d", v);
  if (!aligned16(W_gate) || !aligned16(W_up) || !aligned16(W_down) || !aligned16(Y))
    return fail(ctx, CAMERA_ESHAPE, "W_gate / W_up / W_down / Y: not 16-byte aligned");
  const int64_t n_micro = (int64_t)n_experts * d_ff;
  if (n_micro >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "n_experts * d_ff: too large");
  const int64_t n_pairs = dense ? n * n_experts : n * (int64_t)top_k;
  if (n_pairs >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "routed pairs: must be below 2^31");
  if (n == 0) return CAMERA_OK;

  const int tile_m = camera::gemm_tile_m(dtype, d_ff);
  const int64_t max_tiles64 = dense ? n_experts * ((n + tile_m - 1) / tile_m) : n_pairs / tile_m + n_experts;
  if (max_tiles64 > 65535)
    return fail(ctx, CAMERA_EUNSUPPORTED, "too many token tiles (%lld) for one call: feed the tokens in chunks",
                (long long)max_tiles64);
  const int max_tiles = (int)max_tiles64;
  const int64_t n_blocks = dense ? 0 : camera::bucket_blocks(n_pairs);

  Carver cv;
  BucketPlan plan;
  plan.take(cv, dense, true, n_experts, n_pairs, max_tiles, n_blocks);
  const size_t es = dtype == CAMERA_BF16 ? 2 : 4;
  const size_t o_hidden = cv.take(es * (size_t)n_pairs * d_ff);
  const size_t o_product = cv.take(sizeof(float) * (size_t)n_pairs * d_model);

  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  if (int rc = ensure_workspace(ctx, cv.used)) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  const camera::BucketTables t = plan.bind(ws, ctx->zeros);
  void* hidden = ws + o_hidden;
  float* product = reinterpret_cast<float*>(ws + o_product);

  hipStream_t stream = static_cast<hipStream_t>(stream_);
  {
    Bracket b(ctx, stream, CAMERA_K_BUCKET);
    if (dense)
      CAMERA_HIP(camera::launch_dense_tables(stream, n, n_experts, tile_m, max_tiles, t), "dense tables launch");
    else
      CAMERA_HIP(camera::launch_bucket(stream, topk_idx, topk_w, n, top_k, n_experts, tile_m, max_tiles, t),
                 "bucket launch");
  }
  {
    Bracket b(ctx, stream, CAMERA_K_GEMM);
    camera::GemmEpilogue ep;
    ep.mode = camera::GemmEpilogue::kHidden;
    ep.hidden = hidden;
    ep.keep = keep_mask;
    CAMERA_HIP(camera::launch_grouped_gemm(stream, dtype, X, ldx, d_model, d_ff, n_experts, W_gate, W_up, stride_gu,
                                           max_tiles, t, ep),
               "hidden gemm launch");
  }
  {
    // Lambda W_down^T: the hidden activations are the left operand (K = d_ff); the two halves of W_down's rows
    // (output columns [0, d_model/2) and [d_model/2, d_model)) take the places of the gate and the up matrix.
    Bracket b(ctx, stream, CAMERA_K_DOWN_GEMM);
    const int64_t half = d_model / 2;
    camera::GemmEpilogue ep;
    ep.mode = camera::GemmEpilogue::kProduct;
    ep.product = product;
    ep.ld_product = d_model;
    ep.col_gap = (int)half;
    const char* wd = static_cast<const char*>(W_down);
    CAMERA_HIP(camera::launch_grouped_gemm(stream, dtype, hidden, d_ff, d_ff, half, n_experts, wd,
                                           wd + es * half * d_ff, stride_down, max_tiles, t, ep),
               "down gemm launch");
  }
  {
    Bracket b(ctx, stream, CAMERA_K_COMBINE);
    CAMERA_HIP(camera::launch_combine(stream, product, t.slot_of, n, top_k, n_experts, d_model,
                                      (flags & CAMERA_ACCUMULATE) ? 1 : 0, Y),
               "combine launch");
  }
  return CAMERA_OK;
}

int camera_layer_forward_compact(camera_ctx* ctx, void* stream_, const void* X, int dtype, int64_t n, int64_t d_model,
                                 int64_t ldx, const int32_t* topk_idx, const float* topk_w, int top_k, int n_experts,
                                 int n_shared, const int32_t* count, int down_row_align, const void* W_gate_c,
                                 const void* W_up_c, const void* W_down_c, int flags, float* Y) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (int rc = check_common(ctx, X, dtype, n, d_model, ldx)) return rc;
  if (dtype != CAMERA_BF16) return fail(ctx, CAMERA_EUNSUPPORTED, "dtype: the compacted layer is built for CAMERA_BF16 only");
  const bool dense = topk_idx == nullptr && topk_w == nullptr;
  if (!dense && (topk_idx == nullptr || topk_w == nullptr))
    return fail(ctx, CAMERA_EINVAL, "topk_idx / topk_w: give both or neither");
  if (n_shared < 0 || (dense && n_shared != 0))
    return fail(ctx, CAMERA_EINVAL, "n_shared: must be >= 0, and 0 without routing (every expert is then dense already)");
  const int total = n_experts + n_shared;
  if (n_experts < 1 || total > CAMERA_MAX_EXPERTS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_experts: must be >= 1, n_experts + n_shared at most %d", CAMERA_MAX_EXPERTS);
  if (!dense && (top_k < 1 || top_k > n_experts)) return fail(ctx, CAMERA_EINVAL, "top_k: must be in [1, n_experts]");
  if (flags & ~CAMERA_ACCUMULATE) return fail(ctx, CAMERA_EINVAL, "flags: only CAMERA_ACCUMULATE is accepted");
  if (count == nullptr) return fail(ctx, CAMERA_EINVAL, "count: NULL");
  if (down_row_align < 1 || down_row_align > CAMERA_MAX_ROW_ALIGN)
    return fail(ctx, CAMERA_EINVAL, "down_row_align: must be in [1, %d]", CAMERA_MAX_ROW_ALIGN);
  camera::CompactRows tab;
  camera::CompactDown tab_down;
  tab.n_experts = tab_down.n_experts = total;
  tab_down.k_round = down_row_align % 64 == 0 ? 64 : 8;
  int64_t rows = 0, tiles = 0, widest = 0, chunks = 0, ld_rows = 0;
  int most_chunks = 1;
  for (int e = 0; e < total; ++e) {
    if (count[e] < 0) return fail(ctx, CAMERA_EINVAL, "count[%d]: negative", e);
    tab.row_off[e] = (int32_t)rows;
    tab.tile_off[e] = (int32_t)tiles;
    tab_down.count[e] = count[e];
    tab_down.ld_off[e] = (int32_t)ld_rows;
    tab_down.chunk_off[e] = (int32_t)chunks;
    rows += count[e];
    ld_rows += ((int64_t)count[e] + down_row_align - 1) / down_row_align * down_row_align;
    tiles += (count[e] + 31) / 32;
    chunks += camera::compact_chunks(count[e]);
    most_chunks = std::max(most_chunks, camera::compact_chunks(count[e]));
    widest = std::max<int64_t>(widest, count[e]);
    if (ld_rows >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "sum of count: too large");
  }
  for (int e = total; e <= CAMERA_MAX_EXPERTS; ++e) {
    tab.row_off[e] = (int32_t)rows;
    tab.tile_off[e] = (int32_t)tiles;
    tab_down.ld_off[e] = (int32_t)ld_rows;
    tab_down.chunk_off[e] = (int32_t)chunks;
    if (e < CAMERA_MAX_EXPERTS) tab_down.count[e] = 0;
  }
  if (rows > 0 && (W_gate_c == nullptr || W_up_c == nullptr || W_down_c == nullptr))
    return fail(ctx, CAMERA_EINVAL, "W_gate_c / W_up_c / W_down_c: NULL");
  if (n > 0 && Y == nullptr) return fail(ctx, CAMERA_EINVAL, "Y: NULL");
  if (!aligned16(W_gate_c) || !aligned16(W_up_c) || !aligned16(W_down_c) || !aligned16(Y))
    return fail(ctx, CAMERA_ESHAPE, "W_gate_c / W_up_c / W_down_c / Y: not 16-byte aligned");
  const int terms = dense ? n_experts : top_k + n_shared;  // experts that every token goes through
  const int64_t n_pairs = n * (int64_t)terms;
  if (n_pairs >= (int64_t(1) << 31) - 1024) return fail(ctx, CAMERA_ESHAPE, "routed pairs: must be below 2^31");
  const int k_round = down_row_align % 64 == 0 ? 64 : 8;  // K granularity of the second contraction on the MFMA path
  const int64_t ldh = (widest + k_round - 1) / k_round * k_round;
  if (n_pairs * std::max<int64_t>(ldh, d_model * most_chunks) >= (int64_t(1) << 38))
    return fail(ctx, CAMERA_EUNSUPPORTED, "batch too large for the compacted layer: use camera_layer_forward");
  if (chunks * ((d_model + 31) / 32) >= (int64_t(1) << 31) - 1024)
    return fail(ctx, CAMERA_ESHAPE, "n_experts * d_model: too large");
  if (n == 0) return CAMERA_OK;

  // grid rows of 32 tokens per expert; the last row also takes what lies beyond it
  const int token_groups = (int)std::min<int64_t>((n + 31) / 32, 64);
  // From about 64 tokens per expert on, the tiles of the grouped MFMA kernel are worth filling: the weights are
  // then read once per 256 tokens of an expert instead of once per 32.  Its 16-byte tile loads need W_down rows
  // that are a multiple of 8 elements long and the two halves of d_model to be multiples of 8.
  const bool mfma = n_pairs / total > 64 && down_row_align % 8 == 0 && d_model % 16 == 0;
  const bool small = !dense && !mfma && n_pairs <= camera::kCompactSmallPairs;  // one-workgroup bucket order, no M-tile tables
  const int tile_m = camera::gemm_tile_m(dtype, widest);  // M tiles of the MFMA path; otherwise only the bucket order is used
  const int64_t max_tiles64 = dense ? n_experts * ((n + tile_m - 1) / tile_m) : n_pairs / tile_m + total;
  if (max_tiles64 > 65535)
    return fail(ctx, CAMERA_EUNSUPPORTED, "batch too large for the compacted layer: use camera_layer_forward");
  const int max_tiles = (int)max_tiles64;
  const int64_t n_blocks = (dense || small) ? 0 : camera::bucket_blocks(n_pairs);
  const bool append = !dense && !small && n_shared > 0;

  Carver cv;
  BucketPlan plan;
  plan.take(cv, dense, true, total, n_pairs, max_tiles, n_blocks);
  const size_t o_idx_aug = cv.take(append ? sizeof(int32_t) * n_pairs : 0);
  const size_t o_w_aug = cv.take(append ? sizeof(float) * n_pairs : 0);
  const size_t o_hidden = cv.take(2 * (size_t)n_pairs * ldh);
  const size_t o_product = cv.take(sizeof(float) * (size_t)(mfma ? 1 : most_chunks) * n_pairs * d_model);
  const size_t o_work = cv.take(sizeof(int32_t) * camera::kCompactGemmScratchWords);

  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  if (int rc = ensure_workspace(ctx, cv.used)) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  const camera::BucketTables t = plan.bind(ws, ctx->zeros);
  void* hidden = ws + o_hidden;
  float* product = reinterpret_cast<float*>(ws + o_product);

  hipStream_t stream = static_cast<hipStream_t>(stream_);
  {
    Bracket b(ctx, stream, CAMERA_K_BUCKET);
    if (dense) {
      CAMERA_HIP(camera::launch_dense_tables(stream, n, n_experts, tile_m, max_tiles, t), "dense tables launch");
    } else if (small) {
      CAMERA_HIP(camera::launch_compact_bucket_small(stream, topk_idx, topk_w, n, top_k, n_experts, n_shared, t),
                 "small bucket launch");
    } else {
      const int32_t* idx = topk_idx;
      const float* wts = topk_w;
      if (append) {
        int32_t* idx_aug = reinterpret_cast<int32_t*>(ws + o_idx_aug);
        float* w_aug = reinterpret_cast<float*>(ws + o_w_aug);
        CAMERA_HIP(camera::launch_compact_append_shared(stream, topk_idx, topk_w, n, top_k, n_experts, n_shared, idx_aug,
                                                        w_aug),
                   "append shared launch");
        idx = idx_aug;
        wts = w_aug;
      }
      CAMERA_HIP(camera::launch_bucket(stream, idx, wts, n, terms, total, tile_m, max_tiles, t), "bucket launch");
    }
  }
  if (mfma) {
    int32_t* work_off = reinterpret_cast<int32_t*>(ws + o_work);
    {
      Bracket b(ctx, stream, CAMERA_K_GEMM);
      CAMERA_HIP(camera::launch_compact_hidden_gemm(stream, X, ldx, d_model, W_gate_c, W_up_c, tab, (int)widest, max_tiles,
                                                    t, work_off, hidden, k_round),
                 "compact hidden gemm launch");
    }
    {
      Bracket b(ctx, stream, CAMERA_K_DOWN_GEMM);
      CAMERA_HIP(camera::launch_compact_down_gemm(stream, hidden, d_model, W_down_c, tab_down, max_tiles, t, work_off,
                                                  product),
                 "compact down gemm launch");
    }
    Bracket b(ctx, stream, CAMERA_K_COMBINE);
    CAMERA_HIP(camera::launch_combine(stream, product, t.slot_of, n, terms, n_experts, d_model,
                                      (flags & CAMERA_ACCUMULATE) ? 1 : 0, Y),
               "combine launch");
    return CAMERA_OK;
  }
  {
    Bracket b(ctx, stream, CAMERA_K_COMPACT_HIDDEN);
    CAMERA_HIP(camera::launch_compact_hidden(stream, X, ldx, d_model, W_gate_c, W_up_c, tab, t, token_groups, hidden,
                                             (int)ldh),
               "compact hidden launch");
  }
  {
    Bracket b(ctx, stream, CAMERA_K_COMPACT_DOWN);
    CAMERA_HIP(camera::launch_compact_down(stream, hidden, (int)ldh, W_down_c, d_model, tab_down, t, token_groups, n_pairs,
                                           product),
               "compact down launch");
  }
  {
    Bracket b(ctx, stream, CAMERA_K_COMBINE);
    CAMERA_HIP(camera::launch_compact_combine(stream, product, tab_down, t, n, terms, d_model, n_pairs,
                                              (flags & CAMERA_ACCUMULATE) ? 1 : 0, Y),
               "compact combine launch");
  }
  return CAMERA_OK;
}

int camera_output_error(camera_ctx* ctx, void* stream_, const float* Y, const float* Y_hat, int64_t n,
                        int64_t d_model, float* per_token) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (n < 0 || d_model < 1) return fail(ctx, CAMERA_ESHAPE, "n / d_model: out of range");
  if (n > 0 && (Y == nullptr || Y_hat == nullptr || per_token == nullptr))
    return fail(ctx, CAMERA_EINVAL, "Y / Y_hat / per_token: NULL");
  if (n == 0) return CAMERA_OK;
  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  Bracket b(ctx, stream, CAMERA_K_COMBINE);
  CAMERA_HIP(camera::launch_output_error(stream, Y, Y_hat, n, d_model, d_model, d_model, per_token),
             "output error launch");
  return CAMERA_OK;
}

}  // extern "C"

namespace {

// The host side of every ranking entry point: the cuts of the pruning ratios and of the precision-level boundaries
// on the common order, the tables that turn a class (number of cuts an element is below) into the two output bytes
// and the per-segment counts, and the launch sequence.
struct RankRequest {
  int n_ratios = 0;             // CAMERA-P: pruning ratios, not falling
  const double* ratios = nullptr;
  bool single_mask = false;     // camera_select_prune: one ratio, the output byte is 1 (kept) / 0, kept_idx may be asked for
  uint8_t* keep_out = nullptr;  // keep_mask or keep_bits
  int32_t* kept = nullptr;      // [n_ratios][n_seg]
  int32_t* kept_idx = nullptr;
  int n_levels = 0;             // CAMERA-Q: precision levels, most important first
  const int* bits = nullptr;
  const double* level_ratios = nullptr;
  uint8_t* bit_of = nullptr;
  int32_t* level_count = nullptr;
  int32_t* perm = nullptr;
  uint32_t* rank = nullptr;     // full ascending rank (camera_select_prune only)
};

int check_ratios(camera_ctx* ctx, const RankRequest& r) {
  if (r.n_ratios > 0) {
    if (r.ratios == nullptr) return fail(ctx, CAMERA_EINVAL, "ratios: NULL");
    for (int k = 0; k < r.n_ratios; ++k) {
      if (!(r.ratios[k] >= 0.0 && r.ratios[k] <= 1.0))
        return fail(ctx, CAMERA_EINVAL, r.single_mask ? "ratio: must be in [0, 1]" : "ratios[%d]: must be in [0, 1]", k);
      if (k > 0 && r.ratios[k] < r.ratios[k - 1]) return fail(ctx, CAMERA_EINVAL, "ratios: must not fall");
    }
  }
  if (r.n_levels > 0) {
    if (r.bits == nullptr || r.level_ratios == nullptr) return fail(ctx, CAMERA_EINVAL, "bits / ratios: NULL");
    double total = 0.0;
    for (int m = 0; m < r.n_levels; ++m) {
      if (!(r.level_ratios[m] >= 0.0)) return fail(ctx, CAMERA_EINVAL, "ratios[%d]: negative", m);
      if (r.bits[m] < 0 || r.bits[m] > 255) return fail(ctx, CAMERA_EINVAL, "bits[%d]: must be in [0, 255]", m);
      total += r.level_ratios[m];
    }
    if (std::fabs(total - 1.0) > 1e-9) return fail(ctx, CAMERA_EINVAL, "ratios: must sum to 1");
  }
  return CAMERA_OK;
}

// Cuts and tables of a request on n_micro keys.  An element of ascending rank r is below a cut iff r < its
// cut rank, so an element below k cuts is below the k cuts of highest rank: sorting the cuts by rank tells, for
// every class k, how many of them are pruning cuts and how many are level boundaries.
//   pruning ratio j:      cut rank floor(ratio_j n + 1e-6); below it = pruned at ratio j
//   level boundary m:     cut rank n - floor((r_1 + .. + r_m) n + 1e-6); below it = not in levels 0 .. m
void plan_cuts(const RankRequest& r, int64_t n_micro, camera::RankCuts* cuts, camera::SegOutputs* seg_out) {
  struct Cut {
    int64_t rank;
    bool prune;
  };
  Cut all[CAMERA_MAX_LEVELS];
  int n = 0;
  for (int k = 0; k < r.n_ratios; ++k) all[n++] = {floor_count(r.ratios[k], n_micro), true};
  double acc = 0.0;
  for (int m = 0; m + 1 < r.n_levels; ++m) {
    acc += r.level_ratios[m];
    all[n++] = {n_micro - floor_count(acc, n_micro), false};
  }
  std::stable_sort(all, all + n, [](const Cut& a, const Cut& b) { return a.rank > b.rank; });  // highest rank first
  memset(cuts, 0, sizeof(*cuts));
  memset(seg_out, 0, sizeof(*seg_out));
  cuts->n_cuts = n;
  for (int q = 0; q < n; ++q) cuts->cut_rank[q] = all[q].rank;
  seg_out->n_classes = n + 1;
  seg_out->n_ratios = r.n_ratios;
  seg_out->n_levels = r.n_levels;
  int prune_below = 0, level = 0;  // of a member of class k: pruning cuts it is below, boundaries it is below
  for (int k = 0; k <= n; ++k) {
    if (k > 0) (all[k - 1].prune ? prune_below : level) += 1;
    // first byte: the keep mask (one ratio) or the keep bits (bit j set iff kept at ratio j: below p pruning cuts
    // means pruned at the p largest ratios); second byte, or the first when no ratio is asked for: the bit width
    const uint8_t keep = r.single_mask ? (prune_below == 0 ? 1 : 0) : (uint8_t)((1u << (r.n_ratios - prune_below)) - 1u);
    const uint8_t width = r.n_levels > 0 ? (uint8_t)r.bits[level] : 0;
    cuts->out_of_below[k] = r.n_ratios > 0 ? keep : width;
    cuts->out2_of_below[k] = width;
    seg_out->prune_cuts_of_class |= (uint32_t)prune_below << (4 * k);
    seg_out->level_of_class |= (uint32_t)level << (4 * k);
  }
  seg_out->kept = r.kept;
  seg_out->level_count = r.level_count;
  seg_out->perm = r.perm;
}

// state: the persistent select state; ws: class bytes + per-call words (+ the sort buffers when rank is asked for)
int launch_rank(camera_ctx* ctx, hipStream_t stream, const float* energy, int64_t n_micro, const camera::SegTable& seg,
                const RankRequest& r, void* state, bool* state_dirty, char* ws) {
  camera::RankCuts cuts;
  camera::SegOutputs seg_out;
  plan_cuts(r, n_micro, &cuts, &seg_out);
  Carver cv;
  const size_t o_class = cv.take((size_t)n_micro + 64);
  const size_t o_words = cv.take(sizeof(int32_t) * camera::rank_workspace_words(n_micro, r.rank ? 1 : 0));
  uint8_t* class_buf = reinterpret_cast<uint8_t*>(ws + o_class);
  int32_t* words = reinterpret_cast<int32_t*>(ws + o_words);
  if (*state_dirty) {  // an earlier call failed between its passes: start from a clean state again
    CAMERA_HIP(hipMemsetAsync(state, 0, camera::rank_state_bytes(), stream), "hipMemsetAsync(select state)");
    *state_dirty = false;
  }
  uint8_t* first = r.n_ratios > 0 ? r.keep_out : r.bit_of;
  uint8_t* second = r.n_ratios > 0 && r.n_levels > 0 ? r.bit_of : nullptr;
  hipError_t e = camera::launch_classify(stream, energy, n_micro, cuts, class_buf, first, second, r.kept_idx, state, words);
  if (e != hipSuccess) {
    *state_dirty = true;
    return fail_hip(ctx, e, "classify launch");
  }
  CAMERA_HIP(camera::launch_segment_outputs(stream, class_buf, seg, seg_out), "segment launch");
  if (r.rank) CAMERA_HIP(camera::launch_full_rank(stream, energy, n_micro, r.rank, words), "rank launch");
  return CAMERA_OK;
}

size_t rank_ws_bytes(int64_t n_micro, bool want_rank) {
  Carver cv;
  cv.take((size_t)n_micro + 64);
  cv.take(sizeof(int32_t) * camera::rank_workspace_words(n_micro, want_rank ? 1 : 0));
  return cv.used;
}

// Checks shared by the ranking entry points, then the launches on the context's workspace and select state.
int run_rank(camera_ctx* ctx, void* stream_, const float* energy, int64_t n_micro, const int64_t* seg_offsets, int n_seg,
             const RankRequest& r) {
  if (int rc = check_energy(ctx, energy, n_micro)) return rc;
  camera::SegTable seg;
  if (int rc = check_segments(ctx, seg_offsets, n_seg, n_micro, &seg)) return rc;
  if (int rc = check_ratios(ctx, r)) return rc;
  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  if (int rc = ensure_workspace(ctx, rank_ws_bytes(n_micro, r.rank != nullptr))) return rc;
  if (int rc = ensure_rank_state(ctx)) return rc;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  Bracket b(ctx, stream, CAMERA_K_RANK);
  return launch_rank(ctx, stream, energy, n_micro, seg, r, ctx->rank_state, &ctx->rank_dirty, static_cast<char*>(ctx->ws));
}

}  // namespace

extern "C" {

int camera_select_prune(camera_ctx* ctx, void* stream_, const float* energy, int64_t n_micro,
                        const int64_t* seg_offsets, int n_seg, double ratio, uint8_t* keep_mask,
                        int32_t* kept_per_expert, int32_t* kept_idx, uint32_t* rank) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (kept_per_expert == nullptr) return fail(ctx, CAMERA_EINVAL, "kept_per_expert: NULL");
  if (n_micro > 0 && keep_mask == nullptr) return fail(ctx, CAMERA_EINVAL, "keep_mask: NULL");
  RankRequest r;
  r.n_ratios = 1;
  r.ratios = &ratio;
  r.single_mask = true;
  r.keep_out = keep_mask;
  r.kept = kept_per_expert;
  r.kept_idx = kept_idx;
  r.rank = rank;
  return run_rank(ctx, stream_, energy, n_micro, seg_offsets, n_seg, r);
}

int camera_select_prune_noalloc(camera_ctx* ctx, void* stream_, const float* energy, int64_t n_micro,
                                const int64_t* seg_offsets, int n_seg, double ratio, uint8_t* keep_mask,
                                int32_t* kept_per_expert, int32_t* kept_idx) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (int rc = check_energy(ctx, energy, n_micro)) return rc;
  if (n_micro > CAMERA_NOALLOC_MAX_MICRO)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_micro: %lld exceeds the %d micro-experts the static scratch is sized for; use camera_select_prune",
                (long long)n_micro, CAMERA_NOALLOC_MAX_MICRO);
  camera::SegTable seg;
  if (int rc = check_segments(ctx, seg_offsets, n_seg, n_micro, &seg)) return rc;
  if (kept_per_expert == nullptr) return fail(ctx, CAMERA_EINVAL, "kept_per_expert: NULL");
  if (n_micro > 0 && keep_mask == nullptr) return fail(ctx, CAMERA_EINVAL, "keep_mask: NULL");
  if (ctx->device >= kMaxDevices) return fail(ctx, CAMERA_EUNSUPPORTED, "device: index above %d", kMaxDevices - 1);
  RankRequest r;
  r.n_ratios = 1;
  r.ratios = &ratio;
  r.single_mask = true;
  r.keep_out = keep_mask;
  r.kept = kept_per_expert;
  r.kept_idx = kept_idx;
  if (int rc = check_ratios(ctx, r)) return rc;
  // the scratch: the select state first, the per-call buffers behind it
  const size_t state_bytes = (camera::rank_state_bytes() + 255) & ~size_t(255);
  const size_t need = state_bytes + rank_ws_bytes(n_micro, false);
  if (need > kScratchBytes)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_micro: needs %zu bytes of scratch, the static buffer has %zu", need, kScratchBytes);
  DeviceGuard guard;
  CAMERA_HIP(guard.enter(ctx->device), "hipSetDevice");
  char* base = nullptr;
  {
    // every GPU has its own copy of the array at its own address: looked up once per device, with that device current
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[ctx->device] == nullptr) {
      void* p = nullptr;
      CAMERA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
      if (p == nullptr) return fail(ctx, CAMERA_EHIP, "hipGetSymbolAddress(scratch): null address");
      g_scratch_ptr[ctx->device] = p;
    }
    base = static_cast<char*>(g_scratch_ptr[ctx->device]);
  }
  // The array starts as zeros and keeps the previous call's contents: the select state at its start cleans itself
  // (every pass leaves its histograms and ticket at zero), class bytes and per-workgroup counts are written before
  // they are read.
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  return launch_rank(ctx, stream, energy, n_micro, seg, r, base, &g_scratch_dirty[ctx->device], base + state_bytes);
}

int camera_select_prune_multi(camera_ctx* ctx, void* stream_, const float* energy, int64_t n_micro,
                              const int64_t* seg_offsets, int n_seg, int n_ratios, const double* ratios,
                              uint8_t* keep_bits, int32_t* kept_per_expert) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (n_ratios < 1 || n_ratios > CAMERA_MAX_LEVELS - 1)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_ratios: must be in [1, %d]", CAMERA_MAX_LEVELS - 1);
  if (kept_per_expert == nullptr) return fail(ctx, CAMERA_EINVAL, "kept_per_expert: NULL");
  if (n_micro > 0 && keep_bits == nullptr) return fail(ctx, CAMERA_EINVAL, "keep_bits: NULL");
  RankRequest r;
  r.n_ratios = n_ratios;
  r.ratios = ratios;
  r.keep_out = keep_bits;
  r.kept = kept_per_expert;
  return run_rank(ctx, stream_, energy, n_micro, seg_offsets, n_seg, r);
}

int camera_alloc_bits(camera_ctx* ctx, void* stream_, const float* energy, int64_t n_micro,
                      const int64_t* seg_offsets, int n_seg, int n_levels, const int* bits, const double* ratios,
                      uint8_t* bit_of, int32_t* level_count, int32_t* perm) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (n_levels < 1 || n_levels > CAMERA_MAX_LEVELS)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_levels: must be in [1, %d]", CAMERA_MAX_LEVELS);
  if (level_count == nullptr) return fail(ctx, CAMERA_EINVAL, "level_count: NULL");
  if (n_micro > 0 && bit_of == nullptr) return fail(ctx, CAMERA_EINVAL, "bit_of: NULL");
  RankRequest r;
  r.n_levels = n_levels;
  r.bits = bits;
  r.level_ratios = ratios;
  r.bit_of = bit_of;
  r.level_count = level_count;
  r.perm = perm;
  return run_rank(ctx, stream_, energy, n_micro, seg_offsets, n_seg, r);
}

int camera_rank_decisions(camera_ctx* ctx, void* stream_, const float* energy, int64_t n_micro,
                          const int64_t* seg_offsets, int n_seg, int n_ratios, const double* ratios,
                          uint8_t* keep_bits, int32_t* kept_per_expert, int n_levels, const int* bits,
                          const double* level_ratios, uint8_t* bit_of, int32_t* level_count, int32_t* perm) {
  if (ctx == nullptr) return fail(nullptr, CAMERA_EINVAL, "ctx: NULL");
  if (n_ratios < 1 || n_levels < 1 || n_ratios + n_levels - 1 > CAMERA_MAX_LEVELS - 1)
    return fail(ctx, CAMERA_EUNSUPPORTED, "n_ratios, n_levels: both >= 1 and n_ratios + n_levels - 1 <= %d cuts in one pass",
                CAMERA_MAX_LEVELS - 1);
  if (kept_per_expert == nullptr || level_count == nullptr) return fail(ctx, CAMERA_EINVAL, "kept_per_expert / level_count: NULL");
  if (n_micro > 0 && (keep_bits == nullptr || bit_of == nullptr)) return fail(ctx, CAMERA_EINVAL, "keep_bits / bit_of: NULL");
  RankRequest r;
  r.n_ratios = n_ratios;
  r.ratios = ratios;
  r.keep_out = keep_bits;
  r.kept = kept_per_expert;
  r.n_levels = n_levels;
  r.bits = bits;
  r.level_ratios = level_ratios;
  r.bit_of = bit_of;
  r.level_count = level_count;
  r.perm = perm;
  return run_rank(ctx, stream_, energy, n_micro, seg_offsets, n_seg, r);
}

}  // extern "C"

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
// bf16: v_mfma_f32_16x16x32_bf16 (64-wide wavefront, fp32 accumulate).  Token
// rows (A operand, gathered through the bucket permutation) and weight rows (B
// operand) are both K-contiguous, so both fragments are 16-byte LDS reads; the
// LDS tiles are [row][8 chunks of 8 bf16] with the chunk index XOR-ed by
// ((row >> 1) & 7): the LDS has 64 four-byte banks, so two 128-byte tile rows
// fill one bank row and 16 consecutive rows reading the same K chunk (one
// quarter of a fragment read) then hit 16 different 16-byte bank groups.
// fp32: plain FMA tiles (used by the float32 configuration only).
#include <hip/hip_bf16.h>

#include <algorithm>
#include <type_traits>

#include "camera_internal.h"

namespace camera {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// acc += x * y on a 16 x 16 x 32 tile, the accumulator held in accumulation registers.  The compiler sees an
// opaque instruction: between the last one and the first read of an accumulator the caller waits out the
// matrix pipe itself (mfma_drain), and no accumulator is used again sooner than eight MFMAs later.
__device__ __forceinline__ void mfma_pinned(f32x4& acc, const bf16x8& x, const bf16x8& y) {
  asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(x), "v"(y));
}
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

// silu(g) = g / (1 + exp(-g)); exp2 and rcp are single hardware instructions (about 1 ulp each)
__device__ __forceinline__ float silu_f32(float g) {
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.
//   A workgroup is WM x WN waves: 2 x 2 in the built configuration, one wave per SIMD, each with the whole
//   register file of its SIMD (256 accumulation registers for its outputs, 256 vector registers for the rest).
//   A wave owns TM 32-row blocks of tokens (blocks wave_m, wave_m + WM, ... of the tile, so that a short last
//   tile of an expert is shared evenly and its empty blocks are skipped) by TN*32 channels, for both the gate
//   and the up product: 128 x 64 x {gate, up}.  Block tile BM = 32*WM*TM tokens by BN = 32*WN*TN channels.
//   The large wave tile is what the kernel is built around: per MFMA it reads a third fewer fragment bytes
//   from LDS than a 64-row wave tile, and on real-valued operands the chip runs at its power limit, where
//   throughput is set by the energy per flop and not by how full the matrix pipe is.
//
//   K advances KT elements per tile.  Token tiles and weight tiles each run through a ring of their own in
//   LDS: two stages of 32 KiB for the token rows and three of 32 KiB (gate + up) for the weights in the built
//   configuration, 160 KiB in all.  The weights stream from HBM exactly once and are loaded two tiles ahead;
//   the token rows, re-read by every channel tile of an expert and so served by the L2, one tile ahead.
//   Tiles go from global memory straight into LDS (global_load_lds_dwordx4, no staging registers, no LDS
//   store instructions).  One workgroup barrier per K tile publishes the next stage; it sits before the last
//   quarter of the K tile so that the first fragments of the next tile are in flight while that quarter's
//   MFMAs run.
//
//   Instruction order.  A wave issues one instruction every fourth cycle at best and, alone on its SIMD, has
//   nobody to cover for it: an MFMA occupies the matrix pipe for 16 cycles, so at most three other
//   instructions fit between two MFMAs before the pipe runs dry.  The K loop is therefore written as a
//   sequence of slots, one MFMA each, followed by at most one fragment read, one tile load or one step of
//   wave-uniform bookkeeping, and the order is pinned with scheduling barriers.  The MFMAs are written as
//   assembly with their accumulators constrained to accumulation registers: left to itself the register
//   allocator moves the 64 accumulator tuples around inside the loop (about 90 copies per 128 MFMAs).
// ---------------------------------------------------------------------------
// f(integral_constant<int, LO>), ..., f(integral_constant<int, HI - 1>)
template <int LO, int HI, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (LO < HI) {
    f(std::integral_constant<int, LO>{});
    static_for<LO + 1, HI>(f);
  }
}

constexpr int kXcds = 8;    // accelerator dies, each with a private L2
constexpr int kPatch = 32;     // workgroups an XCD runs at a time (one per CU)
constexpr int kChunkMax = 6;   // an expert with up to this many M-tiles runs them all side by side
constexpr int kChunkM = 4;     // otherwise this many

// What a tile does with its two accumulator sets (named gate and up after their main use).
//   kEpiStats   : Lambda = a * silu(gate) * up, column sums of Lambda^2 and column maxima -> part_phi2 / part_max
//   kEpiHidden  : the same Lambda, times the keep flag of its micro-expert, rounded to bf16 -> hidden[slot row][channel]
//   kEpiProduct : the plain products -> product[slot row][column] (first B matrix) and [column + col_gap] (second);
//                 the token rows of this mode are the bucket slots themselves (A = the hidden activations)
enum { kEpiStats = 0, kEpiHidden = 1, kEpiProduct = 2 };
struct EpiArgs {
  float* part_phi2;
  float* part_max;
  void* hidden;            // [pairs][ld_hidden], bf16 (MFMA kernel) or float32 (FMA kernel)
  const uint8_t* keep;     // [n_experts * d_ff] or nullptr (all kept)
  float* product;          // [pairs][ld_product]
  int64_t ld_product;
  int col_gap;
  int64_t ld_hidden;       // row stride of hidden (d_ff when every expert has the same width)
  int pad_hidden;          // != 0: columns from d_ff up to the next multiple of it are written as zeros (8 or 64)
};

// One wave instruction of the direct global -> LDS path: lane l's 16 bytes at p (+ IMM) go to LDS bytes
// [16 l, 16 l + 16) behind the wave-uniform LDS byte address lds (+ IMM).  Written as assembly on purpose: the compiler's
// wait-count model takes the builtin for an access to both memory and LDS and from then on turns every wait for
// fragment reads into lgkmcnt(0) and every wait for loads into vmcnt(0), which stalls a wave on the fragment
// reads it has just issued for the next phase.  Issued this way the loads are invisible to that model: the
// waits for them are the explicit vmcnt waits of the K loop, and the fragment waits stay exact.
// M0 holds the LDS address; a scalar write of M0 needs one wait state before an LDS-DMA instruction reads it.
// LDS byte address of a pointer into the workgroup's LDS.  Taken once per tile from the named array: a cast of a
// pointer whose address space the compiler cannot see needs a null check that this compiler version miscompiles.
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const void*)p;
}
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
template <int IMM>
__device__ __forceinline__ void lds_dma16(const unsigned char* p, unsigned lds) {
  const unsigned base = __builtin_amdgcn_readfirstlane(lds);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off offset:%2"
               :
               : "s"(base), "v"(p), "n"(IMM)
               : "memory", "m0");
}
// The same with the address split into a wave-uniform base and the lane's 32-bit byte offset, and with M0 written
// apart: the loads of one matrix follow each other in program order (these statements are volatile, the compiler
// keeps their order and has no use of its own for M0 in these kernels), so one M0 write serves up to four of them.
__device__ __forceinline__ void lds_dma_base(unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(lds) : "memory", "m0");
}
template <int IMM>
__device__ __forceinline__ void lds_dma16_scalar(unsigned offset, const unsigned char* base) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(offset), "s"(base), "n"(IMM) : "memory");
}
#pragma clang diagnostic pop

// STAGES_: ring depth of the token (A) tiles; BSTAGES_: ring depth of the weight tiles, the same or one more
// (weights stream from HBM exactly once and need the longer lead; token rows mostly come from the L2).
template <int WM_, int WN_, int TM_, int TN_, int KT_, int STAGES_, int BSTAGES_ = STAGES_>
struct GemmCfg {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_, KT = KT_, kStages = STAGES_, kBStages = BSTAGES_;
  static constexpr int kWaves = WM * WN;
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int BM = 32 * WM * TM;
  static constexpr int BN = 32 * WN * TN;
  static constexpr int kChunks = KT / 8;          // 16-byte chunks per tile row
  static constexpr int kRowBytes = KT * 2;        // 64 or 128
  static constexpr int kRowsPerBankRow = 256 / kRowBytes;  // tile rows that share one 256-byte LDS bank row
  static constexpr int kSteps = KT / 16;          // MFMA K steps per tile
  static constexpr int kATileBytes = BM * kRowBytes;
  static constexpr int kBTileBytes = BN * kRowBytes;  // one of gate / up
  static constexpr int kStageBytes = kATileBytes + 2 * kBTileBytes;
  // one wave instruction fills 1 KiB of LDS = kDmaRows consecutive tile rows
  static constexpr int kDmaRows = 1024 / kRowBytes;
  static constexpr int kADma = BM / kWaves / kDmaRows;  // instructions per wave per tile, A
  static constexpr int kBDma = BN / kWaves / kDmaRows;  // per weight matrix
  static constexpr int kLoadsPerTile = kADma + 2 * kBDma;
  // LDS: the A stages, then the B stages (gate and up tile of a stage side by side), then the per-tile arrays
  // (token ids, routing weights, column reduction).  When the ring alone fills the 160 KiB the per-tile arrays
  // lie over its first bytes: they are only used before the first tile load and after the last fragment read.
  static constexpr int kBStageBytes = 2 * kBTileBytes;
  static constexpr int kRingBytes = kStages * kATileBytes + kBStages * kBStageBytes;
  static constexpr int kAuxBytes = BM * 8 + 2 * WM * BN * 4;
  static constexpr bool kAliasAux = kRingBytes + kAuxBytes > 160 * 1024;
  static constexpr int kSmemBytes = kAliasAux ? kRingBytes : kRingBytes + kAuxBytes;
  static constexpr int a_off(int stage) { return stage * kATileBytes; }
  static constexpr int b_off(int stage) { return kStages * kATileBytes + stage * kBStageBytes; }
  // Loads that may still be in flight when tile kt + 1 must have landed: a tile's loads are issued token rows
  // first, so these are the whole tiles beyond kt + 1 and, with the deeper weight ring, the weight loads of one more.
  static constexpr int kMayFly = (kStages - 2) * kLoadsPerTile + (kBStages - kStages) * 2 * kBDma;
  // workgroups that fit one CU by LDS (160 KiB), hence waves per SIMD the registers must allow
  static constexpr int kBlocksPerCu = (160 * 1024) / kSmemBytes >= 2 ? 2 : 1;
  static constexpr int kWavesPerSimd = kBlocksPerCu * kWaves / 4 > 0 ? kBlocksPerCu * kWaves / 4 : 1;
  // A tile load is issued behind every kLoadEvery-th MFMA of a full tile, counted from the barrier: densely
  // issued loads hold the wave on the vector-memory queue (every 2nd MFMA: 9 % slower than every 6th), and the
  // last third of the K tile stays free of them (the youngest load's time to land; the bookkeeping of the
  // next fill goes there).
  static constexpr int kLoadEvery = 6;
  static_assert(KT == 32 || KT == 64, "K tile");
  static_assert(kStages >= 2, "at least the stage being read and the stage being filled");
  static_assert(kBStages == kStages || kBStages == kStages + 1, "weight ring: as deep as the token ring or one deeper");
  static_assert(kADma >= 1 && kBDma >= 1 && BM % (kWaves * kDmaRows) == 0 && BN % (kWaves * kDmaRows) == 0,
                "every wave fills whole 1 KiB groups");
  static_assert(kSmemBytes <= 160 * 1024, "LDS per workgroup");
  static_assert(kADma <= 8 && kBDma <= 8, "two LDS bases of four immediate offsets each");
};

// LDS image of a tile: row r is kRowBytes long; its 16-byte chunk c sits at chunk position
// c ^ swizzle_key(r).  The LDS has 64 four-byte banks, so kRowsPerBankRow tile rows share a bank
// row; with this key the 16 rows that a quarter of a fragment read touches (same c) fall on 16
// different 16-byte bank groups.
template <class C>
__device__ __forceinline__ int swizzle_key(int row) {
  return (row / C::kRowsPerBankRow) % C::kChunks;
}

// Everything a workgroup needs after its set-up, so that the K loop can be instantiated
// once per number of active row blocks (ACT) without run-time branches inside it.
template <class C>
struct TileState {
  unsigned char* smem;
  const float* s_a;
  float* s_red;
  // direct-to-LDS sources of this lane's row groups.  Two forms: a 64-bit address per group (TAIL), or a wave-uniform
  // base per matrix -- its start moved back by kBias bytes so that every offset stays positive -- plus a 32-bit
  // byte offset per group.  Either way group j's source is moved back by 1024 (j % 4) bytes, which the immediate
  // offset of its instruction brings back (see dma_one).
  static constexpr int kBias = 4096;
  const __hip_bfloat16* a_src[C::kADma];
  const __hip_bfloat16* g_src[C::kBDma];
  const __hip_bfloat16* u_src[C::kBDma];
  unsigned a_off[C::kADma], b_off[C::kBDma];
  const unsigned char* a_base;
  const unsigned char* g_base;
  const unsigned char* u_base;
  const __hip_bfloat16* zeros;  // 16 readable zero bytes (K tail)
  int a_lds, b_lds;             // byte offset of the wave's first A row / weight row in a tile
  int a_k[C::kADma];            // first K element (inside a tile) each A instruction of this lane reads
  int b_k[C::kBDma];
  int d_model;
  // fragments
  int a_frag_base, b_frag_base;
  int k_swz[C::kSteps];
  int wave_m, wave_n, frag_row, frag_half;
  int expert, m_len, row_first;  // for the epilogues that write per token row
};

// ACT: active 32-row blocks of this wave's accumulators.  DEAD: every token row that this wave
// loads lies past the end of the expert's bucket (a short last tile); such rows only have to hold
// finite values (their routing weight is 0), so they are loaded once, in the prologue, and
// the K loop skips their loads.  TAIL: d_model is not a multiple of the K tile (chunks past it come from a page
// of zeros), or a matrix is too large for 32-bit offsets: per-lane 64-bit sources.
template <class C, int ACT, bool TAIL, bool DEAD, int EPI>
__device__ __forceinline__ void tile_body16(const TileState<C>& st, int n0, int d_ff, int slot, const EpiArgs& ep) {
  constexpr int BN = C::BN, TN = C::TN, WM = C::WM, KT = C::KT;
  constexpr int NA = ACT > 0 ? ACT : 1;
  extern __shared__ __align__(16) unsigned char smem[];  // the workgroup's dynamic LDS, named here so that its address space is known
  const unsigned lds0 = lds_address(smem);
  using std::integral_constant;

  // Lane l of a wave instruction writes LDS bytes [16 l, 16 l + 16) after the wave-uniform base,
  // i.e. chunk position l % kChunks of row l / kChunks of its row group; to produce the swizzled
  // image it reads logical chunk (l % kChunks) ^ swizzle_key(row) of that row (set up by the caller).
  // The instruction's immediate offset is added to the global and to the LDS address alike, so the
  // j-th group of a wave uses immediate 1024 (j % 4) on a source that was moved back by as much at
  // set-up: one LDS base (M0) serves four groups of a matrix (immediates reach 4095 bytes).
  // A fill is what goes into the stages that a barrier has just freed: the next token tile and the next weight
  // tile, each with its own ring position.  All of its fields are wave-uniform.
  struct Fill {
    int a_k, b_k;                                // first K element of either tile
    unsigned a_lds, b_lds;                       // LDS address of this wave's rows in the target stages
    const unsigned char *a_ptr, *g_ptr, *u_ptr;  // matrix bases moved on to a_k / b_k (the scalar-base form)
  };
  auto make_fill = [&](unsigned a_st, int a_k, unsigned b_st, int b_k) {
    Fill f;
    f.a_k = a_k;
    f.b_k = b_k;
    f.a_lds = lds0 + a_st + st.a_lds;
    f.b_lds = lds0 + C::kStages * C::kATileBytes + b_st + st.b_lds;
    f.a_ptr = st.a_base + 2 * (unsigned)a_k;
    f.g_ptr = st.g_base + 2 * (unsigned)b_k;
    f.u_ptr = st.u_base + 2 * (unsigned)b_k;
    return f;
  };
  // Load d of a fill's kLoadsPerTile wave instructions: the token groups first, then the gate groups, then the up
  // groups.  The loads of a fill are issued in this order, everywhere: the scalar-base form writes M0 only with
  // the first of every four groups of a matrix, and the waits of the K loop count on the token rows being the older.
  auto dma_one = [&](const Fill& f, auto index) {
    constexpr int d = decltype(index)::value;
    constexpr bool is_a = d < C::kADma, is_g = !is_a && d < C::kADma + C::kBDma;
    constexpr int j = is_a ? d : (is_g ? d - C::kADma : d - C::kADma - C::kBDma);
    constexpr int kOff = (j % 4) * 1024, kBase = (j / 4) * 4096;
    const unsigned dst = (is_a ? f.a_lds : f.b_lds + (is_g ? 0 : C::kBTileBytes)) + kBase;
    if constexpr (TAIL) {
      const __hip_bfloat16* src;
      int k;
      if constexpr (is_a) {
        src = st.a_src[j];
        k = st.a_k[j];
      } else {
        src = is_g ? st.g_src[j] : st.u_src[j];
        k = st.b_k[j];
      }
      const int k0 = is_a ? f.a_k : f.b_k;
      const unsigned char* p = reinterpret_cast<const unsigned char*>(src + k0);
      p = (k0 + k < st.d_model) ? p : reinterpret_cast<const unsigned char*>(st.zeros) - kOff;
      lds_dma16<kOff>(p, dst);
    } else {
      if constexpr (j % 4 == 0) lds_dma_base(__builtin_amdgcn_readfirstlane(dst));
      if constexpr (is_a) lds_dma16_scalar<kOff>(st.a_off[j], f.a_ptr);
      else lds_dma16_scalar<kOff>(st.b_off[j], is_g ? f.g_ptr : f.u_ptr);
    }
  };
  auto dma_unless_dead = [&](const Fill& f, auto index) {
    if constexpr (!(DEAD && decltype(index)::value < C::kADma)) dma_one(f, index);
  };

  // v_mfma_f32_16x16x32_bf16: a 32 x 32 block of the wave's tile is four 16 x 16 sub-blocks (a: rows, b: columns)
  // and an instruction advances K by 32.  With random operand values this instruction holds a shader clock about
  // 10 % higher than the 32x32x16 one at the same flops (the chip is power-limited), which is why it is used.
  // Which way round a 16 x 16 sub-block lies in the registers.  Statistics: a lane owns one channel and four
  // consecutive token rows (the column reduction starts in the lane).  The epilogues that write per token row take
  // the transposed form, a lane owning one token row and four consecutive channels: its four values are 16
  // contiguous bytes of the output row (8 for bf16), one store instead of four.
  constexpr bool kSwap = EPI != kEpiStats;
  f32x4 acc_g[NA][TN][2][2], acc_u[NA][TN][2][2];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int ab = 0; ab < 4; ++ab)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          acc_g[i][j][ab >> 1][ab & 1][r] = 0.0f;
          acc_u[i][j][ab >> 1][ab & 1][r] = 0.0f;
        }
  // The accumulators take their registers here, before anything else is loaded: otherwise the allocator parks other
  // values in accumulation registers and has to move them to scratch when the accumulators arrive.
  // (The other epilogues hold fewer values through the loop and are better off without.)
  if constexpr (EPI == kEpiStats) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
          asm volatile("" : "+a"(acc_g[i][j][ab >> 1][ab & 1]));
          asm volatile("" : "+a"(acc_u[i][j][ab >> 1][ab & 1]));
        }
  }

  // Lane l holds row (l % 16) of a sub-block, K elements 8*(l / 16) .. +7 of a 32-wide K step.
  struct FragA {
    bf16x8 v[NA][2];  // the token rows of one K step: row block i, sub-block a
  };
  struct FragB {
    bf16x8 g[TN], u[TN];  // 16 channels (sub-block b) of every channel block, one K step
  };
  // Per-lane byte offsets of the fragments inside the LDS: token rows of K step ks in the stage at ring offset
  // a_st; weight rows of (K step ks, channel sub-block b) at b_st.
  auto frag_a_at = [&](unsigned a_st, int ks) { return a_st + (unsigned)(st.k_swz[ks] + st.a_frag_base); };
  auto frag_b_at = [&](unsigned b_st, int ks) {
    return C::kStages * C::kATileBytes + b_st + (unsigned)(st.k_swz[ks] + st.b_frag_base);
  };
  // Read r of a phase's fragment reads: the 2 TN weight fragments (gate and up of every channel block) of
  // channel sub-block b first, then, where a new K step begins, the 2 ACT token fragments.
  auto read_one = [&](FragA& ra, FragB& rb, unsigned at_a, unsigned at_b, auto b_index, auto r_index) {
    constexpr int r = decltype(r_index)::value, b = decltype(b_index)::value;
    if constexpr (r < 2 * TN) {
      constexpr int j = r / 2;
      constexpr int off = b * 16 * C::kRowBytes + j * 32 * C::kRowBytes + (r % 2 ? C::kBTileBytes : 0);
      bf16x8& dst = r % 2 == 0 ? rb.g[j] : rb.u[j];
      dst = *reinterpret_cast<const bf16x8*>(smem + at_b + off);
    } else {
      constexpr int i = (r - 2 * TN) / 2, a = (r - 2 * TN) % 2;
      ra.v[i][a] = *reinterpret_cast<const bf16x8*>(smem + at_a + (i * WM * 32 + a * 16) * C::kRowBytes);
    }
  };
  // MFMA m of one phase (K step ks, channel sub-block b), numbered (row block i, row sub-block a,
  // channel block j, gate / up)
  auto mfma_one = [&](const FragA& fa, const FragB& fb, auto b_index, auto m_index) {
    constexpr int b = decltype(b_index)::value, m = decltype(m_index)::value;
    constexpr int gu = m % 2, j = (m / 2) % TN, a = (m / (2 * TN)) % 2, i = m / (4 * TN);
    // kSwap: the weight fragment takes the first operand's place, which transposes the accumulator tile
    if constexpr (gu == 0) {
      if constexpr (kSwap) mfma_pinned(acc_g[i][j][a][b], fb.g[j], fa.v[i][a]);
      else mfma_pinned(acc_g[i][j][a][b], fa.v[i][a], fb.g[j]);
    } else {
      if constexpr (kSwap) mfma_pinned(acc_u[i][j][a][b], fb.u[j], fa.v[i][a]);
      else mfma_pinned(acc_u[i][j][a][b], fa.v[i][a], fb.u[j]);
    }
  };

  // Ring schedule.  Token tiles and weight tiles each cycle through their own ring of LDS stages; the barrier of
  // iteration kt says that tile kt + 1 has landed and that nobody reads tile kt's stages any more, so the next
  // fill goes into them.  A K tile is four phases: K step ks = phase / 2 of 32 elements, channel sub-block
  // b = phase % 2; during a phase the wave reads the weight fragments of the next phase and, before a new K step,
  // its token fragments.  The barrier sits before the last phase.  A phase is a sequence of slots, one MFMA each
  // (see the note on instruction order at the top); counted from the barrier, every kEvery-th slot issues the next
  // load of the fill, token rows first.  Tiles past the end are clamped to the last one (redundant loads, never
  // read) so that the loop body and the outstanding-load count never change.
  static_assert(C::kSteps == 4, "two 32-deep K steps of two phases per K tile");
  const int n_k = (st.d_model + KT - 1) / KT;
  const int k_last = (n_k - 1) * KT;
  constexpr int kMayFly = C::kMayFly;  // loads younger than tile kt + 1
  constexpr int kFull = 4 * ACT * TN;  // MFMAs of a phase
  constexpr int SA = C::kStages, SB = C::kBStages;
  constexpr unsigned kARing = SA * C::kATileBytes, kBRing = SB * C::kBStageBytes;
  // Full tiles spread the wave-uniform bookkeeping of a K tile over the idle slots of its third phase; a short tile
  // is bound by its loads, not by the matrix pipe, and does that work at the barrier.
  constexpr bool kSpread = ACT == C::TM && !TAIL && !DEAD && kFull >= 32;
  constexpr int kEvery = ACT == 0 ? 1
                         : (kSpread ? C::kLoadEvery
                                    : ((3 * kFull) / C::kLoadsPerTile < 1 ? 1
                                       : ((3 * kFull) / C::kLoadsPerTile > C::kLoadEvery ? C::kLoadEvery : (3 * kFull) / C::kLoadsPerTile)));
  static_assert(!kSpread || kEvery * C::kLoadsPerTile <= 3 * kFull, "the loads of a fill end before the bookkeeping of the next one");
  // loads of a fill that the phase behind the barrier issues (the prologue does it for the first fill)
  constexpr int kBehindBarrier = ACT == 0 ? C::kLoadsPerTile
                                          : (kFull / kEvery < C::kLoadsPerTile ? kFull / kEvery : C::kLoadsPerTile);
  FragA fa[2];
  FragB fb[2];
  // Routing weight of the lane's output rows.  They stay in registers when the per-tile arrays lie over the ring:
  // the first tile load may overwrite them, so every wave must have taken its copy (and finished with the token
  // ids) before any load is issued.
  float a_rows[NA][2][4];
  if constexpr (C::kAliasAux) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          a_rows[i][a][r] = st.s_a[(WM * i + st.wave_m) * 32 + a * 16 + (kSwap ? st.frag_row : st.frag_half * 4 + r)];
    __syncthreads();
  }
  auto a_of = [&](int i, int a, int r, int row) { return C::kAliasAux ? a_rows[i][a][r] : st.s_a[row]; };

  // Prologue: whole tiles 0 .. SB - 2 (token rows: 0 .. SA - 2), then what the phase behind a barrier would issue
  // of the first fill (token tile SA - 1, weight tile SB - 1).
  Fill fill = make_fill((SA - 1) * C::kATileBytes, min((SA - 1) * KT, k_last), (SB - 1) * C::kBStageBytes,
                        min((SB - 1) * KT, k_last));
  if constexpr (DEAD) static_for<0, C::kADma>([&](auto d) { dma_one(fill, d); });
#pragma unroll
  for (int t = 0; t + 1 < SB; ++t) {
    const Fill whole = make_fill(t * C::kATileBytes, min(t * KT, k_last), t * C::kBStageBytes, min(t * KT, k_last));
    static_for<0, C::kLoadsPerTile>([&](auto d) {
      if (decltype(d)::value >= C::kADma || t + 1 < SA) dma_one(whole, d);  // the token ring ends one tile earlier
    });
  }
  static_for<0, kBehindBarrier>([&](auto d) { dma_unless_dead(fill, d); });
  constexpr int kFirst = DEAD ? kBehindBarrier - (kBehindBarrier < C::kADma ? kBehindBarrier : C::kADma) : kBehindBarrier;
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kMayFly + kFirst) : "memory");
  __syncthreads();
  if constexpr (ACT > 0) {
    static_for<0, 2 * TN + 2 * ACT>([&](auto r) {
      read_one(fa[0], fb[0], frag_a_at(0, 0), frag_b_at(0, 0), integral_constant<int, 0>{}, r);
    });
  }

  unsigned a_st = 0, b_st = 0;  // ring offsets of the stages that hold tile kt
  auto next_a = [&](unsigned x) { return x + C::kATileBytes == kARing ? 0u : x + C::kATileBytes; };
  auto next_b = [&](unsigned x) { return x + C::kBStageBytes == kBRing ? 0u : x + C::kBStageBytes; };
  if constexpr (ACT == 0) {
    // nothing to multiply: this wave only brings in its share of every fill, in one go behind the barrier
    for (int kt = 0; kt < n_k; ++kt) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kMayFly) : "memory");
      __syncthreads();
      fill = make_fill(a_st, min((kt + SA) * KT, k_last), b_st, min((kt + SB) * KT, k_last));
      static_for<0, C::kLoadsPerTile>([&](auto d) { dma_unless_dead(fill, d); });
      a_st = next_a(a_st);
      b_st = next_b(b_st);
    }
  } else if constexpr (!kSpread) {
    for (int kt = 0; kt < n_k; ++kt) {
      const unsigned a_nx = next_a(a_st), b_nx = next_b(b_st);
      static_for<0, C::kSteps>([&](auto phase) {
        constexpr int s = decltype(phase)::value;
        constexpr bool last = s + 1 == C::kSteps;
        constexpr int ks1 = last ? 0 : (s + 1) / 2, b1 = last ? 0 : (s + 1) % 2;  // what this phase reads for the next
        constexpr int n_reads = 2 * TN + (b1 == 0 ? 2 * ACT : 0);
        constexpr int stride = 2 * n_reads <= kFull ? 2 : 1;
        static_assert(n_reads * stride <= kFull + stride - 1, "a read slot for every fragment");
        if constexpr (last) {
          asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kMayFly) : "memory");
          __syncthreads();
          fill = make_fill(a_st, min((kt + SA) * KT, k_last), b_st, min((kt + SB) * KT, k_last));
        }
        const unsigned at_a = frag_a_at(last ? a_nx : a_st, ks1), at_b = frag_b_at(last ? b_nx : b_st, ks1);
        FragA& ra = fa[ks1 & 1];
        FragB& rb = fb[last ? 0 : (s + 1) & 1];
        static_for<0, kFull>([&](auto mi) {
          constexpr int m = decltype(mi)::value;
          mfma_one(fa[(s / 2) & 1], fb[s & 1], integral_constant<int, s % 2>{}, mi);
          if constexpr (m % stride == 0 && m / stride < n_reads)
            read_one(ra, rb, at_a, at_b, integral_constant<int, b1>{}, integral_constant<int, m / stride>{});
          constexpr int G = (last ? 0 : kFull * (s + 1)) + m;  // slot counted from the barrier
          if constexpr (G % kEvery == kEvery - 1 && G / kEvery < C::kLoadsPerTile)
            dma_unless_dead(fill, integral_constant<int, G / kEvery>{});
          __builtin_amdgcn_sched_barrier(0);
        });
      });
      a_st = a_nx;
      b_st = b_nx;
    }
  } else {
    // Full tile.  State that the slots of phase 2 bring up to date, one step each, pinned where it is computed:
    // the fill behind the coming barrier, the ring offsets of tile kt + 1, and the fragment offsets of the reads
    // of the last phase (from tile kt + 1) and of the next iteration's first three.
    auto pin_s = [](auto& x) { asm volatile("" : "+s"(x)); };
    auto pin_v = [](auto& x) { asm volatile("" : "+v"(x)); };
    int ka = 2 * fill.a_k, kb = 2 * fill.b_k;  // byte offsets along K of the latest fill
    const unsigned lds_a = __builtin_amdgcn_readfirstlane(lds0 + st.a_lds);
    const unsigned lds_b = __builtin_amdgcn_readfirstlane(lds0 + kARing + st.b_lds);
    unsigned a_nx = 0, b_nx = 0;
    unsigned at_a1 = frag_a_at(0, 1), at_b0 = frag_b_at(0, 0), at_b1 = frag_b_at(0, 1);  // this iteration's reads
    unsigned at_a0n = 0, at_b0n = 0, nx_a1 = 0, nx_b0 = 0, nx_b1 = 0;
    for (int kt = 0; kt < n_k; ++kt) {
      static_for<0, C::kSteps>([&](auto phase) {
        constexpr int s = decltype(phase)::value;
        constexpr bool last = s + 1 == C::kSteps;
        constexpr int ks1 = last ? 0 : (s + 1) / 2, b1 = last ? 0 : (s + 1) % 2;
        constexpr int n_reads = 2 * TN + (b1 == 0 ? 2 * ACT : 0);
        static_assert(2 * n_reads <= kFull, "a read behind every other MFMA");
        if constexpr (last) {
          asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kMayFly) : "memory");
          __syncthreads();
        }
        const unsigned at_a = last ? at_a0n : at_a1;
        const unsigned at_b = last ? at_b0n : (s == 0 ? at_b0 : at_b1);
        FragA& ra = fa[ks1 & 1];
        FragB& rb = fb[last ? 0 : (s + 1) & 1];
        static_for<0, kFull>([&](auto mi) {
          constexpr int m = decltype(mi)::value;
          mfma_one(fa[(s / 2) & 1], fb[s & 1], integral_constant<int, s % 2>{}, mi);
          if constexpr (m % 2 == 0 && m / 2 < n_reads)
            read_one(ra, rb, at_a, at_b, integral_constant<int, b1>{}, integral_constant<int, m / 2>{});
          constexpr int G = (last ? 0 : kFull * (s + 1)) + m;
          if constexpr (G % kEvery == kEvery - 1 && G / kEvery < C::kLoadsPerTile) dma_one(fill, integral_constant<int, G / kEvery>{});
          if constexpr (s == 2 && m % 2 == 1) {  // no load is issued from here to the barrier
            constexpr int step = m / 2;
            if constexpr (step == 0) { ka = min(ka + 2 * KT, 2 * k_last); pin_s(ka); }
            if constexpr (step == 1) { kb = min(kb + 2 * KT, 2 * k_last); pin_s(kb); }
            if constexpr (step == 2) { fill.a_ptr = st.a_base + (unsigned)ka; pin_s(fill.a_ptr); }
            if constexpr (step == 3) { fill.g_ptr = st.g_base + (unsigned)kb; pin_s(fill.g_ptr); }
            if constexpr (step == 4) { fill.u_ptr = st.u_base + (unsigned)kb; pin_s(fill.u_ptr); }
            if constexpr (step == 5) { fill.a_lds = lds_a + a_st; pin_s(fill.a_lds); }
            if constexpr (step == 6) { fill.b_lds = lds_b + b_st; pin_s(fill.b_lds); }
            if constexpr (step == 7) { a_nx = next_a(a_st); pin_s(a_nx); }
            if constexpr (step == 8) { b_nx = next_b(b_st); pin_s(b_nx); }
            if constexpr (step == 9) { at_a0n = frag_a_at(a_nx, 0); pin_v(at_a0n); }
            if constexpr (step == 10) { at_b0n = frag_b_at(b_nx, 0); pin_v(at_b0n); }
            if constexpr (step == 11) { nx_b0 = at_b0n; nx_a1 = frag_a_at(a_nx, 1); pin_v(nx_a1); }
            if constexpr (step == 12) { nx_b1 = frag_b_at(b_nx, 1); pin_v(nx_b1); }
          }
          __builtin_amdgcn_sched_barrier(0);
        });
      });
      a_st = a_nx;
      b_st = b_nx;
      at_a1 = nx_a1;
      at_b0 = nx_b0;
      at_b1 = nx_b1;
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may still be writing LDS at exit
  mfma_drain();                                      // the last MFMAs have written their accumulators
  if constexpr (C::kAliasAux && EPI == kEpiStats) __syncthreads();  // the column reduction lies over the ring: every wave has read its last fragments

  // Epilogue.  Accumulator register r of lane l in sub-block (a, b) of block (i, j) is output row
  // 32*block + 16a + 4*(l/16) + r, column 32*block + 16b + l % 16: a lane owns two channels per channel block.
  // Transposed (kSwap): row 32*block + 16a + l % 16, columns 32*block + 16b + 4*(l/16) + r.
  const int lane_col = st.frag_row, lane_rows = st.frag_half * 4;  // l % 16, 4 * (l / 16)
  if constexpr (EPI != kEpiStats) {
    const int pad_end = (EPI == kEpiHidden && ep.pad_hidden) ? (d_ff + ep.pad_hidden - 1) / ep.pad_hidden * ep.pad_hidden : d_ff;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int col0 = n0 + st.wave_n * TN * 32 + j * 32 + b * 16 + lane_rows;  // this lane's four channels
        if (col0 >= pad_end) continue;
        const bool whole = col0 + 3 < d_ff;  // all four inside: one vector store
        float kept[4] = {1.0f, 1.0f, 1.0f, 1.0f};
        if constexpr (EPI == kEpiHidden) {
          if (ep.keep != nullptr) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              kept[r] = (col0 + r < d_ff && ep.keep[(int64_t)st.expert * d_ff + col0 + r]) ? 1.0f : 0.0f;
          }
        }
#pragma unroll
        for (int i = 0; i < ACT; ++i)
#pragma unroll
          for (int a = 0; a < 2; ++a) {
            const int row = (WM * i + st.wave_m) * 32 + a * 16 + lane_col;
            if (row >= st.m_len) continue;
            const int64_t out_row = st.row_first + row;
            if constexpr (EPI == kEpiHidden) {
              __hip_bfloat16* dst = static_cast<__hip_bfloat16*>(ep.hidden) + out_row * ep.ld_hidden + col0;
              const float a_tok = a_of(i, a, 0, row);
              __hip_bfloat16 lam[4];
#pragma unroll
              for (int r = 0; r < 4; ++r)
                lam[r] = __float2bfloat16(a_tok * silu_f32(acc_g[i][j][a][b][r]) * acc_u[i][j][a][b][r] * kept[r]);
              if (whole) {  // rows of the hidden buffer are multiples of 8 elements long: 8-byte aligned
                uint2 v;
                v.x = (uint32_t)__builtin_bit_cast(uint16_t, lam[0]) | ((uint32_t)__builtin_bit_cast(uint16_t, lam[1]) << 16);
                v.y = (uint32_t)__builtin_bit_cast(uint16_t, lam[2]) | ((uint32_t)__builtin_bit_cast(uint16_t, lam[3]) << 16);
                *reinterpret_cast<uint2*>(dst) = v;
              } else {  // the last channels of the expert, then the K padding of the contraction that reads these rows
#pragma unroll
                for (int r = 0; r < 4; ++r)
                  if (col0 + r < pad_end) dst[r] = col0 + r < d_ff ? lam[r] : __float2bfloat16(0.0f);
              }
            } else {
              float* dst = ep.product + out_row * ep.ld_product + col0;
              if (whole) {  // output rows and both column halves are multiples of 4 floats: 16-byte aligned
                *reinterpret_cast<f32x4*>(dst) = acc_g[i][j][a][b];
                *reinterpret_cast<f32x4*>(dst + ep.col_gap) = acc_u[i][j][a][b];
              } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                  if (col0 + r < d_ff) {
                    dst[r] = acc_g[i][j][a][b][r];
                    dst[r + ep.col_gap] = acc_u[i][j][a][b][r];
                  }
              }
            }
          }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float sum = 0.0f, mx = 0.0f;
#pragma unroll
        for (int i = 0; i < ACT; ++i)
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int row = (WM * i + st.wave_m) * 32 + a * 16 + lane_rows + r;
              const float lam = a_of(i, a, r, row) * silu_f32(acc_g[i][j][a][b][r]) * acc_u[i][j][a][b][r];
              sum = fmaf(lam, lam, sum);
              mx = fmaxf(mx, fabsf(lam));  // squared once below: rounding keeps order, so max(x^2) = (max |x|)^2 bit for bit
            }
        mx *= mx;
        sum += __shfl_xor(sum, 16);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        sum += __shfl_xor(sum, 32);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (st.frag_half == 0) {
          const int col = st.wave_n * TN * 32 + j * 32 + b * 16 + lane_col;
          st.s_red[st.wave_m * BN + col] = sum;
          st.s_red[(WM + st.wave_m) * BN + col] = mx;
        }
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
        ep.part_phi2[(int64_t)slot * d_ff + n0 + col] = sum;
        ep.part_max[(int64_t)slot * d_ff + n0 + col] = mx;
      }
    }
  }  // statistics epilogue
}

// What a workgroup has to do: tile (slot, n0 / BN) of expert e.
struct TileWork {
  int e, slot, row_first, m_len, n0;
  int tok_first;  // first token of the tile when every expert sees every token (no permutation)
};

// One tile with the tiling of configuration C.  AUX: byte offset in LDS of the per-tile arrays (token ids,
// routing weights, the column reduction), behind the stages of the largest configuration in use.
template <class C, bool TAIL, int EPI, int AUX>
__device__ __forceinline__ void run_tile(const TileWork& w, const __hip_bfloat16* __restrict__ X, int64_t ldx,
                                         int d_model, int d_ff, const __hip_bfloat16* __restrict__ Wg,
                                         const __hip_bfloat16* __restrict__ Wu, int64_t stride_gu, int64_t ldw,
                                         const int32_t* __restrict__ perm, const float* __restrict__ w_perm,
                                         const __hip_bfloat16* __restrict__ zeros, const EpiArgs& ep) {
  // d_model: the K extent; ldw: elements between consecutive rows of Wg / Wu (d_model unless the rows are padded)
  constexpr int BM = C::BM, BN = C::BN, TM = C::TM, TN = C::TN, WM = C::WM;
  static_assert(C::kAliasAux ? AUX == 0 : C::kRingBytes <= AUX, "the per-tile arrays lie behind the ring, or over its start");
  const int e = w.e, slot = w.slot, row_first = w.row_first, m_len = w.m_len, n0 = w.n0;
  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_tok = reinterpret_cast<int32_t*>(smem + AUX);  // [BM] token id
  float* s_a = reinterpret_cast<float*>(s_tok + BM);                                // [BM] routing weight
  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // in a scalar register: wave-uniform addresses and branches

  // Rows past the end of the expert's bucket read token row 0 of the tile again with weight 0:
  // their Lambda is exactly 0 (finite projections times a = 0), so no load in the K loop is conditional.
  for (int r = tid; r < BM; r += C::kThreads) {
    const int rr = r < m_len ? r : 0;
    if constexpr (EPI == kEpiProduct) s_tok[r] = row_first + rr;  // A rows are the bucket slots themselves
    else s_tok[r] = perm ? perm[row_first + rr] : w.tok_first + rr;
    s_a[r] = r < m_len ? (w_perm ? w_perm[row_first + rr] : 1.0f) : 0.0f;
  }
  __syncthreads();

  TileState<C> st;
  st.smem = smem;
  st.s_a = s_a;
  st.s_red = s_a + BM;  // [2 stats][WM][BN]
  st.d_model = d_model;
  st.zeros = zeros;
  st.wave_m = wave % WM;
  st.wave_n = wave / WM;
  st.frag_row = lane % 16;   // 16x16x32: row of a 16-row sub-block
  st.frag_half = lane / 16;  // and the lane's quarter of the 32-wide K step
  st.expert = e;
  st.m_len = m_len;
  st.row_first = row_first;
  // direct-to-LDS sources of this lane
  const int a_row0 = wave * (BM / C::kWaves), b_row0 = wave * (BN / C::kWaves);
  st.a_lds = a_row0 * C::kRowBytes;
  st.b_lds = b_row0 * C::kRowBytes;
#pragma unroll
  for (int j = 0; j < C::kADma; ++j) {
    const int row = a_row0 + j * C::kDmaRows + lane / C::kChunks;
    const int ck = (lane % C::kChunks) ^ swizzle_key<C>(row);
    st.a_k[j] = ck * 8;
    const int64_t elem = (int64_t)s_tok[row] * ldx + ck * 8;
    st.a_src[j] = X + elem - (j % 4) * 512;  // the immediate offset 1024 (j % 4) bytes comes back
    st.a_off[j] = (unsigned)(2 * elem + TileState<C>::kBias - (j % 4) * 1024);
  }
  st.a_base = reinterpret_cast<const unsigned char*>(X) - TileState<C>::kBias;
  st.g_base = reinterpret_cast<const unsigned char*>(Wg + (int64_t)e * stride_gu) - TileState<C>::kBias;
  st.u_base = reinterpret_cast<const unsigned char*>(Wu + (int64_t)e * stride_gu) - TileState<C>::kBias;
#pragma unroll
  for (int j = 0; j < C::kBDma; ++j) {
    const int row = b_row0 + j * C::kDmaRows + lane / C::kChunks;
    const int ck = (lane % C::kChunks) ^ swizzle_key<C>(row);
    const int c = min(n0 + row, d_ff - 1);  // channels past d_ff read the last channel again; never written
    const int64_t off = (int64_t)e * stride_gu + (int64_t)c * ldw + ck * 8;
    st.b_k[j] = ck * 8;
    st.g_src[j] = Wg + off - (j % 4) * 512;
    st.u_src[j] = Wu + off - (j % 4) * 512;
    st.b_off[j] = (unsigned)(2 * ((int64_t)c * ldw + ck * 8) + TileState<C>::kBias - (j % 4) * 1024);
  }
  // Fragments: lane l holds row (l % 16) of a 16-row sub-block, K elements 8*(l / 16) .. +7 of a 32-wide K step.
  st.a_frag_base = (st.wave_m * 32 + st.frag_row) * C::kRowBytes;       // + i*WM*32 rows: block WM*i + wave_m
  st.b_frag_base = (st.wave_n * TN * 32 + st.frag_row) * C::kRowBytes;  // + j*32 rows
  // the key of row (16 a + l % 16) of a block does not depend on a, so one key per lane here too
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) st.k_swz[ks] = ((ks * 4 + st.frag_half) ^ swizzle_key<C>(st.frag_row)) << 4;

  // accumulator i of this wave covers row block WM*i + wave_m; blocks past m_len are skipped
  const int n_row_blocks = (m_len + 31) / 32;
  const int act = max(0, (n_row_blocks - st.wave_m + WM - 1) / WM);  // wave-uniform, 0 .. TM
  // With two stages the K loop waits for every outstanding load, so a wave may issue fewer of them.
  const bool dead = C::kStages == 2 && a_row0 >= m_len;  // (the ring of the token rows)
  static_assert(TM == 4 || TM == 2 || TM == 1, "dispatch below covers TM = 1, 2 and 4");
#define CAMERA_TILE_FN tile_body16
#define CAMERA_TILE_BODY(A)                                                              \
  do {                                                                                   \
    if (dead) CAMERA_TILE_FN<C, (A), TAIL, true, EPI>(st, n0, d_ff, slot, ep);           \
    else CAMERA_TILE_FN<C, (A), TAIL, false, EPI>(st, n0, d_ff, slot, ep);               \
  } while (0)
  if (act >= TM) CAMERA_TILE_FN<C, TM, TAIL, false, EPI>(st, n0, d_ff, slot, ep);
  else if (act == 3) CAMERA_TILE_BODY((TM > 3 ? 3 : 0));
  else if (act == 2) CAMERA_TILE_BODY((TM > 2 ? 2 : 0));
  else if (act == 1) CAMERA_TILE_BODY((TM > 1 ? 1 : 0));
  else CAMERA_TILE_BODY(0);
#undef CAMERA_TILE_BODY
#undef CAMERA_TILE_FN
}

template <class C, bool TAIL, int EPI>
__global__ __launch_bounds__(C::kThreads, C::kWavesPerSimd) void grouped_gemm_bf16_kernel(
    const __hip_bfloat16* __restrict__ X, int64_t ldx, int d_model, int d_ff,
    const __hip_bfloat16* __restrict__ Wg, const __hip_bfloat16* __restrict__ Wu, int64_t stride_gu,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tile_offset,
    const int32_t* __restrict__ tile_expert, const int32_t* __restrict__ perm, const float* __restrict__ w_perm,
    int n_experts, const __hip_bfloat16* __restrict__ zeros, EpiArgs ep) {
  constexpr int BM = C::BM, BN = C::BN;
  // Workgroup -> tile mapping.  The hardware deals consecutive workgroup ids round-robin to the 8
  // XCDs, each with its own L2 and 32 CUs, and an XCD starts its workgroups in id order.  Every
  // XCD gets an equal, contiguous run of logical ids (sized from the real tile count, which only
  // the device knows), and logical ids are ordered so that the ~32 workgroups an XCD runs at a
  // time form a patch that shares tiles through its L2, and so that the next patch needs the same
  // weight tiles again: expert, then groups of kGroupN-ish N-tiles, then chunks of up to kChunkM
  // M-tiles of that expert (innermost in time: the weight tiles of the group come back from the
  // memory-side cache instead of HBM, and an expert's weights leave HBM once), then the tiles of
  // the chunk.
  const int n_tiles_n = (d_ff + BN - 1) / BN;
  const int total = tile_offset[n_experts] * n_tiles_n;
  const int per_xcd = (total + kXcds - 1) / kXcds;
  const int seq = blockIdx.x / kXcds;
  const int logical = (blockIdx.x % kXcds) * per_xcd + seq;
  if (seq >= per_xcd || logical >= total) return;  // block-uniform: nothing here
  const int e = tile_expert[logical / n_tiles_n];  // expert e owns logical ids tile_offset[e] * n_tiles_n ..
  const int m_e = tile_offset[e + 1] - tile_offset[e];
  const int local = logical - tile_offset[e] * n_tiles_n;
  const int chunk_m = m_e <= kChunkMax ? m_e : kChunkM;       // M-tiles that run side by side
  const int group_n = max(1, kPatch / chunk_m);               // N-tiles that run side by side
  const int group = local / (m_e * group_n);                  // all groups but the last are full
  const int group_w = min(group_n, n_tiles_n - group * group_n);
  const int in_group = local - group * m_e * group_n;
  const int chunk = in_group / (chunk_m * group_w);           // all chunks but the last are full
  const int chunk_h = min(chunk_m, m_e - chunk * chunk_m);
  const int in_chunk = in_group - chunk * chunk_m * group_w;
  const int tile_n = group * group_n + in_chunk / chunk_h;
  const int slot = tile_offset[e] + chunk * chunk_m + in_chunk % chunk_h;
  const int tile_in_expert = slot - tile_offset[e];
  const int row_first = offsets[e] + tile_in_expert * BM;  // first bucket slot of this tile
  const int m_len = min(BM, offsets[e + 1] - row_first);   // >= 1
  const int n0 = tile_n * BN;

  TileWork w;
  w.e = e;
  w.slot = slot;
  w.row_first = row_first;
  w.m_len = m_len;
  w.n0 = n0;
  w.tok_first = tile_in_expert * BM;
  constexpr int kAux = C::kAliasAux ? 0 : C::kRingBytes;  // the per-tile arrays
  run_tile<C, TAIL, EPI, kAux>(w, X, ldx, d_model, d_ff, Wg, Wu, stride_gu, d_model, perm, w_perm, zeros, ep);
}

// ---------------------------------------------------------------------------
// The same tiles on a compacted layer, where every expert has its own width.
//   CompactRows  (first contraction): expert e has n_ext = its kept micro-experts as N extent, K = d_model;
//                its gate / up rows start at row row_off[e] of the packed matrices.
//   CompactDown  (second contraction): N = d_model / 2 for every expert (the two halves of the block's rows
//                stand in for gate and up), K = its kept count rounded up to 8 (the hidden rows and the block's
//                rows are zero there), rows ld(e) elements apart.
// The logical tile ids of expert e start at work_off[e] = sum over the experts before it of (M tiles x N tiles),
// written by compact_work_kernel once the bucket tables exist.
// ---------------------------------------------------------------------------
struct ExpertGeom {
  int n_ext, k_ext;
  int64_t ldw, g_off, u_off;  // row stride and first element of the expert's two B matrices
};
__device__ __forceinline__ ExpertGeom expert_geom(const CompactRows& t, int e, int d_model) {
  const int64_t off = (int64_t)t.row_off[e] * d_model;
  return {t.row_off[e + 1] - t.row_off[e], d_model, d_model, off, off};
}
__device__ __forceinline__ ExpertGeom expert_geom(const CompactDown& t, int e, int d_model) {
  const int64_t ld = t.ld_off[e + 1] - t.ld_off[e];
  const int64_t base = (int64_t)t.ld_off[e] * d_model;
  const int k_ext = (t.count[e] + t.k_round - 1) / t.k_round * t.k_round;  // <= ld: the row alignment is a multiple of k_round
  return {d_model / 2, k_ext, ld, base, base + (int64_t)(d_model / 2) * ld};
}

// Scratch of a compacted-layer launch, written by compact_work_kernel:
//   work_off  [n_experts + 1]  first logical tile id of every expert
//   xcd_first [kXcds + 1]      XCD x runs the logical ids xcd_first[x] .. xcd_first[x + 1].  The cuts are placed by
//                              cost (tiles times K tiles of their expert), not by tile count: in the second
//                              contraction a shared expert's tiles can be many times longer than a routed expert's.
//   hid_off   [n_experts]      (int64) first element of expert e's rows in the hidden buffer, which holds the rows of
//                              expert e back to back, hidden_ld(e) elements each: rows as long as the widest expert's
//                              would spread a routed expert's 3 KB rows over 24 KB strides
struct CompactScratch {
  int32_t* work_off;
  int32_t* xcd_first;
  int64_t* hid_off;
};
__host__ __device__ inline CompactScratch compact_scratch(int32_t* base, int n_experts) {
  CompactScratch s;
  s.work_off = base;
  s.xcd_first = base + n_experts + 1;
  // 8-byte aligned: the int32 part is padded to an even count
  s.hid_off = reinterpret_cast<int64_t*>(base + ((n_experts + 1 + kXcds + 1 + 1) & ~1));
  return s;
}
// Length of expert e's hidden rows: its kept count rounded up to k_round (the K extent of the second contraction).
__device__ __forceinline__ int hidden_ld(const CompactRows& t, int e, int k_round) {
  return (t.row_off[e + 1] - t.row_off[e] + k_round - 1) / k_round * k_round;
}
__device__ __forceinline__ int hidden_ld(const CompactDown& t, int e, int k_round) {
  return (t.count[e] + k_round - 1) / k_round * k_round;
}

// One workgroup, thread e owns expert e: its tile count, cost and hidden rows, then exclusive prefixes over the
// experts (a Hillis-Steele scan in LDS: 256 entries) and, by threads 1 .. kXcds - 1, the cuts.
template <class TABLE>
__global__ __launch_bounds__(CAMERA_MAX_EXPERTS) void compact_work_kernel(TABLE tab, int d_model, int bn, int kt,
                                                                          int k_round,
                                                                          const int32_t* __restrict__ offsets,
                                                                          const int32_t* __restrict__ tile_offset,
                                                                          int32_t* __restrict__ scratch) {
  __shared__ int32_t s_tiles[2][CAMERA_MAX_EXPERTS];   // inclusive prefixes, double-buffered
  __shared__ int64_t s_cost[2][CAMERA_MAX_EXPERTS];
  __shared__ int64_t s_hid[2][CAMERA_MAX_EXPERTS];
  const CompactScratch sc = compact_scratch(scratch, tab.n_experts);
  const int e = threadIdx.x, n = tab.n_experts;
  int32_t tiles = 0;
  int64_t cost = 0, hid = 0;
  if (e < n) {
    const ExpertGeom g = expert_geom(tab, e, d_model);
    tiles = (tile_offset[e + 1] - tile_offset[e]) * ((g.n_ext + bn - 1) / bn);
    cost = (int64_t)tiles * max(1, (g.k_ext + kt - 1) / kt);
    hid = (int64_t)(offsets[e + 1] - offsets[e]) * hidden_ld(tab, e, k_round);
  }
  s_tiles[0][e] = tiles;
  s_cost[0][e] = cost;
  s_hid[0][e] = hid;
  __syncthreads();
  int cur = 0;
  for (int d = 1; d < CAMERA_MAX_EXPERTS; d <<= 1) {
    const int nxt = cur ^ 1;
    s_tiles[nxt][e] = s_tiles[cur][e] + (e >= d ? s_tiles[cur][e - d] : 0);
    s_cost[nxt][e] = s_cost[cur][e] + (e >= d ? s_cost[cur][e - d] : (int64_t)0);
    s_hid[nxt][e] = s_hid[cur][e] + (e >= d ? s_hid[cur][e - d] : (int64_t)0);
    __syncthreads();
    cur = nxt;
  }
  const int32_t run = s_tiles[cur][CAMERA_MAX_EXPERTS - 1];       // all tiles
  const int64_t total = s_cost[cur][CAMERA_MAX_EXPERTS - 1];      // all cost
  if (e < n) {
    sc.work_off[e] = s_tiles[cur][e] - tiles;
    sc.hid_off[e] = s_hid[cur][e] - hid;
  }
  if (e == 0) {
    sc.work_off[n] = run;
    sc.xcd_first[0] = 0;
    sc.xcd_first[kXcds] = run;
  }
  if (e >= 1 && e < kXcds) {
    // cut x: the first expert whose inclusive cost prefix exceeds total x / kXcds, and inside it the tile that does
    const int64_t target = total * e / kXcds;
    int lo = 0, hi = n;  // first expert with inclusive prefix > target
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (s_cost[cur][mid] > target) hi = mid; else lo = mid + 1;
    }
    if (lo >= n) {
      sc.xcd_first[e] = run;
    } else {
      const int32_t first = lo == 0 ? 0 : s_tiles[cur][lo - 1];
      const int32_t mine_tiles = s_tiles[cur][lo] - first;
      const int64_t before = lo == 0 ? 0 : s_cost[cur][lo - 1];
      const int64_t per_tile = (s_cost[cur][lo] - before) / max(1, mine_tiles);
      sc.xcd_first[e] = first + (int)((target - before) / max<int64_t>(1, per_tile));
    }
  }
}

template <class C, bool TAIL, int EPI, class TABLE>
__global__ __launch_bounds__(C::kThreads, C::kWavesPerSimd) void grouped_gemm_bf16_compact_kernel(
    const __hip_bfloat16* __restrict__ X, int64_t ldx, int d_model, const __hip_bfloat16* __restrict__ Wg,
    const __hip_bfloat16* __restrict__ Wu, TABLE tab, int k_round, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ tile_offset, int32_t* __restrict__ scratch,
    const int32_t* __restrict__ perm, const float* __restrict__ w_perm, const __hip_bfloat16* __restrict__ zeros,
    EpiArgs ep_launch) {
  // X: the tokens (first contraction) or the hidden buffer (second contraction, ldx unused: its rows are ragged)
  constexpr int BM = C::BM, BN = C::BN;
  const int n_experts = tab.n_experts;
  const CompactScratch sc = compact_scratch(scratch, n_experts);
  const int32_t* work_off = sc.work_off;
  const int32_t* xcd_first = sc.xcd_first;
  const int xcd = blockIdx.x % kXcds;
  const int stride = gridDim.x / kXcds;  // workgroups per XCD: a workgroup takes every stride-th tile of its XCD's range
  const int last = xcd_first[xcd + 1];
  for (int logical = xcd_first[xcd] + (int)(blockIdx.x / kXcds); logical < last; logical += stride) {
  __syncthreads();  // the previous tile's per-tile arrays in LDS are no longer read
  int lo = 0, hi = n_experts;                      // work_off[lo] <= logical < work_off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (work_off[mid] <= logical) lo = mid; else hi = mid;
  }
  const int e = lo;
  const ExpertGeom g = expert_geom(tab, e, d_model);
  // the expert's rows of the hidden buffer: row of bucket slot s at hid_e + s * hid_ld
  const int64_t hid_ld = hidden_ld(tab, e, k_round);
  const int64_t hid_e = sc.hid_off[e] - (int64_t)offsets[e] * hid_ld;
  EpiArgs ep = ep_launch;
  const __hip_bfloat16* A = X;
  int64_t lda = ldx;
  if constexpr (EPI == kEpiHidden) {
    ep.hidden = static_cast<__hip_bfloat16*>(ep_launch.hidden) + hid_e;
    ep.ld_hidden = hid_ld;
  } else {
    A = X + hid_e;
    lda = hid_ld;
  }
  const int n_tiles_n = (g.n_ext + BN - 1) / BN;  // >= 1: an expert without N tiles owns no logical id
  const int m_e = tile_offset[e + 1] - tile_offset[e];
  const int local = logical - work_off[e];
  // the tile order of grouped_gemm_bf16_kernel inside the expert
  const int chunk_m = m_e <= kChunkMax ? m_e : kChunkM;
  const int group_n = max(1, kPatch / chunk_m);
  const int group = local / (m_e * group_n);
  const int group_w = min(group_n, n_tiles_n - group * group_n);
  const int in_group = local - group * m_e * group_n;
  const int chunk = in_group / (chunk_m * group_w);
  const int chunk_h = min(chunk_m, m_e - chunk * chunk_m);
  const int in_chunk = in_group - chunk * chunk_m * group_w;
  const int tile_n = group * group_n + in_chunk / chunk_h;
  const int slot = tile_offset[e] + chunk * chunk_m + in_chunk % chunk_h;
  const int tile_in_expert = slot - tile_offset[e];
  const int row_first = offsets[e] + tile_in_expert * BM;
  const int m_len = min(BM, offsets[e + 1] - row_first);  // >= 1
  const int n0 = tile_n * BN;

  if constexpr (EPI == kEpiProduct) {
    if (g.k_ext == 0) {  // the expert keeps nothing: its product rows are zero
      const int width = min(BN, g.n_ext - n0);
      for (int i = threadIdx.x; i < m_len * width; i += C::kThreads) {
        float* row = ep.product + (int64_t)(row_first + i / width) * ep.ld_product + n0 + i % width;
        row[0] = 0.0f;
        row[ep.col_gap] = 0.0f;
      }
      continue;
    }
  }
  TileWork w;
  w.e = 0;  // the expert's matrices are addressed through g_off / u_off, not through an expert stride
  w.slot = slot;
  w.row_first = row_first;
  w.m_len = m_len;
  w.n0 = n0;
  w.tok_first = tile_in_expert * BM;
  constexpr int kAux = C::kAliasAux ? 0 : C::kRingBytes;  // the per-tile arrays
  run_tile<C, TAIL, EPI, kAux>(w, A, lda, g.k_ext, g.n_ext, Wg + g.g_off, Wu + g.u_off, 0, g.ldw, perm, w_perm, zeros, ep);
  }
}

// ---------------------------------------------------------------------------
// fp32 FMA kernel: 64 tokens x 64 channels per block of 256 threads, K step 16,
// each thread 4 rows x 4 channels of gate and of up.
// ---------------------------------------------------------------------------
constexpr int F32_BM = 64, F32_BN = 64, F32_KT = 16;

template <int EPI>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(
    const float* __restrict__ X, int64_t ldx, int d_model, int d_ff, const float* __restrict__ Wg,
    const float* __restrict__ Wu, int64_t stride_gu, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ tile_offset, const int32_t* __restrict__ tile_expert,
    const int32_t* __restrict__ perm, const float* __restrict__ w_perm, int n_experts, EpiArgs ep) {
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
      if constexpr (EPI == kEpiProduct) tok = row_first + r;  // the left operand is indexed by bucket slot
      else tok = perm ? perm[row_first + r] : tile_in_expert * F32_BM + r;
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
  if constexpr (EPI != kEpiStats) {  // per token row: hidden activations (float32 here) or the plain products
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= d_ff) continue;
      float kept = 1.0f;
      if constexpr (EPI == kEpiHidden) kept = (ep.keep == nullptr || ep.keep[(int64_t)e * d_ff + col]) ? 1.0f : 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = ty * 4 + i;
        if (row >= m_len) continue;
        const int64_t out_row = row_first + row;
        if constexpr (EPI == kEpiHidden) {
          static_cast<float*>(ep.hidden)[out_row * ep.ld_hidden + col] = s_a[row] * silu_f32(acc_g[i][j]) * acc_u[i][j] * kept;
        } else {
          ep.product[out_row * ep.ld_product + col] = acc_g[i][j];
          ep.product[out_row * ep.ld_product + col + ep.col_gap] = acc_u[i][j];
        }
      }
    }
  } else {
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
    ep.part_phi2[(int64_t)slot * d_ff + n0 + tid] = sum;
    ep.part_max[(int64_t)slot * d_ff + n0 + tid] = mx;
  }
  }  // statistics epilogue
}

// Shape of the bf16 kernel: waves (M x N), 32x32 blocks per wave (M x N), K tile, stages of the token ring, stages
// of the weight ring.  Four waves of 128 x 64 x {gate, up}: one per SIMD.
using Bf16Cfg = GemmCfg<2, 2, 4, 2, 64, 2, 3>;

// Whether the scalar-base form of the tile loads can address the operands: 32-bit byte offsets from the start of
// the token matrix (a_rows rows of lda elements) and of one expert's weight matrix (b_rows rows of ldw elements).
// Kept below 2 GiB, where the offset reads the same as a signed and as an unsigned number.
bool fits_32bit_offsets(int64_t a_rows, int64_t lda, int64_t b_rows, int64_t ldw) {
  const int64_t limit = (int64_t(1) << 31) - 2 * TileState<Bf16Cfg>::kBias - 4096;
  return 2 * a_rows * lda < limit && 2 * b_rows * ldw < limit;
}

}  // namespace

int gemm_tile_m(int dtype, int64_t d_ff) {
  (void)d_ff;
  return dtype == CAMERA_BF16 ? Bf16Cfg::BM : F32_BM;
}

template <int EPI>
static hipError_t launch_bf16(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model, int64_t d_ff,
                              int n_experts, const void* W_gate, const void* W_up, int64_t stride_gu, int max_tiles,
                              const BucketTables& t, const EpiArgs& ep) {
  using C = Bf16Cfg;
  // token rows lie below max_tiles * BM (every token, and every bucket slot, belongs to some tile)
  const bool tail = d_model % C::KT != 0 || !fits_32bit_offsets((int64_t)max_tiles * C::BM, ldx, d_ff, d_model);
  auto kern = tail ? grouped_gemm_bf16_kernel<C, true, EPI> : grouped_gemm_bf16_kernel<C, false, EPI>;
  static bool attr_set[2] = {false, false};
  if (!attr_set[tail]) {
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, C::kSmemBytes);
    if (err != hipSuccess) return err;
    attr_set[tail] = true;
  }
  const int64_t n_tiles_n = (d_ff + C::BN - 1) / C::BN;
  const int64_t n_blocks = (max_tiles * n_tiles_n + kXcds - 1) / kXcds * kXcds;
  if (n_blocks >= (int64_t(1) << 31)) return hipErrorInvalidValue;
  dim3 grid((unsigned)n_blocks);
  hipLaunchKernelGGL(kern, grid, dim3(C::kThreads), C::kSmemBytes, stream, static_cast<const __hip_bfloat16*>(X), ldx,
                     (int)d_model, (int)d_ff, static_cast<const __hip_bfloat16*>(W_gate),
                     static_cast<const __hip_bfloat16*>(W_up), stride_gu, t.offsets, t.tile_offset, t.tile_expert,
                     t.perm, t.w_perm, n_experts, static_cast<const __hip_bfloat16*>(t.zeros), ep);
  return hipGetLastError();
}

hipError_t launch_grouped_gemm(hipStream_t stream, int dtype, const void* X, int64_t ldx, int64_t d_model,
                               int64_t d_ff, int n_experts, const void* W_gate, const void* W_up,
                               int64_t stride_gu, int max_tiles, const BucketTables& t, const GemmEpilogue& e) {
  if (max_tiles <= 0) return hipSuccess;
  EpiArgs ep{e.part_phi2, e.part_max, e.hidden, e.keep, e.product, e.ld_product, e.col_gap, d_ff, 0};
  if (dtype == CAMERA_BF16) {
    switch (e.mode) {
      case GemmEpilogue::kStats:
        return launch_bf16<kEpiStats>(stream, X, ldx, d_model, d_ff, n_experts, W_gate, W_up, stride_gu, max_tiles, t, ep);
      case GemmEpilogue::kHidden:
        return launch_bf16<kEpiHidden>(stream, X, ldx, d_model, d_ff, n_experts, W_gate, W_up, stride_gu, max_tiles, t, ep);
      case GemmEpilogue::kProduct:
        return launch_bf16<kEpiProduct>(stream, X, ldx, d_model, d_ff, n_experts, W_gate, W_up, stride_gu, max_tiles, t, ep);
      default:
        return hipErrorInvalidValue;
    }
  }
  dim3 grid((unsigned)((d_ff + F32_BN - 1) / F32_BN), (unsigned)max_tiles);
  auto kern = e.mode == GemmEpilogue::kStats    ? grouped_gemm_f32_kernel<kEpiStats>
              : e.mode == GemmEpilogue::kHidden ? grouped_gemm_f32_kernel<kEpiHidden>
                                                : grouped_gemm_f32_kernel<kEpiProduct>;
  if (e.mode < GemmEpilogue::kStats || e.mode > GemmEpilogue::kProduct) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, static_cast<const float*>(X), ldx, (int)d_model, (int)d_ff,
                     static_cast<const float*>(W_gate), static_cast<const float*>(W_up), stride_gu, t.offsets,
                     t.tile_offset, t.tile_expert, t.perm, t.w_perm, n_experts, ep);
  return hipGetLastError();
}

template <int EPI, class TABLE>
static hipError_t launch_compact(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model, const void* Wg,
                                 const void* Wu, const TABLE& tab, int k_round, bool tail, int64_t n_tiles_n_max,
                                 int max_tiles, const BucketTables& t, int32_t* scratch, const EpiArgs& ep) {
  // tail: some K extent is not a multiple of the K tile, or an operand is too large for 32-bit offsets
  using C = Bf16Cfg;
  int64_t a_ld = ldx, b_rows = 0, b_ld = d_model;
  if constexpr (std::is_same<TABLE, CompactRows>::value) {
    for (int e = 0; e < tab.n_experts; ++e) b_rows = std::max<int64_t>(b_rows, tab.row_off[e + 1] - tab.row_off[e]);
  } else {
    b_rows = d_model;
    b_ld = a_ld = 0;
    for (int e = 0; e < tab.n_experts; ++e) {
      b_ld = std::max<int64_t>(b_ld, tab.ld_off[e + 1] - tab.ld_off[e]);
      a_ld = std::max<int64_t>(a_ld, (tab.count[e] + k_round - 1) / k_round * k_round);
    }
  }
  tail = tail || !fits_32bit_offsets((int64_t)max_tiles * C::BM, a_ld, b_rows, b_ld);
  auto kern = tail ? grouped_gemm_bf16_compact_kernel<C, true, EPI, TABLE>
                   : grouped_gemm_bf16_compact_kernel<C, false, EPI, TABLE>;
  static bool attr_set[2] = {false, false};
  if (!attr_set[tail]) {
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, C::kSmemBytes);
    if (err != hipSuccess) return err;
    attr_set[tail] = true;
  }
  hipLaunchKernelGGL((compact_work_kernel<TABLE>), dim3(1), dim3(CAMERA_MAX_EXPERTS), 0, stream, tab, (int)d_model, C::BN, C::KT, k_round,
                     t.offsets, t.tile_offset, scratch);
  // an upper bound of the tile count, shared evenly between the XCDs: a workgroup walks on through its XCD's
  // range where the cuts by cost give that XCD more (cheaper) tiles than that
  const int64_t n_blocks = (max_tiles * n_tiles_n_max + kXcds - 1) / kXcds * kXcds;
  if (n_blocks >= (int64_t(1) << 31)) return hipErrorInvalidValue;
  if (n_blocks == 0) return hipGetLastError();
  hipLaunchKernelGGL(kern, dim3((unsigned)n_blocks), dim3(C::kThreads), C::kSmemBytes, stream,
                     static_cast<const __hip_bfloat16*>(X), ldx, (int)d_model, static_cast<const __hip_bfloat16*>(Wg),
                     static_cast<const __hip_bfloat16*>(Wu), tab, k_round, t.offsets, t.tile_offset, scratch, t.perm,
                     t.w_perm, static_cast<const __hip_bfloat16*>(t.zeros), ep);
  return hipGetLastError();
}

hipError_t launch_compact_hidden_gemm(hipStream_t stream, const void* X, int64_t ldx, int64_t d_model,
                                      const void* W_gate, const void* W_up, const CompactRows& tab, int widest,
                                      int max_tiles, const BucketTables& t, int32_t* scratch, void* hidden,
                                      int k_round) {
  EpiArgs ep{nullptr, nullptr, hidden, nullptr, nullptr, 0, 0, 0, k_round};
  return launch_compact<kEpiHidden>(stream, X, ldx, d_model, W_gate, W_up, tab, k_round, d_model % Bf16Cfg::KT != 0,
                                    (widest + Bf16Cfg::BN - 1) / Bf16Cfg::BN, max_tiles, t, scratch, ep);
}

hipError_t launch_compact_down_gemm(hipStream_t stream, const void* hidden, int64_t d_model, const void* W_down,
                                    const CompactDown& tab, int max_tiles, const BucketTables& t, int32_t* scratch,
                                    float* product) {
  const int64_t half = d_model / 2;
  EpiArgs ep{nullptr, nullptr, nullptr, nullptr, product, d_model, (int)half, 0, 0};
  return launch_compact<kEpiProduct>(stream, hidden, 0, d_model, W_down, W_down, tab, tab.k_round,
                                     tab.k_round % Bf16Cfg::KT != 0, (half + Bf16Cfg::BN - 1) / Bf16Cfg::BN, max_tiles, t,
                                     scratch, ep);
}

}  // namespace camera

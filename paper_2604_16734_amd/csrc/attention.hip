// Attention of one block of queries over cache U block (Eq. 1 of the paper),
// for gfx950: bf16 MFMA 32x32x16, wave64, K and V tiles staged through LDS.
//
// Formulation.  Every wave owns QT tiles of 32 query rows and works on the
// TRANSPOSED problem: S^T = K Q^T (A operand = K tile from LDS, B operand = Q
// held in registers for the whole kernel) and O^T = V^T P^T (A operand = V^T
// from LDS, B operand = P^T).  In the 32x32 accumulator layout a lane holds one
// column, so with the transposed problem a lane holds ONE query row: the
// softmax reference and the running sum are one scalar per lane, and the
// exponentiated S^T accumulators are, register for register, the B operand of
// the second product.  P never touches LDS and is never shuffled between lanes.
//
// The contraction index of an MFMA may be permuted freely as long as A and B
// agree.  For O^T the index is the key position: accumulator register r of lane
// (g = lane / 32) holds key  8 (r / 4) + 4 g + r % 4  of the 32-key block, so
// registers 8 m .. 8 m + 7 are fed to MFMA m of the block, and the V^T operand
// is gathered in exactly that key order.
//
// Staging.  K and V tiles go from global memory straight into LDS
// (global_load_lds, 16 bytes per lane, no registers, no LDS store
// instructions), row-major as they are in memory.  A wave instruction fills
// 1 KiB of consecutive LDS, so rows cannot be padded; instead the 16-byte chunks
// of a row are XOR-swizzled by the row number on the way in, each tensor with
// the pattern that makes its own fragment reads conflict-free.  The K operand is
// one ds_read_b128 per fragment; the V^T operand is two ds_read_b64_tr_b16:
// within 16 lanes, lane j receives element j % 4 of the 8-byte chunks addressed
// by lanes j / 4, j / 4 + 4, j / 4 + 8, j / 4 + 12, i.e. four keys of one channel.
//
// A workgroup is QW x KS waves: QW groups of query rows times a KS-way split of
// every staged key tile.  A wave takes 64 keys of each tile as two 32-key
// blocks X and Y; the KS partial results of a row are merged through LDS at the
// end.  The split keeps all 1024 SIMDs busy when a block of the prefix has
// fewer than 1024 wave-sized row tiles.  Three shapes are built: 2 x 2 waves of
// 64 rows (one wave per SIMD, 512 registers), 4 x 2 waves of 32 rows (two waves
// per SIMD, 256 registers each; the fastest on the large shapes) and 2 x 2 waves
// of 32 rows for blocks too small to fill the chip with 128-row workgroups.
//
// Schedule.  Matrix and vector work of one wave are made to overlap in program
// order.  With S_X(t) = scores of block X of tile t, the loop body is
//   phase 1   MFMA: S_Y(t), O += P_Y(t-1) V     | VALU: P_X(t) = exp(S_X(t) - m)
//   barrier
//   phase 2   MFMA: S_X(t+1), O += P_X(t) V     | VALU: P_Y(t) = exp(S_Y(t) - m)
//             and, first thing after the barrier, the loads of K(t+2) and
//             V(t+1) into the buffers whose last readers were in phase 1.
// LDS holds two K tiles and two V tiles; one barrier per tile is enough because
// a buffer is only overwritten in the phase after its last reader.
//
// Softmax reference.  exp(S - m) is exact for ANY per-row reference m as long as
// nothing overflows, so the fast loop fixes m at the maximum of the row's first
// visible block and never touches O again: no rescaling, no branch.  Every block
// maximum is still computed; should one exceed m by more than 2^64 (fp32 would
// overflow near 2^127) the workgroup raises a flag, throws its result away and
// redoes its rows with the textbook online softmax in a plain loop.  Real
// attention logits never get there; adversarial inputs stay correct.
#include <type_traits>

#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float kRedoLog2 = 64.f;   // redo a row tile when a block maximum exceeds the reference by 2^64

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(unsigned, b);
}

// value of the same row held by the other half of the wave (lane ^ 32)
__device__ __forceinline__ float max_with_other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ bf16x8 lds_read_b128(const u16* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}
// two transposing reads: keys k .. k+3 and k+8 .. k+11 of this lane's channel
__device__ __forceinline__ bf16x8 lds_read_vt(const u16* p, int eight_rows) {
  const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)(p));
  const i16x4 hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)(p + eight_rows));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

template <int D, int QT, int QW, int KS>
struct Shape {
  static constexpr int kWaves = QW * KS;
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kRows = QW * QT * 32;          // query rows per workgroup
  static constexpr int kTk = KS * 64;                 // keys per staged tile
  static constexpr int kChunks = D / 8;               // 16-byte chunks per row
  static constexpr int kRowsPerLoad = 64 / kChunks;   // rows one wave instruction brings in
  static constexpr int kRowGroup = kWaves * kRowsPerLoad;  // rows the waves bring in per step
  static constexpr int kLoadsPerWave = kTk / kRowGroup;            // per tensor and tile
  static constexpr int kTile = kTk * D;               // bf16 elements of a K or V tile, unpadded
  static constexpr int kTileBytes = 4 * kTile * 2;    // two K and two V buffers
  static constexpr int kMergeFloats = QT * (D / 32) * 16 * 64 + 2 * QT * 64;  // per wave
  static constexpr int kMergeBytes = (KS - 1) * QW * kMergeFloats * 4;
  static constexpr int kStripRow = 2 * D + 16;        // bytes of an output row staged in LDS, padded
  static constexpr int kEpilogueBytes = kMergeBytes + QW * 32 * kStripRow;
  static constexpr int kMainBytes = kTileBytes > kEpilogueBytes ? kTileBytes : kEpilogueBytes;
  // behind the tiles, for the score sweep: the finished row statistics of the workgroup's rows
  static constexpr int kScoreBytes = QW * QT * 32 * 4;
  static constexpr int kLdsBytes = kMainBytes + kScoreBytes;
  static_assert(kLdsBytes <= 160 * 1024, "LDS of a CU");
  static_assert(kWaves == 4 || kWaves == 8, "four or eight waves per workgroup");
  static_assert(kTk == 128, "the staging map assumes 128-key tiles");
};

template <int D, int QT, int QW, int KS>
__global__ void __launch_bounds__((Shape<D, QT, QW, KS>::kThreads))
attention_kernel(const AttnArgs a) {
  using S = Shape<D, QT, QW, KS>;
  constexpr int kThreads = S::kThreads;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  u16* const lds_k = reinterpret_cast<u16*>(lds_raw);              // [2][kTile]
  u16* const lds_v = lds_k + 2 * S::kTile;                         // [2][kTile]
  float* const lse_lds = reinterpret_cast<float*>(lds_raw + S::kMainBytes);   // [QW][QT][32]

  // XCD-aware order: consecutive work items (same KV head) land on one die
  const int xcd = blockIdx.x % kXcds;
  const int w = xcd * a.work_per_xcd + blockIdx.x / kXcds;
  if (w >= a.total_work) return;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int rt = a.n_row_tiles - 1 - (w % a.n_row_tiles);   // long rows first
  const int h = w / a.n_row_tiles;
  const int hk = h / group;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  // the same number in a scalar register: what a wave derives from it (its rows, its tile counts,
  // its branches, addresses of its loads) is then uniform for the compiler as well
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int qw = wave_s / KS;
  const int ks = wave_s % KS;
  const int l32 = lane & 31;
  const int g = lane >> 5;

  const int n = a.n, c = a.c, n_cand = c + a.n_keys, shift = a.shift;
  // Rows.  A head's rows are cut into blocks of QT * 32 (one per group of KS waves); later rows
  // see more of the block's keys.  A workgroup takes QW / 2 blocks from the front of the head
  // and QW / 2 from the back, so every workgroup has the same amount of work; and since waves w
  // and w + 4 of a workgroup share a SIMD, every SIMD of the eight-wave shape gets one early and
  // one late block: when the early one has run out of visible keys the late one has the SIMD to
  // itself.  first_row_of(q) is the first row of the block the waves with qw = q work on.
  auto first_row_of = [&](int q) __attribute__((always_inline)) -> int {
    constexpr int kHalf = QW / 2;
    const int blocks = a.n_row_tiles * QW;
    const int b = q < kHalf ? rt * kHalf + q : blocks - (rt + 1) * kHalf + (q - kHalf);
    return b * QT * 32;
  };
  const int q0 = first_row_of(qw);                   // first query row of this wave
  // the workgroup as a whole: the last block is the latest; tiles are staged for everybody
  const int wg_rows_end = min(n, first_row_of(QW - 1) + QT * 32);
  const int n_tiles = (min(n_cand, c + wg_rows_end + shift) + S::kTk - 1) / S::kTk;
  // this wave: the tiles its rows can see, and those among them visible in full to all its rows
  const int my_rows_end = min(n, q0 + QT * 32);      // = n for a block that lies past the end: computed, not stored
  const int my_tiles = (min(n_cand, c + my_rows_end + shift) + S::kTk - 1) / S::kTk;
  const int n_plain = min(my_tiles, (min(c + q0 + shift + 1, n_cand)) / S::kTk);
  const u16* kc = a.k_cache + (size_t)hk * a.budget * D;
  const u16* vc = a.v_cache + (size_t)hk * a.budget * D;
  const u16* kn = a.k_new + (size_t)hk * D;
  const u16* vn = a.v_new + (size_t)hk * D;
  const int new_stride = a.n_kv_heads * D;
  const float sl2 = a.scale_log2;

  // ---- staging: global -> LDS, 16 bytes per lane, chunks swizzled by row.
  // Instruction j of wave w brings in rows kRowGroup j + kRowsPerLoad w + (0 .. kRowsPerLoad-1)
  // of the tile; a lane always handles the same row residue, so its swizzle is a constant.
  const int ld_sub = lane / S::kChunks, ld_pos = lane % S::kChunks;
  const int ld_row = S::kRowsPerLoad * wave + ld_sub;          // + kRowGroup j
  const int ld_chunk_k = ld_pos ^ (ld_row % S::kChunks);
  // V rows are read four at a time by each half of a wave (transposing 8-byte reads, 64 bytes
  // of each row): the swizzle sends those four 64-byte pieces to four different quarters of the
  // 64 banks (D = 128: a row spans all banks; D = 64: rows r and r + 2 share their banks)
  auto v_swizzle = [](int row) { return 4 * ((row % 4) >> (D == 64 ? 1 : 0)); };
  const int ld_chunk_v = ld_pos ^ v_swizzle(ld_row);
  // LDS destination of instruction j into `tile`, as the byte address M0 wants: wave-uniform and
  // all scalar arithmetic (the wave number is read into a scalar register once)
  const unsigned lds_base =
      __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) void*)lds_raw);
  auto lds_dst = [&](const u16* tile, int j) __attribute__((always_inline)) -> unsigned {
    return lds_base + 2u * (unsigned)((int)(tile - lds_k) + (S::kRowGroup * j + S::kRowsPerLoad * wave_s) * D);
  };
  // Issued as inline assembly on purpose: the compiler then does not know that these loads write
  // LDS and does not make every later LDS read wait for them.  Ordering is this kernel's job:
  // wait_loads() before the barrier that publishes a tile.
  // Two address forms: a 64-bit address per lane (tiles that straddle the cache and the block or
  // run past the end), and a scalar base with a 32-bit offset per lane (uniform tiles: the base
  // moves from tile to tile on the scalar unit, the lane offsets never change).
  auto load16 = [&](const u16* src, unsigned lds_addr) __attribute__((always_inline)) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr)
                 : "m0", "memory");
  };
  auto load16_scalar_base = [&](const u16* base, unsigned lane_bytes, unsigned lds_addr) __attribute__((always_inline)) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_bytes), "s"(base),
                 "s"(lds_addr)
                 : "m0", "memory");
  };
  auto wait_loads = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0), nothing else
  };
  // tile t lies entirely in the cache or entirely in the block: one base, one stride
  auto tile_is_uniform = [&](int t) __attribute__((always_inline)) -> bool {
    const int base = t * S::kTk;
    return base + S::kTk <= c || (base >= c && base + S::kTk <= n_cand);
  };
  // A uniform tile: the scalar address of the first row this wave brings in, the row stride, and
  // which of the lane offsets goes with it.  The lane part of an address is
  // (ld_sub rows + the swizzled chunk) in bytes, one value per tensor and per stride.
  struct UniformSrc {
    const u16* base;
    int stride;
    bool cached;
  };
  auto uniform_src = [&](const u16* cache, const u16* fresh, int t) __attribute__((always_inline)) -> UniformSrc {
    const int base = t * S::kTk;
    const bool cached = base < c;
    const int stride = cached ? D : new_stride;
    const u16* p = cached ? cache + (size_t)base * D : fresh + (size_t)(base - c) * new_stride;
    return UniformSrc{p + (size_t)(S::kRowsPerLoad * wave_s) * stride, stride, cached};
  };
  const unsigned lane_k_cache = 2u * (unsigned)(ld_sub * D + 8 * ld_chunk_k);
  const unsigned lane_k_new = 2u * (unsigned)(ld_sub * new_stride + 8 * ld_chunk_k);
  const unsigned lane_v_cache = 2u * (unsigned)(ld_sub * D + 8 * ld_chunk_v);
  const unsigned lane_v_new = 2u * (unsigned)(ld_sub * new_stride + 8 * ld_chunk_v);
  auto issue_any_one = [&](const u16* cache, const u16* fresh, u16* tile, int t, int chunk, int j)
      __attribute__((always_inline)) {
    const int kv = min(t * S::kTk + S::kRowGroup * j + ld_row, n_cand - 1);   // past the end: any finite row
    const u16* src = kv < c ? cache + (size_t)kv * D : fresh + (size_t)(kv - c) * new_stride;
    load16(src + 8 * chunk, lds_dst(tile, j));
  };
  auto issue_any = [&](const u16* cache, const u16* fresh, u16* tile, int t, int chunk)
      __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < S::kLoadsPerWave; ++j) issue_any_one(cache, fresh, tile, t, chunk, j);
  };

  // ---- per-lane LDS read offsets (bf16 elements), swizzle folded in
  // K operand, d-slice st: row (block + l32), chunk (2 st + g) ^ (row % kChunks)
  int k_off[D / 16];
  {
    const int q = g ^ (l32 % S::kChunks);
#pragma unroll
    for (int st = 0; st < D / 16; ++st) k_off[st] = l32 * D + 8 * ((2 * st) ^ q);
  }
  // V^T operand, channel tile dt: this lane addresses key row 4 g + (lane % 16) / 4 (+ block + 16 mm
  // + 8 h) and the 8-byte half (lane % 4) & 1 of chunk 4 dt + 2 ((lane / 16) % 2) + (lane % 4) / 2
  int v_off[D / 32];
  {
    const int rsub = 4 * g + ((lane & 15) >> 2);
    const int z = v_swizzle(rsub);
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
      const int chunk = (4 * dt + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) ^ z;
      v_off[dt] = rsub * D + 8 * chunk + 4 * (lane & 1);
    }
  }

  // ================================================================ fast path
  bool redo = false;
  {
    // ---- Q fragments: B operand, lane holds Q[q0 + 32 t + l32][16 s + 8 g .. + 7]
    bf16x8 qf[QT][D / 16];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const int row = min(q0 + 32 * t + l32, n - 1);     // rows past the block are computed, not stored
      const u16* src = a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * g;
#pragma unroll
      for (int s = 0; s < D / 16; ++s)
        qf[t][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * s));
    }
    // Make the compiler finish these loads here.  Left pending, it would wait for them inside the
    // loop, at a point where the hand-issued tile loads are in flight, and drain those as well.
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
      for (int s = 0; s < D / 16; ++s) asm volatile("" ::"v"(qf[t][s]));
    f32x16 o[QT][D / 32];
    float m_ref[QT], l_run[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      m_ref[t] = -INFINITY;
      l_run[t] = 0.f;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][dt][r] = 0.f;
    }
    const float redo_raw = kRedoLog2 / sl2;       // the margin in units of the raw dot product
    const int blk_off = 64 * ks * D;               // this wave's 64 keys inside a tile

    // Hide block keys a row may not see, fix the reference at the first visible block, and
    // watch for a block maximum far above the reference.
    // `track` is off for the tiles after the first plain one: every row has its reference by
    // then, and a logit far above it shows up in the row sum instead (checked after the loop).
    auto prepare = [&](f32x16 (&s)[QT], int kb, auto mask, auto track) __attribute__((always_inline)) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        if constexpr (decltype(mask)::value) {
          // key kb + 8 (r / 4) + 4 g + r % 4 is visible when cached, or a block key not after the row
          const int lim = min(q0 + 32 * t + l32 + shift + c, n_cand - 1) - kb - 4 * g;
#pragma unroll
          for (int r = 0; r < 16; ++r) s[t][r] = (8 * (r >> 2) + (r & 3) <= lim) ? s[t][r] : -INFINITY;
        }
        if constexpr (decltype(track)::value) {
          float v = s[t][0];
#pragma unroll
          for (int r = 1; r < 16; ++r) v = fmaxf(v, s[t][r]);
          const float mx = max_with_other_half(v);
          m_ref[t] = (m_ref[t] == -INFINITY) ? mx : m_ref[t];
          redo |= mx > m_ref[t] + redo_raw;
        }
      }
    };

    // One phase, as one basic block: MFMA i is followed by the exponentials of 128 / D elements
    // of the S block computed in the previous phase, and LDS fragment reads run kAhead operands
    // ahead of their use.  The source is written in exactly that order and a scheduling fence after
    // every MFMA's share keeps the compiler from regrouping it (left to itself it bunches the
    // MFMAs and piles the exponentials up behind them).
    //   s_exp -> p_out   P = exp2((S - m) * scale) for the block whose scores are ready
    //   s_new            S^T of the next block = K[kt rows] Q^T
    //   p_pend, vt       O^T += V^T P^T for the block exponentiated one phase ago
    auto phase_core = [&](const f32x16 (&s_exp)[QT], unsigned (&p_out)[QT][8], f32x16 (&s_new)[QT],
                          const u16* kt, const unsigned (&p_pend)[QT][8], const u16* vt, auto&& after_mfma)
        __attribute__((always_inline)) {
      constexpr int kNK = D / 16;            // K fragments
      constexpr int kNV = (D / 32) * 2;      // V^T fragments
      constexpr int kAhead = D / 32;
      constexpr int kPerMfma = 128 / D;      // elements exponentiated per MFMA
      float neg[QT], sum[QT];
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const float m_use = (m_ref[t] == -INFINITY) ? 0.f : m_ref[t];   // row has seen nothing yet
        neg[t] = -m_use * sl2;
        sum[t] = 0.f;
      }
      bf16x8 kfr[kNK], vfr[kNV];
      auto read_k = [&](int st) __attribute__((always_inline)) { kfr[st] = lds_read_b128(kt + k_off[st]); };
      auto read_v = [&](int vi) __attribute__((always_inline)) {
        vfr[vi] = lds_read_vt(vt + v_off[vi / 2] + 16 * (vi % 2) * D, 8 * D);
      };
      // The vector work of an element is a chain (scale-and-shift, exponential, add to the row sum,
      // pack) and an instruction that needs the result of the one before it stalls the wave, the
      // exponential most of all.  So the chain is skewed over the MFMAs: each call computes the
      // argument of the next element, the exponential of this one, and adds and packs the one before.
      constexpr int kElems = QT * 16;
      int ei = 0;   // next element to exponentiate
      float arg = __builtin_fmaf(s_exp[0][0], sl2, neg[0]), pe1 = 0.f, pe2 = 0.f;
      auto finish_element = [&](int e) __attribute__((always_inline)) {      // element e: pe1, the one before: pe2
        const int t = e / 16, r = e % 16;
        sum[t] += pe1;
        // the sums are only needed after the loop, and left alone the compiler gathers the
        // additions of several phases in one place, keeping every exponential alive until then
        asm volatile("" : "+v"(sum[t]));
        if (r & 1) p_out[t][r >> 1] = pack_bf16(pe2, pe1);
      };
      auto exp_some = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kPerMfma; ++k, ++ei) {
          const float pe = __builtin_amdgcn_exp2f(arg);
          if (ei + 1 < kElems) arg = __builtin_fmaf(s_exp[(ei + 1) / 16][(ei + 1) % 16], sl2, neg[(ei + 1) / 16]);
          if (ei >= 1) finish_element(ei - 1);
          pe2 = pe1;
          pe1 = pe;
        }
      };
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < kAhead; ++st) read_k(st);
      __builtin_amdgcn_sched_barrier(0);     // all of them before the first MFMA
#pragma unroll
      for (int st = 0; st < kNK; ++st) {
        if (st + kAhead < kNK) read_k(st + kAhead);
        else read_v(st + kAhead - kNK);
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          s_new[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[st], qf[t][st], st == 0 ? zero : s_new[t], 0, 0, 0);
          exp_some();
          after_mfma(std::integral_constant<int, 0>{}, st * QT + t);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int vi = 0; vi < kNV; ++vi) {
        if (vi + kAhead < kNV) read_v(vi + kAhead);
        const int dt = vi / 2, mm = vi % 2;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          const u32x4 pw = {p_pend[t][4 * mm], p_pend[t][4 * mm + 1], p_pend[t][4 * mm + 2], p_pend[t][4 * mm + 3]};
          o[t][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[vi], __builtin_bit_cast(bf16x8, pw), o[t][dt], 0, 0, 0);
          exp_some();
          after_mfma(std::integral_constant<int, 1>{}, vi * QT + t);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      finish_element(kElems - 1);
#pragma unroll
      for (int t = 0; t < QT; ++t) l_run[t] += sum[t];
    };

    // ---- prologue: K(0), K(1), V(0) into LDS, S_X(0) computed
    f32x16 sx[QT], sy[QT];
    unsigned px[QT][8], py[QT][8];
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
      for (int r = 0; r < 8; ++r) { px[t][r] = 0u; py[t][r] = 0u; }
    issue_any(kc, kn, lds_k, 0, ld_chunk_k);
    issue_any(vc, vn, lds_v, 0, ld_chunk_v);
    issue_any(kc, kn, lds_k + S::kTile, 1, ld_chunk_k);
    // V buffer 1 is read as "V(-1)" with P = 0 in the first phase: make it finite
    for (int i = tid; i < S::kTile / 8; i += kThreads)
      reinterpret_cast<u32x4*>(lds_v + S::kTile)[i] = u32x4{0u, 0u, 0u, 0u};
    wait_loads();
    __syncthreads();
    {
      // S_X(0) without anything to overlap with
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) sx[t][r] = 0.f;
#pragma unroll
      for (int st = 0; st < D / 16; ++st) {
        const bf16x8 ka = lds_read_b128(lds_k + blk_off + k_off[st]);
#pragma unroll
        for (int t = 0; t < QT; ++t) sx[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[t][st], sx[t], 0, 0, 0);
      }
    }

    // kTag = t & 1 as a compile-time constant in the steady-state loop, -1 for "use t & 1".
    // The steady-state loop also knows that the tiles it prefetches are uniform.
    auto body = [&](int t, auto buf_tag, auto mask, auto track) __attribute__((always_inline)) {
      constexpr int kTag = decltype(buf_tag)::value;
      const int buf = kTag >= 0 ? kTag : (t & 1);
      const int kb = t * S::kTk + ks * 64;
      u16* k_cur = lds_k + buf * S::kTile;
      u16* k_nxt = lds_k + (buf ^ 1) * S::kTile;
      u16* v_cur = lds_v + buf * S::kTile;
      u16* v_prv = lds_v + (buf ^ 1) * S::kTile;
      // ---- phase 1: P_X(t), S_Y(t), O += P_Y(t-1) V(t-1)
      prepare(sx, kb, mask, track);
      phase_core(sx, px, sy, k_cur + blk_off + 32 * D, py, v_prv + blk_off + 32 * D, [](auto, int) {});
      // P_X is only read in phase 2, and the compiler would gladly take its exponentials there,
      // all in a lump behind the barrier: make them due here, in the shadow of this phase's MFMAs
#pragma unroll
      for (int tq = 0; tq < QT; ++tq)
#pragma unroll
        for (int r = 0; r < 8; ++r) asm volatile("" ::"v"(px[tq][r]));
      __builtin_amdgcn_sched_barrier(0);
      wait_loads();               // the loads this wave issued in the last phase 2 have landed
      __syncthreads();
      // ---- phase 2: P_Y(t), S_X(t+1), O += P_X(t) V(t); the loads of K(t+2) and V(t+1) are spread
      // over the matrix instructions so that their issue does not stall the wave in one burst
      prepare(sy, kb + 32, mask, track);
      constexpr int kPerHalf = QT * (D / 16);              // MFMAs in each half of a phase
      constexpr int kEvery = kPerHalf / S::kLoadsPerWave;  // one load every kEvery MFMAs
      static_assert(kEvery >= 1 && kPerHalf % S::kLoadsPerWave == 0, "loads must fit the phase");
      if (kTag >= 0) {
        const UniformSrc k_src = uniform_src(kc, kn, t + 2 < n_tiles ? t + 2 : t);
        const UniformSrc v_src = uniform_src(vc, vn, t + 1 < n_tiles ? t + 1 : t);
        const unsigned k_lane = k_src.cached ? lane_k_cache : lane_k_new;
        const unsigned v_lane = v_src.cached ? lane_v_cache : lane_v_new;
        phase_core(sy, py, sx, k_nxt + blk_off, px, v_cur + blk_off, [&](auto half, int i) __attribute__((always_inline)) {
          if (i % kEvery != 0) return;
          const int j = i / kEvery;
          if (decltype(half)::value == 0)
            load16_scalar_base(k_src.base + (size_t)(S::kRowGroup * j) * k_src.stride, k_lane, lds_dst(k_cur, j));
          else
            load16_scalar_base(v_src.base + (size_t)(S::kRowGroup * j) * v_src.stride, v_lane, lds_dst(v_prv, j));
        });
      } else {
        phase_core(sy, py, sx, k_nxt + blk_off, px, v_cur + blk_off, [&](auto half, int i) __attribute__((always_inline)) {
          if (i % kEvery != 0) return;
          const int j = i / kEvery;
          if (decltype(half)::value == 0) issue_any_one(kc, kn, k_cur, t + 2, ld_chunk_k, j);
          else issue_any_one(vc, vn, v_prv, t + 1, ld_chunk_v, j);
        });
      }
    };
    typedef std::integral_constant<int, 0> Even;
    typedef std::integral_constant<int, 1> Odd;
    typedef std::integral_constant<int, -1> Any;
    // The fast body of tile t needs: tile t visible in full to every row of the workgroup, and the
    // tiles it prefetches (V of t + 1, K of t + 2) uniform, or past the workgroup's last tile (then
    // it fetches its own tile again, into a buffer nobody reads any more).
    auto fast_ok = [&](int t) __attribute__((always_inline)) -> bool {
      return t < n_plain && tile_is_uniform(t + 1 < n_tiles ? t + 1 : t) && tile_is_uniform(t + 2 < n_tiles ? t + 2 : t);
    };
    int n_fast = 0;                // tiles the fast bodies take, two at a time
    while (fast_ok(n_fast) && fast_ok(n_fast + 1)) n_fast += 2;
    int t = 0;
    if (n_fast >= 2) {
      // tile 0 is plain: it gives every row its reference, and nothing after it looks at maxima
      body(0, Even{}, std::false_type{}, std::true_type{});
      body(1, Odd{}, std::false_type{}, std::false_type{});
      t = 2;
    }
    for (; t < n_fast; t += 2) {
      body(t, Even{}, std::false_type{}, std::false_type{});
      body(t + 1, Odd{}, std::false_type{}, std::false_type{});
    }
    for (; t < my_tiles; ++t)      // masking a fully visible tile is harmless
      body(t, Any{}, std::true_type{}, std::true_type{});
    {
      // O += P_Y V of this wave's last tile.  That V was published by the barrier inside the last
      // body and is overwritten only after the barrier of the next tile, which this wave has
      // not reached.
      const u16* vt = lds_v + ((my_tiles + 1) & 1) * S::kTile + blk_off + 32 * D;
#pragma unroll
      for (int vi = 0; vi < (D / 32) * 2; ++vi) {
        const int dt = vi / 2, mm = vi % 2;
        const bf16x8 va = lds_read_vt(vt + v_off[dt] + 16 * mm * D, 8 * D);
#pragma unroll
        for (int tq = 0; tq < QT; ++tq) {
          const u32x4 pw = {py[tq][4 * mm], py[tq][4 * mm + 1], py[tq][4 * mm + 2], py[tq][4 * mm + 3]};
          o[tq][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, pw), o[tq][dt], 0, 0, 0);
        }
      }
    }
    // The workgroup's later tiles, which no row of this wave sees: keep in step with the others
    // (one barrier per tile) and bring in this wave's share of the tiles they read.
    for (; t < n_tiles; ++t) {
      wait_loads();
      __syncthreads();
      issue_any(kc, kn, lds_k + (t & 1) * S::kTile, t + 2, ld_chunk_k);
      issue_any(vc, vn, lds_v + ((t & 1) ^ 1) * S::kTile, t + 1, ld_chunk_v);
    }
    wait_loads();
    __syncthreads();               // nothing is on its way into LDS any more
    // a logit more than 2^64 above its row's reference in a tile that did not track maxima has
    // pushed the row sum past 2^64 (or to infinity or NaN)
#pragma unroll
    for (int tq = 0; tq < QT; ++tq) redo |= !(l_run[tq] <= 0x1p64f);
    redo = __syncthreads_or(redo) != 0;     // workgroup-uniform; also: everybody is done with the tiles

    if (!redo) {
      // lanes l and l + 32 each summed half of the keys of a row
#pragma unroll
      for (int tq = 0; tq < QT; ++tq) l_run[tq] = sum_with_other_half(l_run[tq]);
      // ---- merge the KS partial results of every row through LDS
      if (KS > 1) {
        float* mrg = reinterpret_cast<float*>(lds_raw);
        if (ks > 0) {
          float* mine = mrg + (size_t)((ks - 1) * QW + qw) * S::kMergeFloats;
#pragma unroll
          for (int tq = 0; tq < QT; ++tq) {
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
              for (int r = 0; r < 16; ++r)
                mine[((tq * (D / 32) + dt) * 16 + r) * 64 + lane] = o[tq][dt][r];
            mine[QT * (D / 32) * 16 * 64 + tq * 64 + lane] = m_ref[tq];
            mine[QT * (D / 32) * 16 * 64 + (QT + tq) * 64 + lane] = l_run[tq];
          }
        }
        __syncthreads();
        if (ks == 0) {
#pragma unroll
          for (int tq = 0; tq < QT; ++tq) {
            float mt = m_ref[tq];
            for (int s2 = 1; s2 < KS; ++s2) {
              const float* other = mrg + (size_t)((s2 - 1) * QW + qw) * S::kMergeFloats;
              mt = fmaxf(mt, other[QT * (D / 32) * 16 * 64 + tq * 64 + lane]);
            }
            const float m_use = (mt == -INFINITY) ? 0.f : mt;
            const float f0 = __builtin_amdgcn_exp2f((m_ref[tq] - m_use) * sl2);
            l_run[tq] *= f0;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
              for (int r = 0; r < 16; ++r) o[tq][dt][r] *= f0;
            for (int s2 = 1; s2 < KS; ++s2) {
              const float* other = mrg + (size_t)((s2 - 1) * QW + qw) * S::kMergeFloats;
              const float ms = other[QT * (D / 32) * 16 * 64 + tq * 64 + lane];
              const float ls = other[QT * (D / 32) * 16 * 64 + (QT + tq) * 64 + lane];
              const float fs = __builtin_amdgcn_exp2f((ms - m_use) * sl2);
              l_run[tq] += ls * fs;
#pragma unroll
              for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                  o[tq][dt][r] += fs * other[((tq * (D / 32) + dt) * 16 + r) * 64 + lane];
            }
            m_ref[tq] = mt;
          }
        }
      }
      // ---- normalise and store; lane holds O[row][32 dt + 8 j + 4 g + 0..3].  The rows go
      // through a private LDS strip of the wave so that the global stores are whole 16-byte
      // chunks of consecutive addresses (a row of the output is 2 D contiguous bytes).
      if (ks == 0) {
        unsigned char* strip = lds_raw + S::kMergeBytes + (size_t)qw * 32 * S::kStripRow;
#pragma unroll
        for (int tq = 0; tq < QT; ++tq) {
          const int row = q0 + 32 * tq + l32;
          const float inv = 1.f / l_run[tq];
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              u32x2 pk;
              pk.x = pack_bf16(o[tq][dt][4 * j] * inv, o[tq][dt][4 * j + 1] * inv);
              pk.y = pack_bf16(o[tq][dt][4 * j + 2] * inv, o[tq][dt][4 * j + 3] * inv);
              *reinterpret_cast<u32x2*>(strip + l32 * S::kStripRow + 2 * (32 * dt + 8 * j + 4 * g)) = pk;
            }
          const float lse_row = m_ref[tq] * sl2 + __builtin_log2f(l_run[tq]);
          if (g == 0) lse_lds[(qw * QT + tq) * 32 + l32] = lse_row;
          if (g == 0 && row < n) a.lse2[(size_t)h * a.lse_stride + row] = lse_row;
#pragma unroll
          for (int it = 0; it < D / 16; ++it) {
            const int idx = it * 64 + lane;
            const int r = idx / (D / 8), ch = idx % (D / 8);
            const u32x4 val = *reinterpret_cast<const u32x4*>(strip + r * S::kStripRow + 16 * ch);
            const int orow = q0 + 32 * tq + r;
            if (orow < n && a.out != nullptr)
              *reinterpret_cast<u32x4*>(a.out + ((size_t)orow * a.n_q_heads + h) * D + 8 * ch) = val;
          }
        }
      }
    }
  }

  // ================================================================ careful path
  // Textbook online softmax, one 32-row tile per wave, one tile buffer, no overlap.
  // Only reached when a logit exceeded its row's reference by more than 2^64.
  if (redo) {
    const bool active = wave < S::kRows / 32;
    const int qs = active ? first_row_of(wave / QT) + 32 * (wave % QT) : 0;
    bf16x8 qf[D / 16];
    {
      const int row = min(qs + l32, n - 1);
      const u16* src = a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * g;
#pragma unroll
      for (int s = 0; s < D / 16; ++s)
        qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * s));
    }
    f32x16 o[D / 32];
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    for (int t = 0; t < n_tiles; ++t) {
      __syncthreads();                                   // the tile buffer is free
      issue_any(kc, kn, lds_k, t, ld_chunk_k);
      issue_any(vc, vn, lds_v, t, ld_chunk_v);
      wait_loads();
      __syncthreads();                                   // and full again
      if (!active) continue;
      for (int blk = 0; blk < S::kTk / 32; ++blk) {
        const int kb = t * S::kTk + 32 * blk;
        if (kb >= n_cand || (kb >= c && kb - c > qs + 31 + shift)) continue;    // nothing visible
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int st = 0; st < D / 16; ++st)
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_read_b128(lds_k + 32 * blk * D + k_off[st]), qf[st], s, 0, 0, 0);
        const int lim = min(qs + l32 + shift + c, n_cand - 1) - kb - 4 * g;
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[r] = (8 * (r >> 2) + (r & 3) <= lim) ? s[r] : -INFINITY;
          mx = fmaxf(mx, s[r]);
        }
        mx = max_with_other_half(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * sl2);
        const float neg = -m_use * sl2;
        unsigned pb[8];
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * r], sl2, neg));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * r + 1], sl2, neg));
          sum += p0 + p1;
          pb[r] = pack_bf16(p0, p1);
        }
        l_run = l_run * alpha + sum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
#pragma unroll
          for (int mm = 0; mm < 2; ++mm) {
            const bf16x8 va = lds_read_vt(lds_v + 32 * blk * D + v_off[dt] + 16 * mm * D, 8 * D);
            const u32x4 pw = {pb[4 * mm], pb[4 * mm + 1], pb[4 * mm + 2], pb[4 * mm + 3]};
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, pw), o[dt], 0, 0, 0);
          }
        }
      }
    }
    if (active) {
      l_run = sum_with_other_half(l_run);
      const int row = qs + l32;
      if (row < n) {
        const float inv = 1.f / l_run;
        if (a.out != nullptr) {
          u16* dstp = a.out + ((size_t)row * a.n_q_heads + h) * D + 4 * g;
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              u32x2 pk;
              pk.x = pack_bf16(o[dt][4 * j] * inv, o[dt][4 * j + 1] * inv);
              pk.y = pack_bf16(o[dt][4 * j + 2] * inv, o[dt][4 * j + 3] * inv);
              *reinterpret_cast<u32x2*>(dstp + 32 * dt + 8 * j) = pk;
            }
        }
        if (g == 0) a.lse2[(size_t)h * a.lse_stride + row] = m_run * sl2 + __builtin_log2f(l_run);
      }
      // wave w worked on row group w / QT, tile w % QT: the same order as the fast path's
      if (g == 0) lse_lds[wave * 32 + l32] = m_run * sl2 + __builtin_log2f(l_run);
    }
  }

  // ================================================================ scores
  // Eq. 4 needs every row's FINAL normaliser, so the column sums are a second sweep over the
  // workgroup's keys, now that its rows have their log-sum-exp.  The roles change: the workgroup's
  // query rows go into LDS once (row tiles of 32), and every wave takes every kWaves-th block of
  // 32 keys and keeps it in registers as the B operand while the row tiles pass by as the A
  // operand.  S = Q K^T then has one KEY column per lane and 16 rows of it in the lane's
  // registers: exp2(S - lse) is the exact softmax weight, the column sum is a running add inside
  // the lane, and after the last row tile the lane pair holds the sum over all of the workgroup's
  // rows.  No barrier, no exchange between waves, no atomics: one partial array per workgroup,
  // and the selection adds the arrays of a KV head in a fixed order.
  if (a.partial == nullptr) return;
  {
    constexpr int kNK = D / 16;
    constexpr int kRowTiles = QW * QT;
    static_assert(kRowTiles % 2 == 0, "the two accumulator sets alternate over the row tiles");
    __syncthreads();               // the statistics are in LDS; nobody needs the tile buffers any more
    // ---- the workgroup's query rows, swizzled like a K tile (chunk ch of row r at ch ^ (r % kChunks)):
    // row tile i holds rows first_row_of(i / QT) + 32 (i % QT) + 0..31, as lse_lds does
    u16* const q_lds = lds_k;
    for (int idx = tid; idx < kRowTiles * 32 * S::kChunks; idx += kThreads) {
      const int ch = idx % S::kChunks, r = (idx / S::kChunks) % 32, ti = idx / (S::kChunks * 32);
      const int row = min(first_row_of(ti / QT) + 32 * (ti % QT) + r, n - 1);
      const u32x4 v = *reinterpret_cast<const u32x4*>(a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * ch);
      *reinterpret_cast<u32x4*>(q_lds + (ti * 32 + r) * D + 8 * (ch ^ (r % S::kChunks))) = v;
    }
    // blocks of 32 keys that some row of the workgroup sees
    const int n_kb = (min(n_cand, c + wg_rows_end + shift) + 31) / 32;
    const int split = (h % group) * a.n_row_tiles + rt;
    float* const part = a.partial + ((size_t)hk * a.n_partials + split) * a.cand_stride;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    auto load_keys = [&](bf16x8 (&kf)[kNK], int kbi) __attribute__((always_inline)) {
      const int kv = min(kbi * 32 + l32, n_cand - 1);            // past the end: any real row, never stored
      const u16* src = (kv < c ? kc + (size_t)kv * D : kn + (size_t)(kv - c) * new_stride) + 8 * g;
#pragma unroll
      for (int st = 0; st < kNK; ++st)
        kf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * st));
    };
    // The scale behind an opaque copy for every variant of the stage below, made here, where all
    // lanes are active: the variants then share no subexpression, and the compiler cannot lift the
    // scale-and-shift of all sixteen elements above the branch that picks the variant, out of the
    // MFMAs' shadow.
    float sl2_copy[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("v_mov_b32 %0, %1" : "=v"(sl2_copy[i]) : "s"(sl2));
    // A slot is one key block against kR consecutive row tiles (64 rows when a workgroup has four
    // row tiles: its first two tiles are neighbours, and so are its last two): kR independent
    // chains of matrix instructions, and the costs a slot pays once -- the wait for its first
    // fragments, picking its variant, the distance to the first read of its result -- are shared
    // by twice the work.
    constexpr int kR = kRowTiles == 4 ? 2 : 1;
    constexpr int kSlots = kRowTiles / kR;
    static_assert(kSlots % 2 == 0, "the two accumulator sets alternate over the slots");
    // The slot before the current one: its logits wait in the other accumulator set.
    bool p_vis = false, p_plain = false;
    int p_kb0 = 0, p_row0 = 0, p_tile = 0;

    // One slot: the MFMAs of (key block, row tiles) into s_new among the exponentials of the slot
    // before it from s_exp, laid out MFMA by MFMA as in the first sweep.  Returns this lane's sum
    // of the exponentiated slot over its 16 kR rows.
    auto stage = [&](const f32x16 (&s_exp)[kR], f32x16 (&s_new)[kR], const u16* qt, const bf16x8 (&kf)[kNK],
                     auto do_mfma, auto do_exp, auto mask) __attribute__((always_inline)) -> float {
      constexpr bool kMfma = decltype(do_mfma)::value, kExp = decltype(do_exp)::value, kMask = decltype(mask)::value;
      constexpr int kElems = 16 * kR;
      constexpr int kPer = kMfma ? 16 / kNK : kElems;      // elements per matrix instruction
      constexpr int kAhead = kNK < 4 ? kNK : 4;
      bf16x8 qfr[kR][kNK];
      float ls[kR][16];
      float sum[2] = {0.f, 0.f};
      int first[kR];
      unsigned span[kR];
      if constexpr (kExp) {
        // statistics of the previous slot's rows: register r is row 8 (r / 4) + 4 g + r % 4 of its tile
#pragma unroll
        for (int t = 0; t < kR; ++t)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(&lse_lds[(p_tile + t) * 32 + 8 * j + 4 * g]);
            ls[t][4 * j] = v[0]; ls[t][4 * j + 1] = v[1]; ls[t][4 * j + 2] = v[2]; ls[t][4 * j + 3] = v[3];
          }
        if constexpr (kMask) {
          // key p_kb0 + l32 counts for the row at offset off = 8 (r / 4) + r % 4 from the tile's row
          // 4 g iff first <= off < rows left in the block
#pragma unroll
          for (int t = 0; t < kR; ++t) {
            const int row0 = p_row0 + 32 * t + 4 * g;
            first[t] = p_kb0 + l32 - c - shift - row0;            // negative for a cached key
            span[t] = (unsigned)max(n - row0 - first[t], 0);
          }
        }
      }
      const float sl2_here = sl2_copy[(kMfma ? 0 : 2) + (kMask ? 1 : 0)];
      int ei = 0;
      float arg = 0.f, pe1 = 0.f;
      if constexpr (kExp) arg = __builtin_fmaf(s_exp[0][0], sl2_here, -ls[0][0]);
      auto finish_element = [&](int e) __attribute__((always_inline)) {      // element e is in pe1
        float p = pe1;
        if constexpr (kMask) p = (unsigned)(8 * ((e % 16) >> 2) + (e & 3) - first[e / 16]) < span[e / 16] ? p : 0.f;
        sum[e & 1] += p;
        asm volatile("" : "+v"(sum[e & 1]));
      };
      auto exp_some = [&]() __attribute__((always_inline)) {
        if constexpr (kExp) {
#pragma unroll
          for (int k = 0; k < kPer; ++k, ++ei) {
            const float pe = __builtin_amdgcn_exp2f(arg);
            if (ei + 1 < kElems)
              arg = __builtin_fmaf(s_exp[(ei + 1) / 16][(ei + 1) % 16], sl2_here, -ls[(ei + 1) / 16][(ei + 1) % 16]);
            if (ei >= 1) finish_element(ei - 1);
            pe1 = pe;
          }
        }
      };
      if constexpr (kMfma) {
#pragma unroll
        for (int st = 0; st < kAhead; ++st)
#pragma unroll
          for (int t = 0; t < kR; ++t) qfr[t][st] = lds_read_b128(qt + t * 32 * D + k_off[st]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < kNK; ++st) {
#pragma unroll
          for (int t = 0; t < kR; ++t) {
            if (st + kAhead < kNK) qfr[t][st + kAhead] = lds_read_b128(qt + t * 32 * D + k_off[st + kAhead]);
            s_new[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr[t][st], kf[st], st == 0 ? zero : s_new[t], 0, 0, 0);
            exp_some();
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      } else {
        exp_some();
      }
      if constexpr (kExp) finish_element(kElems - 1);
      if constexpr (kMfma) {
        // A vector instruction may read the result of a 32x32x16 matrix instruction only twelve wait
        // states after it was issued.  The next reader of s_new sits in another basic block (the next
        // slot's variant, or a register copy the compiler puts at a block boundary), and measured
        // results show that nobody counts the distance across that boundary: a slot that consists
        // of matrix instructions only was read too early.  So every slot pays the distance itself.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 7\n\ts_nop 3");
        __builtin_amdgcn_sched_barrier(0);
      }
      return sum[0] + sum[1];
    };
    typedef std::true_type Yes;
    typedef std::false_type No;
    // the slot as it stands: is the current pair visible at all, was the previous one, did it need the mask
    auto slot = [&](const f32x16 (&s_exp)[kR], f32x16 (&s_new)[kR], const u16* qt, const bf16x8 (&kf)[kNK], bool vis)
        __attribute__((always_inline)) -> float {
      if (vis) {
        if (!p_vis) return stage(s_exp, s_new, qt, kf, Yes{}, No{}, No{});
        return p_plain ? stage(s_exp, s_new, qt, kf, Yes{}, Yes{}, No{}) : stage(s_exp, s_new, qt, kf, Yes{}, Yes{}, Yes{});
      }
      if (!p_vis) return 0.f;
      return p_plain ? stage(s_exp, s_new, qt, kf, No{}, Yes{}, No{}) : stage(s_exp, s_new, qt, kf, No{}, Yes{}, Yes{});
    };
    auto store_block = [&](int kbi, float mine) __attribute__((always_inline)) {
      const float tot = sum_with_other_half(mine);       // lanes l and l + 32 hold the two halves of the rows
      const int kv = kbi * 32 + l32;
      if (g == 0 && kv < n_cand) part[kv] = tot;
    };

    f32x16 sa[kR], sb[kR];
#pragma unroll
    for (int t = 0; t < kR; ++t) { sa[t] = zero; sb[t] = zero; }
    float carry = 0.f;             // sums of the block before the current one, its last slot still to come
    int carry_kb = -1;
    // all row tiles against one key block; the next block of this wave is fetched meanwhile
    auto do_block = [&](const bf16x8 (&kf)[kNK], int kbi) __attribute__((always_inline)) {
      const int kb0 = kbi * 32;
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < kSlots; ++i) {
        // the slot's rows: row0 .. row0 + 32 kR - 1 (row tiles kR i .. kR i + kR - 1 are neighbours)
        const int tile = kR * i;
        const int row0 = first_row_of(tile / QT) + 32 * (tile % QT);
        // some row of the slot sees some key of the block; every row sees every key and all are real
        const bool vis = row0 < n && (kb0 < c || kb0 - c <= row0 + 32 * kR - 1 + shift);
        const bool plain = kb0 + 31 < n_cand && (kb0 + 31 < c || kb0 + 31 - c <= row0 + shift) && row0 + 32 * kR <= n;
        const float got = (i & 1) ? slot(sa, sb, q_lds + tile * 32 * D, kf, vis) : slot(sb, sa, q_lds + tile * 32 * D, kf, vis);
        if (i == 0) {
          if (carry_kb >= 0) store_block(carry_kb, carry + got);   // the last slot of the block before
        } else {
          acc += got;
        }
        p_vis = vis; p_plain = plain; p_kb0 = kb0; p_row0 = row0; p_tile = tile;
      }
      carry = acc;
      carry_kb = kbi;
    };
    // This wave's key blocks are wave, wave + kWaves, ...; two register sets take turns, the block
    // after the current one is on its way while the current one is worked on (a third set, two
    // blocks ahead, was tried: it spills and is slower).  The fetches are unconditional (past the
    // wave's last block they read it again): the compiler counts the loads in flight to place its
    // waits, and a fetch that may or may not have been issued would make it wait for the newest one.
    bf16x8 kfa[kNK], kfb[kNK];
    const int last_kb = max(n_kb - 1, 0);
    load_keys(kfa, min(wave_s, last_kb));
    __syncthreads();               // the query rows are in LDS
    for (int kbi = wave_s; kbi < n_kb; kbi += 2 * S::kWaves) {
      load_keys(kfb, min(kbi + S::kWaves, last_kb));
      do_block(kfa, kbi);
      load_keys(kfa, min(kbi + 2 * S::kWaves, last_kb));
      if (kbi + S::kWaves < n_kb) do_block(kfb, kbi + S::kWaves);
    }
    if (carry_kb >= 0) {
      // the last slot of the last block: its logits are in the second accumulator set
      const float got = slot(sb, sa, q_lds, kfa, false);
      store_block(carry_kb, carry + got);
    }
    // keys that none of this workgroup's rows see: zeros (the selection adds every partial array)
    for (int kv = n_kb * 32 + tid; kv < n_cand; kv += kThreads) part[kv] = 0.f;
  }
}

template <int D, int QT, int QW, int KS>
hipError_t launch_shape(const AttnArgs& a, hipStream_t s) {
  using S = Shape<D, QT, QW, KS>;
  const int grid = kXcds * a.work_per_xcd;
  hipLaunchKernelGGL((attention_kernel<D, QT, QW, KS>), dim3(grid), dim3(S::kThreads), S::kLdsBytes, s, a);
  return hipGetLastError();
}

template <int D, int QT, int QW, int KS>
hipError_t prepare_shape() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(attention_kernel<D, QT, QW, KS>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, Shape<D, QT, QW, KS>::kLdsBytes);
}

}  // namespace

// Every shape needs more dynamic LDS than a kernel gets by default.  The attribute belongs to the
// function on the current device, so this runs once per cache creation, on the cache's device.
hipError_t prepare_attention() {
  hipError_t e;
  if ((e = prepare_shape<128, 2, 2, 2>()) != hipSuccess) return e;
  if ((e = prepare_shape<128, 1, 4, 2>()) != hipSuccess) return e;
  if ((e = prepare_shape<128, 1, 2, 2>()) != hipSuccess) return e;
  if ((e = prepare_shape<64, 2, 2, 2>()) != hipSuccess) return e;
  if ((e = prepare_shape<64, 1, 4, 2>()) != hipSuccess) return e;
  return prepare_shape<64, 1, 2, 2>();
}

hipError_t launch_attention(const AttnArgs& a, int head_dim, hipStream_t s) {
  if (head_dim == 128) {
    if (a.variant == 0) return launch_shape<128, 2, 2, 2>(a, s);
    if (a.variant == 2) return launch_shape<128, 1, 4, 2>(a, s);
    return launch_shape<128, 1, 2, 2>(a, s);
  }
  if (a.variant == 0) return launch_shape<64, 2, 2, 2>(a, s);
  if (a.variant == 2) return launch_shape<64, 1, 4, 2>(a, s);
  return launch_shape<64, 1, 2, 2>(a, s);
}

}  // namespace kvp

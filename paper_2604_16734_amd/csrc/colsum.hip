// Importance of every candidate key (Eq. 4 of the paper summed over the
// observation queries): score_j = sum over rows r and over the query heads of
// the KV group of softmax(S)[r, j].
//
// A column sum mixes rows whose softmax normalisers are only known once the
// row has seen its last key, so it cannot ride along with the online softmax
// of the attention kernel.  This kernel takes the finished row statistics
// (log2-domain log-sum-exp) and sweeps S a second time with the roles of the
// operands exchanged: a wave keeps its keys in registers as the B operand for
// the whole kernel and streams 32-row query tiles through LDS as the A
// operand, for every query head of the KV group in turn.  In the accumulator
// layout a lane then holds one key column, so the column sum is a plain
// per-lane running add and nothing is reduced across lanes until the very end.
// No atomics: every row split writes its own partial array and the select
// kernel adds them in a fixed order.
//
// Inside a wave the work is software-pipelined: the MFMAs of query tile i run
// while the exponentials of tile i - 1 are taken, from a second set of
// accumulators, with the instruction mix laid out by sched_group_barrier (a
// wave that first issues all MFMAs and then all exponentials leaves each pipe
// idle half of the time, and two such waves on one SIMD fall into step rather
// than filling each other's gaps).
//
// Query tiles go from global memory straight into a ring of LDS buffers
// (global_load_lds, 16-byte chunks XOR-swizzled by row so that the fragment
// reads are conflict-free), a pair of tiles at a time while the pair before it is
// in use; the loads are issued as inline assembly and waited for by hand, one
// barrier per pair.
//
// Work split: a workgroup owns one block of keys of one KV head and a range of
// query tiles.  Key blocks that lie in the new part of the candidates are seen
// by fewer rows (causal mask), so they get fewer row splits: every workgroup
// has about the same number of tiles and the whole launch is one round of two
// four-wave workgroups per CU (their barriers are independent, so one fills the
// gaps the other leaves around its barrier).
#include <type_traits>

#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kRing = 4;               // LDS query-tile buffers: the pair of tiles in use and the pair in flight
constexpr int kStatRing = 8;           // row statistics stay one step longer than their tile: a longer ring

// W waves per workgroup, NT 32-key subtiles per wave: a wave owns 32 NT keys, a workgroup 32 NT W
template <int D, int NT, int W>
__global__ void __launch_bounds__(64 * W, 8 / W)
colsum_kernel(const ColsumArgs a) {
  constexpr int kChunks = D / 8;                   // 16-byte chunks per query row
  constexpr int kTile = 32 * D;                    // bf16 elements of a query tile
  constexpr int kRowsPerInstr = 64 / kChunks;      // rows one 1 KiB load instruction brings in
  constexpr int kInstrPerTile = 32 / kRowsPerInstr;
  constexpr int kQLoads = kInstrPerTile > W ? kInstrPerTile / W : 1;   // 1 KiB pieces per wave and tile
  constexpr int kWaveKeys = 32 * NT;
  constexpr int kBlockKeys = W * kWaveKeys;
  constexpr int kMfmas = NT * (D / 16);            // per wave and tile
  __shared__ __align__(1024) u16 q_lds[kRing][kTile];
  __shared__ __align__(256) float lse_lds[kStatRing][64];

  const int xcd = blockIdx.x % kXcds;
  const int w = xcd * a.work_per_xcd + blockIdx.x / kXcds;
  if (w >= a.total_work) return;
  // grid y: the layer of the group
  const int li = blockIdx.y;
  const u16* const q_rows = a.q_layer[li];
  const u16* const k_new = a.g.k_new[li];
  const u16* const k_cache = a.k_cache + (long long)li * a.g.kv_stride;
  const float* const lse2 = in_set_of(a.lse2, a.g, li);
  float* const partial = in_set_of(a.partial, a.g, li);
  const int hk = w / a.wgs_per_head;
  const int rem = w % a.wgs_per_head;
  int kvb = 0;
  while (a.split_prefix[kvb + 1] <= rem) ++kvb;
  const int split = rem - a.split_prefix[kvb];
  const int splits = a.split_prefix[kvb + 1] - a.split_prefix[kvb];
  const int group = a.n_q_heads / a.n_kv_heads;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: branches on it are scalar
  const int l32 = lane & 31, g = lane >> 5;
  const int n = a.n, c = a.c, n_cand = c + a.n_keys, shift = a.shift;
  const int blk0 = kvb * kBlockKeys;
  const int key0 = blk0 + wave * kWaveKeys;       // first key of this wave

  // rows before the block's first key see none of its keys; the tiles from there on are
  // divided evenly among the block's row splits
  const int n_qt = (n + 31) / 32;
  const int first_tile = blk0 - c > shift ? (blk0 - c - shift) / 32 : 0;
  const int visible = n_qt - first_tile;
  const int qt_begin = first_tile + (split * visible) / splits;
  const int qt_end = first_tile + ((split + 1) * visible) / splits;
  const int tiles = qt_end - qt_begin;
  const int n_steps = tiles * group;              // step i: head i / tiles, tile qt_begin + i % tiles

  // ---- staging of query tiles: piece p = wave + W j of a tile is rows kRowsPerInstr p + ld_sub;
  // surplus waves repeat a piece (same data, same place) so that every wave has the same number
  // of loads in flight.  The steps are issued in order; (iq_head, iq_tile) is the next one.
  const int ld_sub = lane / kChunks, ld_pos = lane % kChunks;
  int iq_head = 0, iq_tile = 0, iq_buf = 0, iq_stat = 0;
  auto issue_step = [&]() __attribute__((always_inline)) {
    const int h = hk * group + iq_head;
    const int qt = qt_begin + iq_tile;
#pragma unroll
    for (int j = 0; j < kQLoads; ++j) {
      const int piece = (wave + W * j) % kInstrPerTile;
      const int ld_row = kRowsPerInstr * piece + ld_sub;
      const int ld_chunk = ld_pos ^ (ld_row % kChunks);
      const int row = min(qt * 32 + ld_row, n - 1);
      const u16* src = q_rows + ((size_t)row * a.n_q_heads + h) * D + 8 * ld_chunk;
      const unsigned dst = __builtin_amdgcn_readfirstlane(
          (unsigned)(size_t)(__attribute__((address_space(3))) void*)(&q_lds[iq_buf][kRowsPerInstr * piece * D]));
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst) : "m0", "memory");
    }
    {
      const int row = min(qt * 32 + l32, n - 1);
      const float* src = lse2 + (size_t)h * a.lse_stride + row;
      const unsigned dst = __builtin_amdgcn_readfirstlane(
          (unsigned)(size_t)(__attribute__((address_space(3))) void*)(&lse_lds[iq_stat][0]));
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(dst) : "m0", "memory");
    }
    // steps past the end fetch the last one again: the count of loads in flight stays the same
    iq_buf = iq_buf + 1 == kRing ? 0 : iq_buf + 1;
    iq_stat = iq_stat + 1 == kStatRing ? 0 : iq_stat + 1;
    if (iq_tile + 1 < tiles) ++iq_tile;
    else if (iq_head + 1 < group) { ++iq_head; iq_tile = 0; }
  };
  if (n_steps > 0) {
    issue_step();
    issue_step();
  }

  // ---- this wave's keys: B operand, lane holds K[key0 + 32 t + l32][16 s + 8 g .. + 7]
  bf16x8 kf[NT][D / 16];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int kv = min(key0 + 32 * t + l32, n_cand - 1);     // columns past the end are not stored
    const u16* src = kv < c ? k_cache + ((size_t)hk * a.budget + kv) * D
                            : k_new + ((size_t)(kv - c) * a.n_kv_heads + hk) * D;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      kf[t][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * s + 8 * g));
  }
  // Make the compiler finish these loads here (and with them the first tiles, which are older).
  // Left pending, it would wait for them inside the loop, where the hand-issued tile loads are in
  // flight, and drain those as well.
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int s = 0; s < D / 16; ++s) asm volatile("" ::"v"(kf[t][s]));

  // A operand: row l32, chunk (2 st + g) ^ (l32 % kChunks) of the tile
  int q_off[D / 16];
  {
    const int q = g ^ (l32 % kChunks);
#pragma unroll
    for (int st = 0; st < D / 16; ++st) q_off[st] = l32 * D + 8 * ((2 * st) ^ q);
  }

  // two running sums per key column, so that consecutive adds do not wait for each other
  float colacc[NT][2];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int k = 0; k < 2; ++k) colacc[t][k] = 0.f;
  const float sl2 = a.scale_log2;
  // the same value behind an opaque copy: the masked and the plain branch of a stage then have no
  // common subexpressions for the compiler to hoist above the branch, out of the MFMAs' shadow
  float sl2_masked;
  asm volatile("v_mov_b32 %0, %1" : "=v"(sl2_masked) : "s"(sl2));

  // Tiles are published in pairs, one barrier for two stages: the pair has landed for this wave
  // when none of its loads remain ... and for everybody after the barrier; everybody has also
  // read the pair before by then, so its buffers take the next pair.  A bare s_barrier on
  // purpose: __syncthreads() carries a fence the compiler places waits around.
  auto publish = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    issue_step();
    issue_step();
  };
  // S of the tile in ring buffer BUF for this wave's keys
  auto logits = [&](auto buf_c, f32x16 (&s)[NT]) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buf_c)::value;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const bf16x8 qa = *reinterpret_cast<const bf16x8*>(&q_lds[BUF][q_off[st]]);
#pragma unroll
      for (int t = 0; t < NT; ++t)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[t][st], st == 0 ? zero : s[t], 0, 0, 0);
    }
  };
  // the row statistics of a tile (accumulator register r of lane group g is row 8 (r / 4) + 4 g + r % 4)
  auto statistics = [&](int slot, float (&ls)[16]) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(&lse_lds[slot][8 * j + 4 * g]);
      ls[4 * j] = v[0]; ls[4 * j + 1] = v[1]; ls[4 * j + 2] = v[2]; ls[4 * j + 3] = v[3];
    }
  };
  // how a tile stands to this wave's keys: every key visible to every row and the tile full
  // (plain), no key visible to any row (nothing to add), or the causal boundary or the end of
  // the block runs through it (masked)
  auto is_plain = [&](int row0) {
    return (key0 + kWaveKeys - 1 < c || key0 + kWaveKeys - 1 - c <= row0 + shift) && row0 + 32 <= n;
  };
  auto is_hidden = [&](int row0) { return key0 - c > row0 + 31 + shift; };
  auto sum_plain = [&](const f32x16 (&s)[NT], const float (&ls)[16]) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        colacc[t][r & 1] += __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2, -ls[r]));
  };
  auto sum_masked = [&](int row0, const f32x16 (&s)[NT], const float (&ls)[16]) __attribute__((always_inline)) {
    // row row0 + 4 g + off, off = 8 (r / 4) + r % 4, counts for key kv when kv - c - shift <= row < n:
    // first <= off < rows_left, one unsigned comparison (first < rows_left for every real key)
    const int rows_left = n - row0 - 4 * g;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int first = key0 + 32 * t + l32 - c - shift - row0 - 4 * g;      // negative for a cached key
      const unsigned span = (unsigned)(rows_left - first);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int off = 8 * (r >> 2) + (r & 3);
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2_masked, -ls[r]));
        colacc[t][r & 1] += (unsigned)(off - first) < span ? p : 0.f;
      }
    }
  };
  // one pipeline stage: MFMAs of the tile in buffer BUF into `sn` among the exponentials of the
  // tile before it (first row `row0`, statistics in `slot`) from `sp`
  auto stage = [&](auto buf_c, int row0, int slot, const f32x16 (&sp)[NT], f32x16 (&sn)[NT])
      __attribute__((always_inline)) {
    if (decltype(buf_c)::value % 2 == 0) publish();
    constexpr int kElemsPerMfma = 16 * NT / kMfmas;       // 2 (D = 128) or 4 (D = 64)
    constexpr int kFragsAhead = 4;                         // operand fragments read before the first MFMA
    float ls[16];
    if (is_plain(row0)) {
      statistics(slot, ls);
      logits(buf_c, sn);
      sum_plain(sp, ls);
      __builtin_amdgcn_sched_group_barrier(0x100, 4 + kFragsAhead, 0);
      // the reads take a while to come back: start on the exponentials meanwhile
      __builtin_amdgcn_sched_group_barrier(0x002, 2 * kElemsPerMfma, 0);
      __builtin_amdgcn_sched_group_barrier(0x400, 2 * kElemsPerMfma, 0);
#pragma unroll
      for (int m = 0; m < kMfmas; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (m % NT == 0 && m / NT + kFragsAhead < D / 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 2 * kElemsPerMfma, 0);   // fma and add per element
        __builtin_amdgcn_sched_group_barrier(0x400, kElemsPerMfma, 0);
      }
    } else if (is_hidden(row0)) {
      logits(buf_c, sn);
    } else {
      statistics(slot, ls);
      logits(buf_c, sn);
      sum_masked(row0, sp, ls);
      __builtin_amdgcn_sched_group_barrier(0x100, 4 + kFragsAhead, 0);
#pragma unroll
      for (int m = 0; m < kMfmas; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (m % NT == 0 && m / NT + kFragsAhead < D / 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 5 * kElemsPerMfma, 0);
        __builtin_amdgcn_sched_group_barrier(0x400, kElemsPerMfma, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto drain = [&](int row0, int slot, const f32x16 (&s)[NT]) __attribute__((always_inline)) {
    float ls[16];
    if (is_plain(row0)) { statistics(slot, ls); sum_plain(s, ls); }
    else if (!is_hidden(row0)) { statistics(slot, ls); sum_masked(row0, s, ls); }
  };

  if (n_steps > 0) {
    f32x16 sa[NT], sb[NT];
    publish();
    logits(std::integral_constant<int, 0>{}, sa);
    __builtin_amdgcn_sched_barrier(0);
    // step i is head i / tiles, tile qt_begin + i % tiles, in ring buffer i % kRing (a constant
    // in each of the four copies of the stage); `prev_tile` and `prev_slot` are the tile whose
    // sums are due and the place of its statistics
    static_assert(kRing == 4, "the loop below is unrolled over the ring");
    int prev_tile = 0, prev_slot = 0, i = 1;
    auto row0_prev = [&]() { return (qt_begin + prev_tile) * 32; };
    auto advance = [&]() {
      prev_tile = prev_tile + 1 == tiles ? 0 : prev_tile + 1;
      prev_slot = prev_slot + 1 == kStatRing ? 0 : prev_slot + 1;
      ++i;
    };
    for (;;) {
      if (i >= n_steps) { drain(row0_prev(), prev_slot, sa); break; }
      stage(std::integral_constant<int, 1>{}, row0_prev(), prev_slot, sa, sb);
      advance();
      if (i >= n_steps) { drain(row0_prev(), prev_slot, sb); break; }
      stage(std::integral_constant<int, 2>{}, row0_prev(), prev_slot, sb, sa);
      advance();
      if (i >= n_steps) { drain(row0_prev(), prev_slot, sa); break; }
      stage(std::integral_constant<int, 3>{}, row0_prev(), prev_slot, sa, sb);
      advance();
      if (i >= n_steps) { drain(row0_prev(), prev_slot, sb); break; }
      stage(std::integral_constant<int, 0>{}, row0_prev(), prev_slot, sb, sa);
      advance();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the surplus loads must not outlive the workgroup's LDS
  }

  // lanes l and l + 32 hold the two halves of the rows of one key column
  float* dstp = partial + ((size_t)hk * a.n_partials + split) * a.cand_stride;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const float mine = colacc[t][0] + colacc[t][1];
    const float tot = mine + __shfl_xor(mine, 32, 64);
    const int kv = key0 + 32 * t + l32;
    if (g == 0 && kv < n_cand) dstp[kv] = tot;
  }
  // a key block with fewer row splits than the launch's partial count leaves the rest at zero
  if (split == 0) {
    for (int p = splits + g; p < a.n_partials; p += 2) {
      float* z = partial + ((size_t)hk * a.n_partials + p) * a.cand_stride;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int kv = key0 + 32 * t + l32;
        if (kv < n_cand) z[kv] = 0.f;
      }
    }
  }
}

}  // namespace

hipError_t launch_colsum(const ColsumArgs& a, int head_dim, hipStream_t s) {
  if (a.g.n_layers < 1 || a.g.n_layers > kMaxGroupLayers) return hipErrorInvalidValue;
  const int grid = kXcds * a.work_per_xcd;
  const dim3 g(grid, a.g.n_layers), b(64 * kColsumWaves);
  if (head_dim == 128) {
    if (a.subtiles == 2) hipLaunchKernelGGL((colsum_kernel<128, 2, kColsumWaves>), g, b, 0, s, a);
    else hipLaunchKernelGGL((colsum_kernel<128, 1, kColsumWaves>), g, b, 0, s, a);
  } else {
    if (a.subtiles == 2) hipLaunchKernelGGL((colsum_kernel<64, 2, kColsumWaves>), g, b, 0, s, a);
    else hipLaunchKernelGGL((colsum_kernel<64, 1, kColsumWaves>), g, b, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace kvp

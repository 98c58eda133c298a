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
// Query tiles go from global memory straight into a ring of LDS buffers
// (global_load_lds, 16-byte chunks XOR-swizzled by row so that the fragment
// reads are conflict-free), three tiles ahead of their use; the loads are
// issued as inline assembly and ordered by hand (a counted s_waitcnt before the
// barrier that publishes a tile) so that later tiles stay in flight.
#include <type_traits>

#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kRing = 4;               // LDS query-tile buffers
constexpr int kAhead = 3;              // tiles in flight ahead of the one in use
constexpr int kMaxRowSplits = 16;
constexpr int kTargetWorkgroups = 768;    // three per CU: two resident, startup of the third hidden

// NT = 32-key subtiles per wave: a wave owns 32 NT keys, a workgroup 128 NT
template <int D, int NT>
__global__ void __launch_bounds__(kThreads, 2)
colsum_kernel(const ColsumArgs a) {
  constexpr int kChunks = D / 8;                  // 16-byte chunks per query row
  constexpr int kTile = 32 * D;                   // bf16 elements of a query tile
  constexpr int kQLoads = (32 * kChunks) / 256;   // 1 KiB instructions per wave and tile
  constexpr int kLoadsPerStep = kQLoads + 1;      // plus the row statistics
  constexpr int kWaveKeys = 32 * NT;
  constexpr int kBlockKeys = 4 * kWaveKeys;
  __shared__ __align__(1024) u16 q_lds[kRing][kTile];
  __shared__ __align__(256) float lse_lds[kRing][64];

  const int xcd = blockIdx.x % kXcds;
  const int w = xcd * a.work_per_xcd + blockIdx.x / kXcds;
  if (w >= a.total_work) return;
  const int split = w % a.row_splits;
  const int kvb = (w / a.row_splits) % a.n_kv_blocks;
  const int hk = w / (a.row_splits * a.n_kv_blocks);
  const int group = a.n_q_heads / a.n_kv_heads;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int n = a.n, c = a.c, n_cand = c + n;
  const int blk0 = kvb * kBlockKeys;
  const int key0 = blk0 + wave * kWaveKeys;       // first key of this wave

  // ---- this wave's keys: B operand, lane holds K[key0 + 32 t + l32][16 s + 8 g .. + 7]
  bf16x8 kf[NT][D / 16];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int kv = min(key0 + 32 * t + l32, n_cand - 1);     // columns past the end are not stored
    const u16* src = kv < c ? a.k_cache + ((size_t)hk * a.budget + kv) * D
                            : a.k_new + ((size_t)(kv - c) * a.n_kv_heads + hk) * D;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      kf[t][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * s + 8 * g));
  }
  // Make the compiler finish these loads here.  Left pending, it would wait for them inside the
  // loop, at a point where the hand-issued tile loads are in flight, and drain those as well.
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int s = 0; s < D / 16; ++s) asm volatile("" ::"v"(kf[t][s]));

  // rows [qt_begin, qt_end) in units of 32-row tiles; rows before the block's first key see none
  // of its block keys, so a block past the cache starts later
  const int n_qt = (n + 31) / 32;
  int qt_begin = split * a.q_tiles_per_split;
  const int qt_end = min(n_qt, qt_begin + a.q_tiles_per_split);
  if (blk0 >= c) qt_begin = max(qt_begin, (blk0 - c) / 32);
  const int tiles = max(qt_end - qt_begin, 0);
  const int n_steps = tiles * group;              // step i: head i / tiles, tile qt_begin + i % tiles

  // ---- staging of query tiles
  const int ld_sub = lane / kChunks, ld_pos = lane % kChunks;
  const int ld_chunk = ld_pos ^ (ld_sub + (64 / kChunks) * (wave % (kChunks * kChunks / 64)));
  auto issue_step = [&](int i) __attribute__((always_inline)) {
    // steps past the end fetch the last one again: the count of loads in flight stays the same
    const int ii = min(i, n_steps - 1);
    const int h = hk * group + ii / tiles;
    const int qt = qt_begin + ii % tiles;
    const int buf = i % kRing;
#pragma unroll
    for (int j = 0; j < kQLoads; ++j) {
      // instruction (wave + 4 j) brings in rows (64 / kChunks) (wave + 4 j) + ld_sub of the tile
      const int r_in_tile = (64 / kChunks) * (wave + 4 * j) + ld_sub;
      const int row = min(qt * 32 + r_in_tile, n - 1);
      const u16* src = a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * ld_chunk;
      const unsigned dst = __builtin_amdgcn_readfirstlane(
          (unsigned)(size_t)(__attribute__((address_space(3))) void*)(&q_lds[buf][(64 / kChunks) * (wave + 4 * j) * D]));
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst) : "m0", "memory");
    }
    {
      // every wave fetches the same 64 statistics: same data to the same place, so that all waves
      // have the same number of loads in flight
      const int row = min(qt * 32 + (lane & 31), n - 1);
      const float* src = a.lse2 + (size_t)h * a.lse_stride + row;
      const unsigned dst = __builtin_amdgcn_readfirstlane(
          (unsigned)(size_t)(__attribute__((address_space(3))) void*)(&lse_lds[buf][0]));
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(dst) : "m0", "memory");
    }
  };

  // A operand offsets: row l32, chunk (2 st + g) ^ (l32 % kChunks)
  int q_off[D / 16];
  {
    const int q = g ^ (l32 % kChunks);
#pragma unroll
    for (int st = 0; st < D / 16; ++st) q_off[st] = l32 * D + 8 * ((2 * st) ^ q);
  }

  float colacc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) colacc[t] = 0.f;
  const float sl2 = a.scale_log2;

  if (n_steps > 0) {
#pragma unroll
    for (int i = 0; i < kAhead; ++i) issue_step(i);
    for (int i = 0; i < n_steps; ++i) {
      // tile i has landed for this wave when at most the loads of the (kAhead - 1) later tiles remain
      // ... and for everybody after the barrier; everybody is also done with tile i - 1 then.
      // A bare s_barrier on purpose: __syncthreads() carries a fence that drains ALL loads in
      // flight, which would throw the prefetch ring away at every step.
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((kAhead - 1) * kLoadsPerStep) : "memory");
      issue_step(i + kAhead);          // into the buffer of tile i - 1
      const int buf = i % kRing;
      const int row0 = (qt_begin + i % tiles) * 32;

      f32x16 s[NT];
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < D / 16; ++st) {
        const bf16x8 qa = *reinterpret_cast<const bf16x8*>(&q_lds[buf][q_off[st]]);
#pragma unroll
        for (int t = 0; t < NT; ++t)
          s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[t][st], st == 0 ? zero : s[t], 0, 0, 0);
      }
      // accumulator register r of lane group g is row 8 (r / 4) + 4 g + r % 4
      float nl[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float4 v = *reinterpret_cast<const float4*>(&lse_lds[buf][8 * j + 4 * g]);
        nl[4 * j] = -v.x; nl[4 * j + 1] = -v.y; nl[4 * j + 2] = -v.z; nl[4 * j + 3] = -v.w;
      }
      // plain step: every key of the wave is visible to every row of the tile, and the tile is full
      const bool plain = (key0 + kWaveKeys - 1 < c || key0 + kWaveKeys - 1 - c <= row0) && row0 + 32 <= n;
      if (plain) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float sum = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2, nl[r]));
          colacc[t] += sum;
        }
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int kv = key0 + 32 * t + l32;
          float sum = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qr = row0 + 8 * (r >> 2) + 4 * g + (r & 3);
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2, nl[r]));
            sum += (qr < n && (kv < c || kv - c <= qr)) ? p : 0.f;
          }
          colacc[t] += sum;
        }
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the surplus loads must not outlive the workgroup's LDS
  }

  // lanes l and l + 32 hold the two halves of the rows of one key column
  float* dstp = a.partial + ((size_t)hk * a.n_partials + split) * a.cand_stride;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const float tot = colacc[t] + __shfl_xor(colacc[t], 32, 64);
    const int kv = key0 + 32 * t + l32;
    if (g == 0 && kv < n_cand) dstp[kv] = tot;
  }
}

}  // namespace

int colsum_max_partials(int /*group*/, int /*chunk_max*/) { return kMaxRowSplits; }

void plan_colsum(ColsumArgs& a, int /*head_dim*/) {
  const int n_cand = a.c + a.n;
  const int n_qt = (a.n + 31) / 32;
  // keys per workgroup: 512, or 256 / 128 when that is what it takes to fill the chip
  int nt = 4;
  while (nt > 1 && a.n_kv_heads * ((n_cand + 128 * nt - 1) / (128 * nt)) * kMaxRowSplits < 256) nt >>= 1;
  a.subtiles = nt;
  const int block_keys = 128 * nt;
  a.n_kv_blocks = (n_cand + block_keys - 1) / block_keys;
  const int base = a.n_kv_heads * a.n_kv_blocks;
  int rs = (kTargetWorkgroups + base - 1) / base;
  rs = rs < 1 ? 1 : rs;
  rs = rs > kMaxRowSplits ? kMaxRowSplits : rs;
  rs = rs > n_qt ? n_qt : rs;
  a.q_tiles_per_split = (n_qt + rs - 1) / rs;
  a.row_splits = (n_qt + a.q_tiles_per_split - 1) / a.q_tiles_per_split;
  a.n_partials = a.row_splits;
  a.total_work = base * a.row_splits;
  a.work_per_xcd = (a.total_work + kXcds - 1) / kXcds;
}

hipError_t launch_colsum(const ColsumArgs& a, int head_dim, hipStream_t s) {
  const int grid = kXcds * a.work_per_xcd;
  const dim3 g(grid), b(kThreads);
  if (head_dim == 128) {
    if (a.subtiles == 4) hipLaunchKernelGGL((colsum_kernel<128, 4>), g, b, 0, s, a);
    else if (a.subtiles == 2) hipLaunchKernelGGL((colsum_kernel<128, 2>), g, b, 0, s, a);
    else hipLaunchKernelGGL((colsum_kernel<128, 1>), g, b, 0, s, a);
  } else {
    if (a.subtiles == 4) hipLaunchKernelGGL((colsum_kernel<64, 4>), g, b, 0, s, a);
    else if (a.subtiles == 2) hipLaunchKernelGGL((colsum_kernel<64, 2>), g, b, 0, s, a);
    else hipLaunchKernelGGL((colsum_kernel<64, 1>), g, b, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace kvp

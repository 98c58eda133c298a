// Importance of every candidate key (Eq. 4 of the paper summed over the
// observation queries): score_j = sum over rows r and over the query heads of
// the KV group of softmax(S)[r, j].
//
// A column sum mixes rows whose softmax normalisers are only known once the
// row has seen its last key, so it cannot ride along with the online softmax
// of the attention kernel.  This kernel takes the finished row statistics
// (log2-domain log-sum-exp) and sweeps S a second time with the roles of the
// operands exchanged: a wave keeps its 128 keys in registers as the B operand
// for the whole kernel and streams 32-row query tiles through LDS as the A
// operand.  In the accumulator layout a lane then holds one key column, so the
// column sum is a plain per-lane running add and nothing is reduced across
// lanes until the very end.  No atomics: every (query head, row split) writes
// its own partial array and the select kernel adds them in a fixed order.
#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;
constexpr int kNt = 4;                 // 32-key subtiles per wave
constexpr int kWaveKeys = 32 * kNt;    // 128
constexpr int kBlockKeys = 4 * kWaveKeys;
constexpr int kMaxRowSplits = 8;
constexpr int kTargetWorkgroups = 512;

template <int D>
__global__ void __launch_bounds__(kThreads, 2)
colsum_kernel(const ColsumArgs a) {
  constexpr int kQStride = D + 8;
  constexpr int kQTile = 32 * kQStride;        // bf16 elements
  __shared__ __align__(16) u16 q_lds[2][kQTile];
  __shared__ __align__(16) float lse_lds[2][32];

  const int xcd = blockIdx.x % kXcds;
  const int w = xcd * a.work_per_xcd + blockIdx.x / kXcds;
  if (w >= a.total_work) return;
  const int split = w % a.row_splits;
  const int kvb = (w / a.row_splits) % a.n_kv_blocks;
  const int h = w / (a.row_splits * a.n_kv_blocks);
  const int group = a.n_q_heads / a.n_kv_heads;
  const int hk = h / group;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int n = a.n, c = a.c, n_cand = c + n;
  const int key0 = kvb * kBlockKeys + wave * kWaveKeys;   // first key of this wave

  // ---- this wave's keys: B operand, lane holds K[key0 + 32 t + l32][16 s + 8 g .. + 7]
  bf16x8 kf[kNt][D / 16];
#pragma unroll
  for (int t = 0; t < kNt; ++t) {
    const int kv = key0 + 32 * t + l32;
    const u16* src = nullptr;
    if (kv < c) src = a.k_cache + ((size_t)hk * a.budget + kv) * D;
    else if (kv < n_cand) src = a.k_new + ((size_t)(kv - c) * a.n_kv_heads + hk) * D;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      uint4 x = make_uint4(0, 0, 0, 0);
      if (src) x = *reinterpret_cast<const uint4*>(src + 16 * s + 8 * g);
      kf[t][s] = __builtin_bit_cast(bf16x8, x);
    }
  }

  // rows [qt_begin, qt_end) in units of 32-row tiles; rows before the block's
  // first key see none of its block keys, so a block past the cache starts later
  const int n_qt = (n + 31) / 32;
  int qt_begin = split * a.q_tiles_per_split;
  const int qt_end = min(n_qt, qt_begin + a.q_tiles_per_split);
  const int blk0 = kvb * kBlockKeys;
  if (blk0 >= c) qt_begin = max(qt_begin, (blk0 - c) / 32);

  float colacc[kNt];
#pragma unroll
  for (int t = 0; t < kNt; ++t) colacc[t] = 0.f;

  constexpr int kPieces = 32 * (D / 8);
  constexpr int kPer = (kPieces + kThreads - 1) / kThreads;
  uint4 qreg[kPer];
  float lreg = 0.f;
  auto load_tile = [&](int qt) {
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      const int i = tid + kThreads * j;
      qreg[j] = make_uint4(0, 0, 0, 0);
      if (i < kPieces) {
        const int row = qt * 32 + i / (D / 8), c8 = i % (D / 8);
        if (row < n)
          qreg[j] = *reinterpret_cast<const uint4*>(a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * c8);
      }
    }
    if (tid < 32) {
      const int row = qt * 32 + tid;
      // a padding row gets +inf so that its weights vanish
      lreg = row < n ? a.lse2[(size_t)h * a.lse_stride + row] : INFINITY;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      const int i = tid + kThreads * j;
      if (i < kPieces) {
        const int row = i / (D / 8), c8 = i % (D / 8);
        *reinterpret_cast<uint4*>(&q_lds[buf][row * kQStride + 8 * c8]) = qreg[j];
      }
    }
    if (tid < 32) lse_lds[buf][tid] = lreg;
  };

  const float sl2 = a.scale_log2;
  if (qt_begin < qt_end) {
    load_tile(qt_begin);
    store_tile(0);
    __syncthreads();
    for (int qt = qt_begin; qt < qt_end; ++qt) {
      const int buf = (qt - qt_begin) & 1;
      const bool more = qt + 1 < qt_end;
      if (more) load_tile(qt + 1);

      const int row0 = qt * 32;
      // which of the wave's subtiles can any row of this tile see
      bool act[kNt];
      bool any = false;
#pragma unroll
      for (int t = 0; t < kNt; ++t) {
        const int kb = key0 + 32 * t;
        act[t] = kb < n_cand && (kb < c || kb - c <= row0 + 31);
        any |= act[t];
      }
      if (any) {
        f32x16 s[kNt];
#pragma unroll
        for (int t = 0; t < kNt; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
        const u16* qrow = &q_lds[buf][l32 * kQStride + 8 * g];
#pragma unroll
        for (int st = 0; st < D / 16; ++st) {
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(qrow + 16 * st);
#pragma unroll
          for (int t = 0; t < kNt; ++t)
            if (act[t]) s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[t][st], s[t], 0, 0, 0);
        }
        // accumulator register r of lane group g is row 8 (r / 4) + 4 g + r % 4
        float nl[16];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float4 v = *reinterpret_cast<const float4*>(&lse_lds[buf][8 * j + 4 * g]);
          nl[4 * j] = -v.x; nl[4 * j + 1] = -v.y; nl[4 * j + 2] = -v.z; nl[4 * j + 3] = -v.w;
        }
#pragma unroll
        for (int t = 0; t < kNt; ++t) {
          if (!act[t]) continue;
          const int kv = key0 + 32 * t + l32;
          const int kb = key0 + 32 * t;
          const bool all_visible = kb + 31 < c || kb + 31 - c <= row0;
          float sum = 0.f;
          if (all_visible) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              sum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2, nl[r]));
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int qr = row0 + 8 * (r >> 2) + 4 * g + (r & 3);
              const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2, nl[r]));
              sum += (kv < c || kv - c <= qr) ? p : 0.f;
            }
          }
          colacc[t] += sum;
        }
      }
      if (more) store_tile(buf ^ 1);
      __syncthreads();
    }
  }

  // lanes l and l + 32 hold the two halves of the rows of one key column
  const int part = (h % group) * a.row_splits + split;
  float* dstp = a.partial + ((size_t)hk * a.n_partials + part) * a.cand_stride;
#pragma unroll
  for (int t = 0; t < kNt; ++t) {
    const float tot = colacc[t] + __shfl_xor(colacc[t], 32, 64);
    const int kv = key0 + 32 * t + l32;
    if (g == 0 && kv < n_cand) dstp[kv] = tot;
  }
}

}  // namespace

int colsum_max_partials(int group, int /*chunk_max*/) { return group * kMaxRowSplits; }

void plan_colsum(ColsumArgs& a, int /*head_dim*/) {
  const int n_cand = a.c + a.n;
  a.n_kv_blocks = (n_cand + kBlockKeys - 1) / kBlockKeys;
  const int n_qt = (a.n + 31) / 32;
  const int base = a.n_q_heads * a.n_kv_blocks;
  int rs = (kTargetWorkgroups + base - 1) / base;
  rs = rs < 1 ? 1 : rs;
  rs = rs > kMaxRowSplits ? kMaxRowSplits : rs;
  rs = rs > n_qt ? n_qt : rs;
  a.q_tiles_per_split = (n_qt + rs - 1) / rs;
  a.row_splits = (n_qt + a.q_tiles_per_split - 1) / a.q_tiles_per_split;
  a.n_partials = (a.n_q_heads / a.n_kv_heads) * a.row_splits;
  a.total_work = base * a.row_splits;
  a.work_per_xcd = (a.total_work + kXcds - 1) / kXcds;
}

hipError_t launch_colsum(const ColsumArgs& a, int head_dim, hipStream_t s) {
  const int grid = kXcds * a.work_per_xcd;
  if (head_dim == 128)
    hipLaunchKernelGGL(colsum_kernel<128>, dim3(grid), dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(colsum_kernel<64>, dim3(grid), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace kvp

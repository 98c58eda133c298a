// Attention of one block of queries over cache U block (Eq. 1 of the paper),
// for gfx950: bf16 MFMA 32x32x16, wave64, K and V tiles staged through LDS.
//
// Formulation.  Every wave owns QT tiles of 32 query rows and works on the
// TRANSPOSED problem: S^T = K Q^T (A operand = K tile from LDS, B operand = Q
// held in registers for the whole kernel) and O^T = V^T P^T (A operand = V^T
// from LDS, B operand = P^T).  In the 32x32 accumulator layout a lane holds one
// column, so with the transposed problem a lane holds ONE query row: the
// running maximum, the running sum and the rescale factor of the online
// softmax are one scalar per lane, and the exponentiated S^T accumulators are,
// register for register, the B operand of the second product.  P never touches
// LDS and is never shuffled between lanes.  The price is that V must sit
// transposed in LDS; the transpose happens in registers on the way in.
//
// The contraction index of an MFMA may be permuted freely as long as A and B
// agree.  For O^T the index is the key position: accumulator register r of lane
// (g = lane / 32) holds key  8 (r / 4) + 4 g + r % 4  of the 32-key block, so
// registers 8 m .. 8 m + 7 are fed to MFMA m of the block and V^T is stored in
// LDS with the key order permuted to match (bits 2 and 3 of the key swapped),
// which makes the A operand one 16-byte LDS read.
//
// A workgroup is QW x KS waves: QW groups of query rows times KS-way split of
// every staged key tile (wave ks takes keys [32 ks, 32 ks + 32) of each tile).
// The KS partial results of a row are merged through LDS at the end.  This is
// what keeps all 1024 SIMDs busy when a block has fewer than 1024 wave-sized
// row tiles.
#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(unsigned, b);
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

template <int D, int QT, int QW, int KS>
struct Shape {
  static constexpr int kRows = QW * QT * 32;          // query rows per workgroup
  static constexpr int kTk = KS * 32;                 // keys per staged tile
  static constexpr int kKStride = D + 8;              // bf16 elements per K row in LDS
  static constexpr int kVStride = kTk + 8;            // bf16 elements per V^T row in LDS
  static constexpr int kKTile = kTk * kKStride;       // elements
  static constexpr int kVTile = D * kVStride;
  static constexpr int kTileBytes = 2 * (kKTile + kVTile) * 2;   // two buffers
  static constexpr int kMergeFloats = QT * (D / 32) * 16 * 64 + 2 * QT * 64;  // per wave
  static constexpr int kMergeBytes = (KS - 1) * QW * kMergeFloats * 4;
  static constexpr int kLdsBytes = kTileBytes > kMergeBytes ? kTileBytes : kMergeBytes;
  static constexpr int kKPieces = kTk * (D / 8);      // 16-byte pieces of a K tile
  static constexpr int kKPer = (kKPieces + kThreads - 1) / kThreads;
  static constexpr int kVGroups = (kTk / 4) * (D / 8);  // 4 keys x 8 channels each
  static constexpr int kVPer = (kVGroups + kThreads - 1) / kThreads;
};

template <int D, int QT, int QW, int KS>
__global__ void __launch_bounds__(kThreads)
attention_kernel(const AttnArgs a) {
  using S = Shape<D, QT, QW, KS>;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  u16* lds = reinterpret_cast<u16*>(lds_raw);

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
  const int qw = wave / KS;
  const int ks = wave % KS;
  const int l32 = lane & 31;
  const int g = lane >> 5;

  const int n = a.n, c = a.c;
  const int row0 = rt * S::kRows;                    // first query row of the workgroup
  const int q0 = row0 + qw * QT * 32;                // first query row of this wave
  const int rows_end = min(n, row0 + S::kRows);
  const int kv_end = c + rows_end;                   // keys any row of the workgroup can see
  const int n_iter = (kv_end + S::kTk - 1) / S::kTk;

  const u16* kc = a.k_cache + (size_t)hk * a.budget * D;
  const u16* vc = a.v_cache + (size_t)hk * a.budget * D;
  const u16* kn = a.k_new + (size_t)hk * D;
  const u16* vn = a.v_new + (size_t)hk * D;
  const size_t new_stride = (size_t)a.n_kv_heads * D;

  // ---- Q fragments: B operand, lane holds Q[q0 + 32 t + l32][16 s + 8 g .. + 7]
  bf16x8 qf[QT][D / 16];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int row = q0 + 32 * t + l32;
    const u16* src = a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      uint4 x = make_uint4(0, 0, 0, 0);
      if (row < n) x = *reinterpret_cast<const uint4*>(src + 16 * s);
      qf[t][s] = __builtin_bit_cast(bf16x8, x);
    }
  }

  f32x16 o[QT][D / 32];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[t][dt][r] = 0.f;
  }

  // ---- staging of one key tile: global -> registers -> LDS
  uint4 kreg[S::kKPer];
  uint4 vreg[S::kVPer][4];

  auto row_ptr = [&](int kv, const u16* cache, const u16* fresh) -> const u16* {
    if (kv < c) return cache + (size_t)kv * D;
    if (kv < c + n) return fresh + (size_t)(kv - c) * new_stride;
    return nullptr;
  };
  auto load_tile = [&](int it) {
    const int base = it * S::kTk;
#pragma unroll
    for (int j = 0; j < S::kKPer; ++j) {
      const int i = tid + kThreads * j;
      kreg[j] = make_uint4(0, 0, 0, 0);
      if (i < S::kKPieces) {
        const int row = i / (D / 8), c8 = i % (D / 8);
        const u16* p = row_ptr(base + row, kc, kn);
        if (p) kreg[j] = *reinterpret_cast<const uint4*>(p + 8 * c8);
      }
    }
#pragma unroll
    for (int j = 0; j < S::kVPer; ++j) {
      const int i = tid + kThreads * j;
#pragma unroll
      for (int e = 0; e < 4; ++e) vreg[j][e] = make_uint4(0, 0, 0, 0);
      if (i < S::kVGroups) {
        const int quad = i % (S::kTk / 4), oct = i / (S::kTk / 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const u16* p = row_ptr(base + 4 * quad + e, vc, vn);
          if (p) vreg[j][e] = *reinterpret_cast<const uint4*>(p + 8 * oct);
        }
      }
    }
  };
  auto store_tile = [&](int buf) {
    u16* kt = lds + buf * (S::kKTile + S::kVTile);
    u16* vt = kt + S::kKTile;
#pragma unroll
    for (int j = 0; j < S::kKPer; ++j) {
      const int i = tid + kThreads * j;
      if (i < S::kKPieces) {
        const int row = i / (D / 8), c8 = i % (D / 8);
        *reinterpret_cast<uint4*>(kt + row * S::kKStride + 8 * c8) = kreg[j];
      }
    }
#pragma unroll
    for (int j = 0; j < S::kVPer; ++j) {
      const int i = tid + kThreads * j;
      if (i < S::kVGroups) {
        const int quad = i % (S::kTk / 4), oct = i / (S::kTk / 4);
        const int key = 4 * quad;
        // key order inside a 32-key block: swap bits 2 and 3
        const int pos = (key & ~12) | ((key & 4) << 1) | ((key & 8) >> 1);
        const unsigned* r0 = reinterpret_cast<const unsigned*>(&vreg[j][0]);
        const unsigned* r1 = reinterpret_cast<const unsigned*>(&vreg[j][1]);
        const unsigned* r2 = reinterpret_cast<const unsigned*>(&vreg[j][2]);
        const unsigned* r3 = reinterpret_cast<const unsigned*>(&vreg[j][3]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int wd = e >> 1;
          uint2 col;
          if ((e & 1) == 0) {
            col.x = (r0[wd] & 0xFFFFu) | (r1[wd] << 16);
            col.y = (r2[wd] & 0xFFFFu) | (r3[wd] << 16);
          } else {
            col.x = (r0[wd] >> 16) | (r1[wd] & 0xFFFF0000u);
            col.y = (r2[wd] >> 16) | (r3[wd] & 0xFFFF0000u);
          }
          *reinterpret_cast<uint2*>(vt + (8 * oct + e) * S::kVStride + pos) = col;
        }
      }
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  const float sl2 = a.scale_log2;
  const int q_last = q0 + QT * 32 - 1;

  for (int it = 0; it < n_iter; ++it) {
    const bool more = it + 1 < n_iter;
    if (more) load_tile(it + 1);

    const u16* kt = lds + (it & 1) * (S::kKTile + S::kVTile);
    const u16* vt = kt + S::kKTile;
    const int kb = it * S::kTk + ks * 32;            // first key of this wave's block
    // a block contributes unless every (row, key) pair of it is hidden
    const bool active = kb < c + n && (kb < c || kb - c <= q_last);
    if (active) {
      // ---- S^T = K Q^T
      f32x16 s[QT];
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
      const u16* krow = kt + (ks * 32 + l32) * S::kKStride + 8 * g;
#pragma unroll
      for (int st = 0; st < D / 16; ++st) {
        const bf16x8 ka = *reinterpret_cast<const bf16x8*>(krow + 16 * st);
#pragma unroll
        for (int t = 0; t < QT; ++t)
          s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[t][st], s[t], 0, 0, 0);
      }
      // ---- hide what the row may not see: block keys after the row itself
      const bool all_visible = kb + 31 < c || (kb + 31 - c <= q0 && kb + 31 < c + n);
      if (!all_visible) {
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          const int qrow = q0 + 32 * t + l32;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = kb + 8 * (r >> 2) + 4 * g + (r & 3);
            const bool vis = kv < c || (kv - c <= qrow && kv < c + n);
            if (!vis) s[t][r] = -INFINITY;
          }
        }
      }
      // ---- online softmax, one query row per lane (shared by lanes l and l + 32)
      unsigned pb[QT][8];
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        float mx = s[t][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m_run[t], mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run[t] - m_use) * sl2);
        const float neg = -m_use * sl2;
        float sum = 0.f;
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], sl2, neg));
          sum += p[r];
        }
        l_run[t] = l_run[t] * alpha + sum;
        m_run[t] = m_new;
#pragma unroll
        for (int r = 0; r < 8; ++r) pb[t][r] = pack_bf16(p[2 * r], p[2 * r + 1]);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][dt][r] *= alpha;
      }
      // ---- O^T += V^T P^T
      const u16* vrow = vt + l32 * S::kVStride + ks * 32 + 8 * g;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const bf16x8 va =
              *reinterpret_cast<const bf16x8*>(vrow + dt * 32 * S::kVStride + 16 * mm);
#pragma unroll
          for (int t = 0; t < QT; ++t) {
            uint4 px = make_uint4(pb[t][4 * mm], pb[t][4 * mm + 1], pb[t][4 * mm + 2],
                                  pb[t][4 * mm + 3]);
            o[t][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                va, __builtin_bit_cast(bf16x8, px), o[t][dt], 0, 0, 0);
          }
        }
      }
    }
    if (more) store_tile((it + 1) & 1);
    __syncthreads();
  }

  // lanes l and l + 32 each summed half of the keys of a row
#pragma unroll
  for (int t = 0; t < QT; ++t) l_run[t] += xor32(l_run[t]);

  // ---- merge the KS partial results of every row through LDS
  if (KS > 1) {
    float* mrg = reinterpret_cast<float*>(lds_raw);
    // the loop's last barrier has passed: nobody reads the tiles any more
    if (ks > 0) {
      float* mine = mrg + (size_t)((ks - 1) * QW + qw) * S::kMergeFloats;
#pragma unroll
      for (int t = 0; t < QT; ++t) {
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            mine[((t * (D / 32) + dt) * 16 + r) * 64 + lane] = o[t][dt][r];
        mine[QT * (D / 32) * 16 * 64 + t * 64 + lane] = m_run[t];
        mine[QT * (D / 32) * 16 * 64 + (QT + t) * 64 + lane] = l_run[t];
      }
    }
    __syncthreads();
    if (ks == 0) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        float mt = m_run[t];
        for (int s2 = 1; s2 < KS; ++s2) {
          const float* other = mrg + (size_t)((s2 - 1) * QW + qw) * S::kMergeFloats;
          mt = fmaxf(mt, other[QT * (D / 32) * 16 * 64 + t * 64 + lane]);
        }
        const float m_use = (mt == -INFINITY) ? 0.f : mt;
        const float f0 = __builtin_amdgcn_exp2f((m_run[t] - m_use) * sl2);
        l_run[t] *= f0;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][dt][r] *= f0;
        for (int s2 = 1; s2 < KS; ++s2) {
          const float* other = mrg + (size_t)((s2 - 1) * QW + qw) * S::kMergeFloats;
          const float ms = other[QT * (D / 32) * 16 * 64 + t * 64 + lane];
          const float ls = other[QT * (D / 32) * 16 * 64 + (QT + t) * 64 + lane];
          const float fs = __builtin_amdgcn_exp2f((ms - m_use) * sl2);
          l_run[t] += ls * fs;
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              o[t][dt][r] += fs * other[((t * (D / 32) + dt) * 16 + r) * 64 + lane];
        }
        m_run[t] = mt;
      }
    }
  }

  // ---- normalise and store; lane holds O[row][32 dt + 8 j + 4 g + 0..3]
  if (ks == 0) {
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const int row = q0 + 32 * t + l32;
      if (row < n) {
        const float inv = 1.f / l_run[t];
        u16* dstp = a.out + ((size_t)row * a.n_q_heads + h) * D + 4 * g;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint2 pk;
            pk.x = pack_bf16(o[t][dt][4 * j] * inv, o[t][dt][4 * j + 1] * inv);
            pk.y = pack_bf16(o[t][dt][4 * j + 2] * inv, o[t][dt][4 * j + 3] * inv);
            *reinterpret_cast<uint2*>(dstp + 32 * dt + 8 * j) = pk;
          }
        if (g == 0)
          a.lse2[(size_t)h * a.lse_stride + row] = m_run[t] * sl2 + __builtin_log2f(l_run[t]);
      }
    }
  }
}

template <int D, int QT, int QW, int KS>
hipError_t launch_shape(const AttnArgs& a, hipStream_t s) {
  using S = Shape<D, QT, QW, KS>;
  auto kern = attention_kernel<D, QT, QW, KS>;
  static bool attr_done = false;   // per-process; the attribute is per function
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, S::kLdsBytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int grid = kXcds * a.work_per_xcd;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), S::kLdsBytes, s, a);
  return hipGetLastError();
}

constexpr int kRowsOfVariant[3] = {128, 64, 32};

}  // namespace

void plan_attention(AttnArgs& a, int /*head_dim*/) {
  auto wgs = [&](int rows) { return ((a.n + rows - 1) / rows) * a.n_q_heads; };
  if (wgs(128) >= 192) a.variant = 0;
  else if (wgs(64) >= 128) a.variant = 1;
  else a.variant = 2;
  const int rows = kRowsOfVariant[a.variant];
  a.n_row_tiles = (a.n + rows - 1) / rows;
  a.total_work = a.n_row_tiles * a.n_q_heads;
  a.work_per_xcd = (a.total_work + kXcds - 1) / kXcds;
}

hipError_t launch_attention(const AttnArgs& a, int head_dim, hipStream_t s) {
  if (head_dim == 128) {
    switch (a.variant) {
      case 0: return launch_shape<128, 2, 2, 2>(a, s);
      case 1: return launch_shape<128, 2, 1, 4>(a, s);
      default: return launch_shape<128, 1, 1, 4>(a, s);
    }
  }
  switch (a.variant) {
    case 0: return launch_shape<64, 2, 2, 2>(a, s);
    case 1: return launch_shape<64, 2, 1, 4>(a, s);
    default: return launch_shape<64, 1, 1, 4>(a, s);
  }
}

}  // namespace kvp

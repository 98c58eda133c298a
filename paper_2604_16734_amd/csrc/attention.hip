// Attention of one block of queries over cache U block (Eq. 1 of the paper),
// for gfx950: bf16 MFMA 32x32x16, wave64, K and V tiles staged through LDS.
//
// Formulation.  Every wave owns QT tiles of 32 query rows and works on the
// TRANSPOSED problem: S^T = K Q^T (A operand = K tile from LDS, B operand = Q
// held in registers for the whole kernel) and O^T = V^T P^T (A operand = V^T
// from LDS, B operand = P^T).  In the 32x32 accumulator layout a lane holds one
// column, so with the transposed problem a lane holds ONE query row: the
// reference maximum, the running sum and the rescale factor of the online
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
// A workgroup is QW x KS waves: QW groups of query rows times a KS-way split of
// every staged key tile.  A wave takes 64 keys of each tile as two 32-key
// blocks X and Y; the KS partial results of a row are merged through LDS at the
// end.  The split keeps all 1024 SIMDs busy when a block of the prefix has
// fewer than 1024 wave-sized row tiles.
//
// Schedule.  One wave per SIMD, so matrix and vector work overlap inside the
// wave.  With S_X(t) = scores of block X of tile t, the loop body is
//   phase 1   MFMA: S_Y(t), O += P_Y(t-1) V     | VALU: P_X(t) = exp(S_X(t) - m)
//   barrier
//   phase 2   MFMA: O += P_X(t) V, S_X(t+1)     | VALU: P_Y(t) = exp(S_Y(t) - m)
//             then tile t+2 of K and tile t+1 of V go from registers to LDS and
//             the global loads of the tiles after them are issued.
// LDS holds two K tiles and two V tiles; one barrier per tile is enough because
// a buffer is only overwritten in the phase after its last reader.
//
// The reference maximum m is lazy: it is raised (and O, the running sum and the
// pending P rescaled) only when a block's maximum exceeds it by more than 2^8,
// which after the first tile practically never happens; exp(S - m) then stays
// below 2^8, harmless in fp32 and in bf16.  The result does not depend on which
// reference is used.
#include <type_traits>

#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kThreads = 256;
constexpr float kLazyLog2 = 8.f;   // raise the reference when a block maximum exceeds it by 2^8

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(unsigned, b);
}
__device__ __forceinline__ float bf16_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(unsigned x) { return __uint_as_float(x & 0xFFFF0000u); }

// value of the same row held by the other half of the wave (lane ^ 32)
__device__ __forceinline__ float max_with_other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D, int QT, int QW, int KS>
struct Shape {
  static constexpr int kRows = QW * QT * 32;          // query rows per workgroup
  static constexpr int kTk = KS * 64;                 // keys per staged tile
  static constexpr int kKStride = D + 8;              // bf16 elements per K row in LDS
  static constexpr int kVStride = kTk + 8;            // bf16 elements per V^T row in LDS
  static constexpr int kKTile = kTk * kKStride;       // elements
  static constexpr int kVTile = D * kVStride;
  static constexpr int kTileBytes = 2 * (kKTile + kVTile) * 2;   // two buffers each
  static constexpr int kMergeFloats = QT * (D / 32) * 16 * 64 + 2 * QT * 64;  // per wave
  static constexpr int kMergeBytes = (KS - 1) * QW * kMergeFloats * 4;
  static constexpr int kLdsBytes = kTileBytes > kMergeBytes ? kTileBytes : kMergeBytes;
  static constexpr int kKPieces = kTk * (D / 8);      // 16-byte pieces of a K tile
  static constexpr int kKPer = kKPieces / kThreads;
  static constexpr int kVGroups = (kTk / 4) * (D / 8);  // 4 keys x 8 channels each
  static constexpr int kVPer = kVGroups / kThreads;
  static_assert(kKPieces % kThreads == 0 && kVGroups % kThreads == 0, "tile must split evenly");
};

template <int D, int QT, int QW, int KS>
__global__ void __launch_bounds__(kThreads)
attention_kernel(const AttnArgs a) {
  using S = Shape<D, QT, QW, KS>;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  u16* const lds_k = reinterpret_cast<u16*>(lds_raw);              // [2][kKTile]
  u16* const lds_v = lds_k + 2 * S::kKTile;                        // [2][kVTile]

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

  const int n = a.n, c = a.c, n_cand = c + n;
  const int row0 = rt * S::kRows;                    // first query row of the workgroup
  const int q0 = row0 + qw * QT * 32;                // first query row of this wave
  const int rows_end = min(n, row0 + S::kRows);
  const int kv_end = c + rows_end;                   // keys any row of the workgroup can see
  const int n_tiles = (kv_end + S::kTk - 1) / S::kTk;
  // tiles [0, n_plain) are visible in full to every row of the workgroup
  const int n_plain = min(n_tiles, (c + row0 + 1) / S::kTk);

  const u16* kc = a.k_cache + (size_t)hk * a.budget * D;
  const u16* vc = a.v_cache + (size_t)hk * a.budget * D;
  const u16* kn = a.k_new + (size_t)hk * D;
  const u16* vn = a.v_new + (size_t)hk * D;
  const int new_stride = a.n_kv_heads * D;

  // ---- Q fragments: B operand, lane holds Q[q0 + 32 t + l32][16 s + 8 g .. + 7]
  bf16x8 qf[QT][D / 16];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int row = q0 + 32 * t + l32;
    const u16* src = a.q + ((size_t)row * a.n_q_heads + h) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      u32x4 x = {0u, 0u, 0u, 0u};
      if (row < n) x = *reinterpret_cast<const u32x4*>(src + 16 * s);
      qf[t][s] = __builtin_bit_cast(bf16x8, x);
    }
  }

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

  // ---- staging of key tiles: global -> registers -> LDS
  // K piece i = tid + 256 j: row i / (D/8), 16-byte column i % (D/8)
  // V group i = tid + 256 j: keys 4 (i % (Tk/4)) .. + 3, channels 8 (i / (Tk/4)) .. + 7
  u32x4 kst[S::kKPer];
  u32x4 vst[S::kVPer][4];
  const int k_row = tid / (D / 8), k_c8 = tid % (D / 8);
  constexpr int kKRowStep = kThreads / (D / 8);          // rows between a thread's K pieces
  const int v_quad = tid % (S::kTk / 4), v_oct = tid / (S::kTk / 4);
  constexpr int kVOctStep = kThreads / (S::kTk / 4);     // channel octets between a thread's V groups

  auto load_k = [&](int t) __attribute__((always_inline)) {
    const int base = t * S::kTk;
    if (base + S::kTk <= c) {
      const u16* p = kc + (size_t)base * D + k_row * D + 8 * k_c8;
#pragma unroll
      for (int j = 0; j < S::kKPer; ++j) kst[j] = *reinterpret_cast<const u32x4*>(p + j * kKRowStep * D);
    } else if (base >= c && base + S::kTk <= n_cand) {
      const u16* p = kn + (size_t)(base - c) * new_stride + (size_t)k_row * new_stride + 8 * k_c8;
#pragma unroll
      for (int j = 0; j < S::kKPer; ++j)
        kst[j] = *reinterpret_cast<const u32x4*>(p + (size_t)j * kKRowStep * new_stride);
    } else {
#pragma unroll
      for (int j = 0; j < S::kKPer; ++j) {
        const int kv = min(base + k_row + j * kKRowStep, n_cand - 1);   // past the end: any finite row
        const u16* p = kv < c ? kc + (size_t)kv * D : kn + (size_t)(kv - c) * new_stride;
        kst[j] = *reinterpret_cast<const u32x4*>(p + 8 * k_c8);
      }
    }
  };
  auto load_v = [&](int t) __attribute__((always_inline)) {
    const int base = t * S::kTk;
    if (base + S::kTk <= c) {
      const u16* p = vc + (size_t)base * D + 4 * v_quad * D + 8 * v_oct;
#pragma unroll
      for (int j = 0; j < S::kVPer; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          vst[j][e] = *reinterpret_cast<const u32x4*>(p + e * D + 8 * j * kVOctStep);
    } else if (base >= c && base + S::kTk <= n_cand) {
      const u16* p = vn + (size_t)(base - c) * new_stride + (size_t)(4 * v_quad) * new_stride + 8 * v_oct;
#pragma unroll
      for (int j = 0; j < S::kVPer; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          vst[j][e] = *reinterpret_cast<const u32x4*>(p + (size_t)e * new_stride + 8 * j * kVOctStep);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int kv = min(base + 4 * v_quad + e, n_cand - 1);
        const u16* p = (kv < c ? vc + (size_t)kv * D : vn + (size_t)(kv - c) * new_stride) + 8 * v_oct;
#pragma unroll
        for (int j = 0; j < S::kVPer; ++j) vst[j][e] = *reinterpret_cast<const u32x4*>(p + 8 * j * kVOctStep);
      }
    }
  };
  auto store_k = [&](int buf) __attribute__((always_inline)) {
    u16* kt = lds_k + buf * S::kKTile + k_row * S::kKStride + 8 * k_c8;
#pragma unroll
    for (int j = 0; j < S::kKPer; ++j)
      *reinterpret_cast<u32x4*>(kt + j * kKRowStep * S::kKStride) = kst[j];
  };
  auto store_v = [&](int buf) __attribute__((always_inline)) {
    const int key = 4 * v_quad;
    // key order inside a 32-key block: swap bits 2 and 3
    const int pos = (key & ~12) | ((key & 4) << 1) | ((key & 8) >> 1);
    u16* vt = lds_v + buf * S::kVTile + 8 * v_oct * S::kVStride + pos;
#pragma unroll
    for (int j = 0; j < S::kVPer; ++j) {
      const u32x4 r0 = vst[j][0], r1 = vst[j][1], r2 = vst[j][2], r3 = vst[j][3];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int wd = e >> 1;
        u32x2 col;
        if ((e & 1) == 0) {
          col.x = (r0[wd] & 0xFFFFu) | (r1[wd] << 16);
          col.y = (r2[wd] & 0xFFFFu) | (r3[wd] << 16);
        } else {
          col.x = (r0[wd] >> 16) | (r1[wd] & 0xFFFF0000u);
          col.y = (r2[wd] >> 16) | (r3[wd] & 0xFFFF0000u);
        }
        *reinterpret_cast<u32x2*>(vt + (8 * j * kVOctStep + e) * S::kVStride) = col;
      }
    }
  };

  const float sl2 = a.scale_log2;
  const float lazy_raw = kLazyLog2 / sl2;     // the lazy margin in units of the raw dot product

  // S^T block = K[block rows] Q^T, block x in {0 (X), 1 (Y)} of this wave's 64 keys of the tile
  auto qk = [&](f32x16 (&s)[QT], int kbuf, int x) __attribute__((always_inline)) {
    const u16* krow = lds_k + kbuf * S::kKTile + (ks * 64 + 32 * x + l32) * S::kKStride + 8 * g;
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const bf16x8 ka = *reinterpret_cast<const bf16x8*>(krow + 16 * st);
#pragma unroll
      for (int t = 0; t < QT; ++t)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[t][st], s[t], 0, 0, 0);
    }
  };
  // O^T += V^T[block] P^T
  auto pv = [&](const unsigned (&pb)[QT][8], int vbuf, int x) __attribute__((always_inline)) {
    const u16* vrow = lds_v + vbuf * S::kVTile + l32 * S::kVStride + ks * 64 + 32 * x + 8 * g;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8 va = *reinterpret_cast<const bf16x8*>(vrow + dt * 32 * S::kVStride + 16 * mm);
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          const u32x4 px = {pb[t][4 * mm], pb[t][4 * mm + 1], pb[t][4 * mm + 2], pb[t][4 * mm + 3]};
          o[t][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, px), o[t][dt], 0, 0, 0);
        }
      }
    }
  };
  // Hide block keys a row may not see, then decide whether the reference maximum must rise.
  // `pend` is the P block that has been computed against the old reference but not yet
  // multiplied into O: it is rescaled together with O.
  auto prepare = [&](f32x16 (&s)[QT], unsigned (&pend)[QT][8], int kb, auto mask) __attribute__((always_inline)) {
    if constexpr (decltype(mask)::value) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        // key kb + 8 (r / 4) + 4 g + r % 4 is visible when it is cached, or a block key not after the row
        const int lim = min(q0 + 32 * t + l32 + c, n_cand - 1) - kb - 4 * g;   // visible iff 8 (r/4) + r%4 <= lim
#pragma unroll
        for (int r = 0; r < 16; ++r) s[t][r] = (8 * (r >> 2) + (r & 3) <= lim) ? s[t][r] : -INFINITY;
      }
    }
    float mx[QT];
    bool raise = false;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float v = s[t][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) v = fmaxf(v, s[t][r]);
      mx[t] = max_with_other_half(v);
      raise |= mx[t] > m_ref[t] + lazy_raw;     // also true for the first visible key (m_ref = -inf)
    }
    if (__any(raise)) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const bool up = mx[t] > m_ref[t] + lazy_raw;
        const float m_new = up ? mx[t] : m_ref[t];
        const float alpha = up ? __builtin_amdgcn_exp2f((m_ref[t] - m_new) * sl2) : 1.f;
        m_ref[t] = m_new;
        l_run[t] *= alpha;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][dt][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 8; ++r)
          pend[t][r] = pack_bf16(bf16_lo(pend[t][r]) * alpha, bf16_hi(pend[t][r]) * alpha);
      }
    }
  };
  // P = exp2((S - m) * scale): the part that overlaps with the matrix work
  auto exponentiate = [&](const f32x16 (&s)[QT], unsigned (&pb)[QT][8]) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const float m_use = (m_ref[t] == -INFINITY) ? 0.f : m_ref[t];   // row has seen nothing yet
      const float neg = -m_use * sl2;
      float sum = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][2 * r], sl2, neg));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][2 * r + 1], sl2, neg));
        sum += p0 + p1;
        pb[t][r] = pack_bf16(p0, p1);
      }
      l_run[t] += sum;
    }
  };

  // ---- prologue: K(0), K(1), V(0) in LDS, K(2), V(1) in registers, S_X(0) computed
  f32x16 sx[QT], sy[QT];
  unsigned px[QT][8], py[QT][8];
#pragma unroll
  for (int t = 0; t < QT; ++t)
#pragma unroll
    for (int r = 0; r < 8; ++r) { px[t][r] = 0u; py[t][r] = 0u; }
  load_k(0);
  load_v(0);
  store_k(0);
  store_v(0);
  load_k(1);
  // V buffer 1 is read as "V(-1)" with P = 0 in the first phase: make it finite
  for (int i = tid; i < S::kVTile / 8; i += kThreads)
    reinterpret_cast<u32x4*>(lds_v + S::kVTile)[i] = u32x4{0u, 0u, 0u, 0u};
  store_k(1);
  load_k(2);
  load_v(1);
  __syncthreads();
  qk(sx, 0, 0);

  auto body = [&](int t, auto mask) __attribute__((always_inline)) {
    const int kb = t * S::kTk + ks * 64;
    // ---- phase 1
    prepare(sx, py, kb, mask);
    qk(sy, t & 1, 1);
    pv(py, (t + 1) & 1, 1);
    exponentiate(sx, px);
    __syncthreads();
    // ---- phase 2
    prepare(sy, px, kb + 32, mask);
    pv(px, t & 1, 0);
    qk(sx, (t + 1) & 1, 0);
    exponentiate(sy, py);
    store_k(t & 1);            // K(t+2)
    store_v((t + 1) & 1);      // V(t+1)
    load_k(t + 3);
    load_v(t + 2);
  };
  for (int t = 0; t < n_plain; ++t) body(t, std::false_type{});
  for (int t = n_plain; t < n_tiles; ++t) body(t, std::true_type{});
  __syncthreads();
  pv(py, (n_tiles + 1) & 1, 1);   // P_Y of the last tile

  // lanes l and l + 32 each summed half of the keys of a row
#pragma unroll
  for (int t = 0; t < QT; ++t) l_run[t] = sum_with_other_half(l_run[t]);

  // ---- merge the KS partial results of every row through LDS
  if (KS > 1) {
    float* mrg = reinterpret_cast<float*>(lds_raw);
    __syncthreads();   // everybody is done with the tiles
    if (ks > 0) {
      float* mine = mrg + (size_t)((ks - 1) * QW + qw) * S::kMergeFloats;
#pragma unroll
      for (int t = 0; t < QT; ++t) {
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            mine[((t * (D / 32) + dt) * 16 + r) * 64 + lane] = o[t][dt][r];
        mine[QT * (D / 32) * 16 * 64 + t * 64 + lane] = m_ref[t];
        mine[QT * (D / 32) * 16 * 64 + (QT + t) * 64 + lane] = l_run[t];
      }
    }
    __syncthreads();
    if (ks == 0) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        float mt = m_ref[t];
        for (int s2 = 1; s2 < KS; ++s2) {
          const float* other = mrg + (size_t)((s2 - 1) * QW + qw) * S::kMergeFloats;
          mt = fmaxf(mt, other[QT * (D / 32) * 16 * 64 + t * 64 + lane]);
        }
        const float m_use = (mt == -INFINITY) ? 0.f : mt;
        const float f0 = __builtin_amdgcn_exp2f((m_ref[t] - m_use) * sl2);
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
        m_ref[t] = mt;
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
            u32x2 pk;
            pk.x = pack_bf16(o[t][dt][4 * j] * inv, o[t][dt][4 * j + 1] * inv);
            pk.y = pack_bf16(o[t][dt][4 * j + 2] * inv, o[t][dt][4 * j + 3] * inv);
            *reinterpret_cast<u32x2*>(dstp + 32 * dt + 8 * j) = pk;
          }
        if (g == 0)
          a.lse2[(size_t)h * a.lse_stride + row] = m_ref[t] * sl2 + __builtin_log2f(l_run[t]);
      }
    }
  }
}

template <int D, int QT, int QW, int KS>
hipError_t launch_shape(const AttnArgs& a, hipStream_t s) {
  using S = Shape<D, QT, QW, KS>;
  auto kern = attention_kernel<D, QT, QW, KS>;
  static bool attr_done = false;   // per process; the attribute belongs to the function
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

constexpr int kRowsOfVariant[2] = {128, 64};

}  // namespace

void plan_attention(AttnArgs& a, int /*head_dim*/) {
  auto wgs = [&](int rows) { return ((a.n + rows - 1) / rows) * a.n_q_heads; };
  a.variant = wgs(128) >= 192 ? 0 : 1;
  const int rows = kRowsOfVariant[a.variant];
  a.n_row_tiles = (a.n + rows - 1) / rows;
  a.total_work = a.n_row_tiles * a.n_q_heads;
  a.work_per_xcd = (a.total_work + kXcds - 1) / kXcds;
}

hipError_t launch_attention(const AttnArgs& a, int head_dim, hipStream_t s) {
  if (head_dim == 128) {
    if (a.variant == 0) return launch_shape<128, 2, 2, 2>(a, s);
    return launch_shape<128, 1, 2, 2>(a, s);
  }
  if (a.variant == 0) return launch_shape<64, 2, 2, 2>(a, s);
  return launch_shape<64, 1, 2, 2>(a, s);
}

}  // namespace kvp

// Bringing the cache back to its budget in place (Alg. 1 line 10, "reduce cache
// to budget M"), plus this library's grid-neighbour merge.
//
// Two kernels, because a freed slot may still be needed as a merge source:
//   merge_kernel  every destination row becomes the weighted mean of itself
//                 and its sources, all read at their pre-compaction places.
//                 A destination that already sits in the cache is rewritten in
//                 place (no other row reads it: sources are evicted rows,
//                 destinations are kept rows); a destination that is a block
//                 token goes to a staging row.
//   move_kernel   every kept block token is copied into its free slot, from
//                 the staging row if it was a merge destination, and the
//                 slot's token index and weight are set.  Kept cache rows never
//                 move.  With `identity` it is the plain append of a block to a
//                 cache that is not full.
// One wave per row pair: lanes 0-31 carry the K row, lanes 32-63 the V row.
#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = kThreads / 64;

__device__ __forceinline__ float bf16_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(unsigned x) { return __uint_as_float(x & 0xFFFF0000u); }
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(unsigned, b);
}

// W words of 2 bf16 per lane: head_dim = 64 W
template <int W>
struct Row {
  unsigned w[W];
};

template <int W>
__device__ __forceinline__ Row<W> load_row(const u16* p, int l32) {
  Row<W> r;
  if (W == 2) {
    const uint2 x = *reinterpret_cast<const uint2*>(p + 4 * l32);
    r.w[0] = x.x; r.w[W - 1] = x.y;
  } else {
    r.w[0] = *reinterpret_cast<const unsigned*>(p + 2 * l32);
  }
  return r;
}
template <int W>
__device__ __forceinline__ void store_row(u16* p, int l32, const Row<W>& r) {
  if (W == 2) {
    *reinterpret_cast<uint2*>(p + 4 * l32) = make_uint2(r.w[0], r.w[W - 1]);
  } else {
    *reinterpret_cast<unsigned*>(p + 2 * l32) = r.w[0];
  }
}

template <int W>
__global__ void __launch_bounds__(kThreads)
merge_kernel(const CompactArgs a) {
  constexpr int D = 64 * W;
  const int hk = blockIdx.y;
  const int j = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (j >= a.counts[hk].n_dst) return;
  const int lane = threadIdx.x & 63, l32 = lane & 31;
  const bool is_v = lane >= 32;
  const DstEntry e = a.dsts[(size_t)hk * a.chunk_max + j];

  u16* cache = (is_v ? a.v_cache : a.k_cache) + (size_t)hk * a.budget * D;
  const u16* fresh = (is_v ? a.v_new : a.k_new) + (size_t)hk * D;
  const size_t fresh_stride = (size_t)a.n_kv_heads * D;
  const float* wts = a.weight + (size_t)hk * a.budget;
  auto row_of = [&](int pos) -> const u16* {
    return pos < a.c ? cache + (size_t)pos * D : fresh + (size_t)(pos - a.c) * fresh_stride;
  };
  auto weight_of = [&](int pos) -> float { return pos < a.c ? wts[pos] : 1.f; };

  // fetch the destination and all (at most six) sources at once, then add them up in order
  // sources arrive in no particular order: sort them by candidate position (unused slots last)
  // so that the fp32 sum below is taken in one fixed order
  int pos[kNeighbours + 1];
  pos[0] = e.pos;
#pragma unroll
  for (int k = 0; k < kNeighbours; ++k) pos[k + 1] = k < e.n_src ? e.src[k] : 0x7FFFFFFF;
#pragma unroll
  for (int pass = 0; pass < kNeighbours; ++pass)
#pragma unroll
    for (int k = 1 + (pass & 1); k + 1 <= kNeighbours; k += 2) {
      const int lo = min(pos[k], pos[k + 1]), hi = max(pos[k], pos[k + 1]);
      pos[k] = lo; pos[k + 1] = hi;
    }
  float wt[kNeighbours + 1];
  Row<W> rows[kNeighbours + 1];
#pragma unroll
  for (int k = 0; k <= kNeighbours; ++k) {
    const bool on = k <= e.n_src;
    const int pk = on ? pos[k] : e.pos;          // an unused entry re-reads the destination, weight 0
    wt[k] = on ? weight_of(pk) : 0.f;
    rows[k] = load_row<W>(row_of(pk), l32);
  }
  float total = wt[0];
  float acc[2 * W];
#pragma unroll
  for (int k = 0; k < W; ++k) {
    acc[2 * k] = wt[0] * bf16_lo(rows[0].w[k]);
    acc[2 * k + 1] = wt[0] * bf16_hi(rows[0].w[k]);
  }
#pragma unroll
  for (int s = 1; s <= kNeighbours; ++s) {
    total += wt[s];
#pragma unroll
    for (int k = 0; k < W; ++k) {
      acc[2 * k] = __builtin_fmaf(wt[s], bf16_lo(rows[s].w[k]), acc[2 * k]);
      acc[2 * k + 1] = __builtin_fmaf(wt[s], bf16_hi(rows[s].w[k]), acc[2 * k + 1]);
    }
  }
  Row<W> res;
#pragma unroll
  for (int k = 0; k < W; ++k) res.w[k] = pack_bf16(acc[2 * k] / total, acc[2 * k + 1] / total);

  if (e.pos < a.c) {
    store_row<W>(cache + (size_t)e.pos * D, l32, res);
    if (lane == 0) a.weight[(size_t)hk * a.budget + e.pos] = total;
  } else {
    u16* st = (is_v ? a.stage_v : a.stage_k) + ((size_t)hk * a.chunk_max + j) * D;
    store_row<W>(st, l32, res);
    if (lane == 0) a.stage_w[(size_t)hk * a.chunk_max + j] = total;
  }
}

template <int W>
__global__ void __launch_bounds__(kThreads)
move_kernel(const CompactArgs a) {
  constexpr int D = 64 * W;
  const int hk = blockIdx.y;
  const int i = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  const int count = a.identity ? a.n : a.counts[hk].n_moves;
  if (i >= count) return;
  const int lane = threadIdx.x & 63, l32 = lane & 31;
  const bool is_v = lane >= 32;
  int pos, slot, stage;
  if (a.identity) {
    pos = a.c + i; slot = a.c + i; stage = -1;
  } else {
    const MoveEntry e = a.moves[(size_t)hk * a.chunk_max + i];
    pos = e.pos; slot = e.slot; stage = e.stage;
  }
  const u16* src;
  if (stage >= 0)
    src = (is_v ? a.stage_v : a.stage_k) + ((size_t)hk * a.chunk_max + stage) * D;
  else
    src = (is_v ? a.v_new : a.k_new) + ((size_t)(pos - a.c) * a.n_kv_heads + hk) * D;
  u16* dstp = (is_v ? a.v_cache : a.k_cache) + ((size_t)hk * a.budget + slot) * D;
  store_row<W>(dstp, l32, load_row<W>(src, l32));
  if (lane == 0) {
    a.token_idx[(size_t)hk * a.budget + slot] = a.t0 + (pos - a.c);
    a.weight[(size_t)hk * a.budget + slot] = stage >= 0 ? a.stage_w[(size_t)hk * a.chunk_max + stage] : 1.f;
  }
}

struct InitArgs {
  Seg segs[KVP_MAX_SEGMENTS];
  Seg* dst;
  int n_segs;
};

__global__ void fill_kernel(int32_t* token_idx, float* weight, size_t n, InitArgs ia) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    token_idx[i] = -1;
    weight[i] = 0.f;
  }
  if (i < (size_t)ia.n_segs) ia.dst[i] = ia.segs[i];
}

}  // namespace

hipError_t launch_merge(const CompactArgs& a, hipStream_t s) {
  const dim3 grid(a.blocks_per_head, a.n_kv_heads);
  if (a.head_dim == 128)
    hipLaunchKernelGGL(merge_kernel<2>, grid, dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(merge_kernel<1>, grid, dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_move(const CompactArgs& a, hipStream_t s) {
  const dim3 grid(a.blocks_per_head, a.n_kv_heads);
  if (a.head_dim == 128)
    hipLaunchKernelGGL(move_kernel<2>, grid, dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(move_kernel<1>, grid, dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

int rows_per_compact_block() { return kRowsPerBlock; }

hipError_t launch_init(int32_t* token_idx, float* weight, size_t n_slots, const Seg* host_segs,
                       int n_segs, Seg* dev_segs, hipStream_t s) {
  InitArgs ia;
  for (int i = 0; i < KVP_MAX_SEGMENTS; ++i) ia.segs[i] = i < n_segs ? host_segs[i] : Seg{0, 0, 0, 0, 0, 0, 0};
  ia.dst = dev_segs;
  ia.n_segs = n_segs;
  size_t n = n_slots > (size_t)n_segs ? n_slots : (size_t)n_segs;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, s, token_idx, weight, n_slots, ia);
  return hipGetLastError();
}

}  // namespace kvp

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
// A row pair (the K row and the V row of one slot) is carried by 2 D / 8 lanes, 16 bytes each:
// 32 lanes at head dimension 128 (two pairs per wave), 16 at 64 (four pairs per wave).  A launch
// covers a group of layers: grid (row blocks, KV heads, layers).
#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kThreads = kCompactThreads;

__device__ __forceinline__ float bf16_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(unsigned x) { return __uint_as_float(x & 0xFFFF0000u); }
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(unsigned, b);
}

template <int D>
struct Lanes {
  static constexpr int kPerRow = D / 8;               // 16-byte pieces of a row
  static constexpr int kPerPair = 2 * kPerRow;        // K row then V row
  static constexpr int kPairsPerBlock = kThreads / kPerPair;
};

template <int D>
__global__ void __launch_bounds__(kThreads)
merge_kernel(const CompactArgs a) {
  using L = Lanes<D>;
  const int hk = blockIdx.y, li = blockIdx.z;
  const int n_dst = in_set_of(a.counts, a.g, li)[hk].n_dst;
  const int sub = threadIdx.x % L::kPerPair;
  const bool is_v = sub >= L::kPerRow;
  const int piece = sub % L::kPerRow;
  // The grid is capped (a launch for sixteen layers would otherwise be mostly workgroups that find
  // nothing to do, and starting those costs more than the rows take): a workgroup walks the
  // destinations with the stride of the grid.
  for (int j = blockIdx.x * L::kPairsPerBlock + threadIdx.x / L::kPerPair; j < n_dst;
       j += gridDim.x * L::kPairsPerBlock) {
    const DstEntry e = in_set_of(a.dsts, a.g, li)[(size_t)hk * a.chunk_max + j];

    u16* cache = (is_v ? a.v_cache : a.k_cache) + (long long)li * a.g.kv_stride + (size_t)hk * a.budget * D;
    const u16* fresh = (is_v ? a.g.v_new[li] : a.g.k_new[li]) + (size_t)hk * D;
    const size_t fresh_stride = (size_t)a.n_kv_heads * D;
    float* wts = a.weight + (long long)li * a.g.meta_stride + (size_t)hk * a.budget;
    auto row_of = [&](int pos) -> const u16* {
      return pos < a.c ? cache + (size_t)pos * D : fresh + (size_t)(pos - a.c) * fresh_stride;
    };
    auto weight_of = [&](int pos) -> float { return pos < a.c ? wts[pos] : 1.f; };

    // fetch the destination and all (at most six) sources at once, then add them up in order.
    // Sources arrive in no particular order: sort them by candidate position (unused slots last)
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
    uint4 rows[kNeighbours + 1];
#pragma unroll
    for (int k = 0; k <= kNeighbours; ++k) {
      const bool on = k <= e.n_src;
      const int pk = on ? pos[k] : e.pos;          // an unused entry re-reads the destination, weight 0
      wt[k] = on ? weight_of(pk) : 0.f;
      rows[k] = *reinterpret_cast<const uint4*>(row_of(pk) + 8 * piece);
    }
    float total = wt[0];
    float acc[8];
    {
      const unsigned w[4] = {rows[0].x, rows[0].y, rows[0].z, rows[0].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] = wt[0] * bf16_lo(w[k]);
        acc[2 * k + 1] = wt[0] * bf16_hi(w[k]);
      }
    }
#pragma unroll
    for (int s = 1; s <= kNeighbours; ++s) {
      total += wt[s];
      const unsigned w[4] = {rows[s].x, rows[s].y, rows[s].z, rows[s].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] = __builtin_fmaf(wt[s], bf16_lo(w[k]), acc[2 * k]);
        acc[2 * k + 1] = __builtin_fmaf(wt[s], bf16_hi(w[k]), acc[2 * k + 1]);
      }
    }
    uint4 res;
    res.x = pack_bf16(acc[0] / total, acc[1] / total);
    res.y = pack_bf16(acc[2] / total, acc[3] / total);
    res.z = pack_bf16(acc[4] / total, acc[5] / total);
    res.w = pack_bf16(acc[6] / total, acc[7] / total);

    if (e.pos < a.c) {
      *reinterpret_cast<uint4*>(cache + (size_t)e.pos * D + 8 * piece) = res;
      if (sub == 0) wts[e.pos] = total;
    } else {
      u16* st = in_set_of(is_v ? a.stage_v : a.stage_k, a.g, li) + ((size_t)hk * a.chunk_max + j) * D;
      *reinterpret_cast<uint4*>(st + 8 * piece) = res;
      if (sub == 0) in_set_of(a.stage_w, a.g, li)[(size_t)hk * a.chunk_max + j] = total;
    }
  }
}

// kIdentity: the plain append of all n block tokens to slots c .. c + n - 1 (a compile-time switch:
// chosen at run time, the two sources of the row count, a kernel argument and a device array, make
// the compiler keep the arguments in memory)
template <int D, bool kIdentity>
__global__ void __launch_bounds__(kThreads)
move_kernel(const CompactArgs a) {
  using L = Lanes<D>;
  const int hk = blockIdx.y, li = blockIdx.z;
  const int sub = threadIdx.x % L::kPerPair;
  const bool is_v = sub >= L::kPerRow;
  const int piece = sub % L::kPerRow;
  int n_rows;
  if constexpr (kIdentity) n_rows = a.n;
  else n_rows = in_set_of(a.counts, a.g, li)[hk].n_moves;
  // capped grid, as in merge_kernel: a workgroup walks the rows with the stride of the grid
  for (int i = blockIdx.x * L::kPairsPerBlock + threadIdx.x / L::kPerPair; i < n_rows;
       i += gridDim.x * L::kPairsPerBlock) {
    int pos, slot, stage;
    if constexpr (kIdentity) {
      pos = a.c + i; slot = a.c + i; stage = -1;
    } else {
      const MoveEntry e = in_set_of(a.moves, a.g, li)[(size_t)hk * a.chunk_max + i];
      pos = e.pos; slot = e.slot; stage = e.stage;
    }
    // (both candidates are formed outside the branch: they come from the kernel arguments, and a load
    // of an argument whose address depends on a per-lane condition would push the arguments to memory)
    const u16* const k_new = a.g.k_new[li];
    const u16* const v_new = a.g.v_new[li];
    const u16* const staged = in_set_of(is_v ? a.stage_v : a.stage_k, a.g, li) + ((size_t)hk * a.chunk_max + max(stage, 0)) * D;
    const u16* const fresh = (is_v ? v_new : k_new) + ((size_t)(pos - a.c) * a.n_kv_heads + hk) * D;
    const u16* const src = stage >= 0 ? staged : fresh;
    u16* dstp = (is_v ? a.v_cache : a.k_cache) + (long long)li * a.g.kv_stride + ((size_t)hk * a.budget + slot) * D;
    *reinterpret_cast<uint4*>(dstp + 8 * piece) = *reinterpret_cast<const uint4*>(src + 8 * piece);
    if (sub == 0) {
      const size_t m = (size_t)((long long)li * a.g.meta_stride) + (size_t)hk * a.budget + slot;
      a.token_idx[m] = a.t0 + (pos - a.c);
      a.weight[m] = stage >= 0 ? in_set_of(a.stage_w, a.g, li)[(size_t)hk * a.chunk_max + stage] : 1.f;
    }
  }
}

struct InitArgs {
  Seg segs[KVP_MAX_SEGMENTS];
  Seg* dst;
  unsigned long long* totals;
  int n_segs;
};

__global__ void fill_kernel(int32_t* token_idx, float* weight, size_t n, InitArgs ia) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    token_idx[i] = -1;
    weight[i] = 0.f;
  }
  if (i < (size_t)ia.n_segs) ia.dst[i] = ia.segs[i];
  if (i < (size_t)KVP_T_COUNT) ia.totals[i] = 0ull;
}

}  // namespace

namespace {
// row blocks per (KV head, layer): what the rows could need, but not more than keeps the whole
// launch at about kCompactTargetWorkgroups workgroups
int capped_blocks(const CompactArgs& a) {
  const int pairs = a.n_kv_heads * a.g.n_layers;
  int cap = (kCompactTargetWorkgroups + pairs - 1) / pairs;
  if (cap < 1) cap = 1;
  return a.blocks_per_head < cap ? a.blocks_per_head : cap;
}
}  // namespace

hipError_t launch_merge(const CompactArgs& a, hipStream_t s) {
  const dim3 grid(capped_blocks(a), a.n_kv_heads, a.g.n_layers);
  if (a.head_dim == 128)
    hipLaunchKernelGGL(merge_kernel<128>, grid, dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(merge_kernel<64>, grid, dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_move(const CompactArgs& a, hipStream_t s) {
  const dim3 grid(capped_blocks(a), a.n_kv_heads, a.g.n_layers);
  if (a.head_dim == 128) {
    if (a.identity) hipLaunchKernelGGL((move_kernel<128, true>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((move_kernel<128, false>), grid, dim3(kThreads), 0, s, a);
  } else {
    if (a.identity) hipLaunchKernelGGL((move_kernel<64, true>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((move_kernel<64, false>), grid, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_init(int32_t* token_idx, float* weight, size_t n_slots, const Seg* host_segs,
                       int n_segs, Seg* dev_segs, unsigned long long* totals, hipStream_t s) {
  InitArgs ia;
  for (int i = 0; i < KVP_MAX_SEGMENTS; ++i) ia.segs[i] = i < n_segs ? host_segs[i] : Seg{0, 0, 0, 0, 0, 0, 0};
  ia.dst = dev_segs;
  ia.totals = totals;
  ia.n_segs = n_segs;
  size_t n = n_slots > (size_t)KVP_MAX_SEGMENTS ? n_slots : (size_t)KVP_MAX_SEGMENTS;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, s, token_idx, weight, n_slots, ia);
  return hipGetLastError();
}

}  // namespace kvp

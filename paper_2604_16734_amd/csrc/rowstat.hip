// Row statistics (log2-domain log-sum-exp of every softmax row of Eq. 4) for a
// short list of proxy queries (Sec. 3.2) over all candidates of a KV head.
//
// The attention kernel gives these statistics as a by-product, but it spreads
// its work over query rows: a few dozen proxy queries would leave most of the
// chip idle while a handful of workgroups walk all the keys.  Here the keys are
// spread instead.  A workgroup takes 256 keys of one KV head, which its four
// waves keep in registers (64 each), and a share of the (query head, 32-row
// tile) items of the KV group; per item a wave computes S^T = K Q^T (a lane then
// holds one query row, its logits in registers), reduces them to (max, sum of
// exp2) per row, and the four pairs are folded through LDS into one partial per
// (head, row, key block).  A second, tiny kernel folds the
// partials of all key blocks, in a fixed order, into the statistic the scoring
// kernel reads.  Every candidate is visible to every proxy query (the prompt
// follows the visual tokens), so there is no mask beyond the end of the keys.
#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kSub = 2;                        // 32-key subtiles per wave
constexpr int kWaveKeys = 32 * kSub;
constexpr int kBlockKeys = 4 * kWaveKeys;
static_assert(kBlockKeys == kRowstatBlockKeys, "the host plans with this block size");

__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

// grid (key blocks, KV heads x item splits, layers of the group).  An item is one 32-row tile of
// one query head of the KV group; a workgroup keeps its 256 keys in registers (A operand: a wave
// its 64) and takes `items_per_wg` items one after the other, the query fragments of the next
// item on their way while the current one is worked on: every key is fetched once per workgroup
// instead of once per item.
template <int D>
__global__ void __launch_bounds__(kThreads)
rowstat_kernel(const RowstatArgs a) {
  __shared__ float s_m[2][4][32], s_l[2][4][32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int kb = blockIdx.x, li = blockIdx.z;
  const int hk = blockIdx.y / a.item_splits, isplit = blockIdx.y % a.item_splits;
  const int n_rt = (a.n + 31) / 32;
  const int n_items = group * n_rt;
  const int item0 = isplit * a.items_per_wg, item1 = min(n_items, item0 + a.items_per_wg);
  if (item0 >= item1) return;
  const u16* const q_rows = a.q_layer[li];
  const u16* const k_new = a.g.k_new[li];
  const u16* const k_cache = a.k_cache + (long long)li * a.g.kv_stride;
  float* const part_m = in_set_of(a.part_m, a.g, li);
  float* const part_l = in_set_of(a.part_l, a.g, li);
  const int c = a.c, n_cand = a.c + a.n_keys;
  const int key0 = kb * kBlockKeys + wave * kWaveKeys;

  // A operand: subtile t of this wave is keys key0 + 32 t + (0..31); lane holds K[key][16 s + 8 g .. + 7]
  bf16x8 kf[kSub][D / 16];
#pragma unroll
  for (int t = 0; t < kSub; ++t) {
    const int kv = min(key0 + 32 * t + l32, n_cand - 1);
    const u16* src = (kv < c ? k_cache + ((size_t)hk * a.budget + kv) * D
                             : k_new + ((size_t)(kv - c) * a.n_kv_heads + hk) * D) + 8 * g;
#pragma unroll
    for (int st = 0; st < D / 16; ++st)
      kf[t][st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * st));
  }
  // B operand of item i: lane holds Q[32 rt + l32][16 s + 8 g .. + 7] of head hk group + i / n_rt
  auto load_q = [&](bf16x8 (&qf)[D / 16], int item) __attribute__((always_inline)) {
    const int h = hk * group + item / n_rt, rt = item % n_rt;
    const int row = min(32 * rt + l32, a.n - 1);
    const u16* src = q_rows + ((size_t)row * a.n_q_heads + h) * D + 8 * g;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) qf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * st));
  };
  auto one_item = [&](const bf16x8 (&qf)[D / 16], int item, int buf) __attribute__((always_inline)) {
    // S^T subtile t: rows = keys, columns = the 32 query rows
    float m = -INFINITY, l = 0.f;
    f32x16 s[kSub];
#pragma unroll
    for (int t = 0; t < kSub; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
      for (int st = 0; st < D / 16; ++st) s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t][st], qf[st], s[t], 0, 0, 0);
      // accumulator register r of lane group g is key 8 (r / 4) + 4 g + r % 4 of the subtile
      const int left = n_cand - (key0 + 32 * t) - 4 * g;      // keys of this lane's list that exist
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (8 * (r >> 2) + (r & 3) >= left) s[t][r] = -INFINITY;
        m = fmaxf(m, s[t][r]);
      }
    }
    m = fmaxf(m, other_half(m));               // lanes l and l + 32 hold the two halves of a row's keys
    const float m_use = m == -INFINITY ? 0.f : m;
#pragma unroll
    for (int t = 0; t < kSub; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) l += __builtin_amdgcn_exp2f((s[t][r] - m_use) * a.scale_log2);
    l += other_half(l);
    if (g == 0) { s_m[buf][wave][l32] = m; s_l[buf][wave][l32] = l; }
    __syncthreads();             // one barrier per item: the next item writes the other buffer
    if (tid < 32) {
      float mm = s_m[buf][0][tid];
#pragma unroll
      for (int w = 1; w < 4; ++w) mm = fmaxf(mm, s_m[buf][w][tid]);
      const float mu = mm == -INFINITY ? 0.f : mm;
      float ll = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) ll += s_l[buf][w][tid] * __builtin_amdgcn_exp2f((s_m[buf][w][tid] - mu) * a.scale_log2);
      const int h = hk * group + item / n_rt, rt = item % n_rt;
      const int row = 32 * rt + tid;
      if (row < a.n) {
        const size_t at = ((size_t)h * a.n + row) * a.n_kv_blocks + kb;
        part_m[at] = mm;
        part_l[at] = ll;
      }
    }
  };
  bf16x8 qa[D / 16], qb[D / 16];
  load_q(qa, item0);
  for (int item = item0; item < item1; item += 2) {
    load_q(qb, min(item + 1, item1 - 1));
    one_item(qa, item, 0);
    load_q(qa, min(item + 2, item1 - 1));
    if (item + 1 < item1) one_item(qb, item + 1, 1);
  }
}

// lse2[h][row] from the partials of all key blocks, folded in block order
__global__ void rowstat_fold_kernel(const RowstatArgs a) {
  // grid (blocks of 256 rows, layers of the group)
  const int i = blockIdx.x * blockDim.x + threadIdx.x, li = blockIdx.y;
  if (i >= a.n_q_heads * a.n) return;
  const float* const part_m = in_set_of(a.part_m, a.g, li);
  const float* const part_l = in_set_of(a.part_l, a.g, li);
  const int h = i / a.n, row = i % a.n;
  const size_t at = ((size_t)h * a.n + row) * a.n_kv_blocks;
  float mm = -INFINITY;
  for (int b = 0; b < a.n_kv_blocks; ++b) mm = fmaxf(mm, part_m[at + b]);
  float ll = 0.f;
  for (int b = 0; b < a.n_kv_blocks; ++b) ll += part_l[at + b] * __builtin_amdgcn_exp2f((part_m[at + b] - mm) * a.scale_log2);
  in_set_of(a.lse2, a.g, li)[(size_t)h * a.lse_stride + row] = mm * a.scale_log2 + __builtin_log2f(ll);
}

}  // namespace

hipError_t launch_rowstat(RowstatArgs a, int head_dim, hipStream_t s) {
  a.n_kv_blocks = rowstat_key_blocks(a.c + a.n_keys);
  if (a.g.n_layers < 1 || a.g.n_layers > kMaxGroupLayers) return hipErrorInvalidValue;
  // items (32-row tiles x query heads of a KV group) per workgroup: as many as still leave about
  // two workgroups per compute unit
  const int n_items = (a.n_q_heads / a.n_kv_heads) * ((a.n + 31) / 32);
  const long long units = (long long)n_items * a.n_kv_blocks * a.n_kv_heads * a.g.n_layers;
  long long per = units / 512;
  a.items_per_wg = (int)(per < 1 ? 1 : per > n_items ? n_items : per);
  a.item_splits = (n_items + a.items_per_wg - 1) / a.items_per_wg;
  if ((long long)a.n_kv_heads * a.item_splits > 65535) return hipErrorInvalidValue;
  const dim3 grid(a.n_kv_blocks, a.n_kv_heads * a.item_splits, a.g.n_layers);
  if (head_dim == 128) hipLaunchKernelGGL(rowstat_kernel<128>, grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(rowstat_kernel<64>, grid, dim3(kThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int total = a.n_q_heads * a.n;
  hipLaunchKernelGGL(rowstat_fold_kernel, dim3((total + 255) / 256, a.g.n_layers), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace kvp

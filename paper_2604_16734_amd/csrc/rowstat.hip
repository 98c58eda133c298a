// Row statistics (log2-domain log-sum-exp of every softmax row of Eq. 4) for a
// short list of proxy queries (Sec. 3.2) over all candidates of a KV head.
//
// The attention kernel gives these statistics as a by-product, but it spreads
// its work over query rows: a few dozen proxy queries would leave most of the
// chip idle while a handful of workgroups walk all the keys.  Here the keys are
// spread instead.  A workgroup takes 32 rows of one query head and 512 keys;
// each of its four waves computes S^T = K Q^T for 128 keys straight from global
// memory (a lane then holds one query row, its logits in registers), reduces
// them to (max, sum of exp2) per row, and the four pairs are folded through LDS
// into one partial per (head, row, key block).  A second, tiny kernel folds the
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
constexpr int kSub = 4;                        // 32-key subtiles per wave
constexpr int kWaveKeys = 32 * kSub;
constexpr int kBlockKeys = 4 * kWaveKeys;
static_assert(kBlockKeys == kRowstatBlockKeys, "the host plans with this block size");

__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

template <int D>
__global__ void __launch_bounds__(kThreads)
rowstat_kernel(const RowstatArgs a) {
  __shared__ float s_m[4][32], s_l[4][32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  // grid (key blocks, row tiles, layers of the group x query heads)
  const int kb = blockIdx.x, rt = blockIdx.y, li = blockIdx.z / a.n_q_heads, h = blockIdx.z % a.n_q_heads;
  const int hk = h / (a.n_q_heads / a.n_kv_heads);
  const u16* const q_rows = a.q_layer[li];
  const u16* const k_new = a.g.k_new[li];
  const u16* const k_cache = a.k_cache + (long long)li * a.g.kv_stride;
  float* const part_m = in_set_of(a.part_m, a.g, li);
  float* const part_l = in_set_of(a.part_l, a.g, li);
  const int c = a.c, n_cand = a.c + a.n_keys;
  const int key0 = kb * kBlockKeys + wave * kWaveKeys;

  // B operand: lane holds Q[32 rt + l32][16 s + 8 g .. + 7]
  bf16x8 qf[D / 16];
  {
    const int row = min(32 * rt + l32, a.n - 1);
    const u16* src = q_rows + ((size_t)row * a.n_q_heads + h) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * s));
  }
  // S^T subtile t: rows = keys key0 + 32 t + (0..31), columns = the 32 query rows
  float m = -INFINITY, l = 0.f;
  f32x16 s[kSub];
#pragma unroll
  for (int t = 0; t < kSub; ++t) {
    const int kv = min(key0 + 32 * t + l32, n_cand - 1);
    const u16* src = (kv < c ? k_cache + ((size_t)hk * a.budget + kv) * D
                             : k_new + ((size_t)(kv - c) * a.n_kv_heads + hk) * D) + 8 * g;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const bf16x8 ka = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * st));
      s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[st], s[t], 0, 0, 0);
    }
    // accumulator register r of lane group g is key 8 (r / 4) + 4 g + r % 4 of the subtile
    const int left = n_cand - (key0 + 32 * t) - 4 * g;      // keys of this lane's list that exist
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if (8 * (r >> 2) + (r & 3) >= left) s[t][r] = -INFINITY;
      m = fmaxf(m, s[t][r]);
    }
  }
  m = fmaxf(m, other_half(m));                 // lanes l and l + 32 hold the two halves of a row's keys
  const float m_use = m == -INFINITY ? 0.f : m;
#pragma unroll
  for (int t = 0; t < kSub; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) l += __builtin_amdgcn_exp2f((s[t][r] - m_use) * a.scale_log2);
  l += other_half(l);
  if (g == 0) { s_m[wave][l32] = m; s_l[wave][l32] = l; }
  __syncthreads();
  if (tid < 32) {
    float mm = s_m[0][tid];
#pragma unroll
    for (int w = 1; w < 4; ++w) mm = fmaxf(mm, s_m[w][tid]);
    const float mu = mm == -INFINITY ? 0.f : mm;
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) ll += s_l[w][tid] * __builtin_amdgcn_exp2f((s_m[w][tid] - mu) * a.scale_log2);
    const int row = 32 * rt + tid;
    if (row < a.n) {
      const size_t at = ((size_t)h * a.n + row) * a.n_kv_blocks + kb;
      part_m[at] = mm;
      part_l[at] = ll;
    }
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
  if (a.g.n_layers < 1 || a.g.n_layers > kMaxGroupLayers || (long long)a.g.n_layers * a.n_q_heads > 65535)
    return hipErrorInvalidValue;
  const dim3 grid(a.n_kv_blocks, (a.n + 31) / 32, a.g.n_layers * a.n_q_heads);
  if (head_dim == 128) hipLaunchKernelGGL(rowstat_kernel<128>, grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(rowstat_kernel<64>, grid, dim3(kThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int total = a.n_q_heads * a.n;
  hipLaunchKernelGGL(rowstat_fold_kernel, dim3((total + 255) / 256, a.g.n_layers), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace kvp

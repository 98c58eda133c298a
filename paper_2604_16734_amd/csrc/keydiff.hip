// Query-agnostic importance (the KeyDiff-style strategy of Sec. 3.2): the anchor
// is the mean of the candidate keys of a KV head, and a key scores the higher
// the less it resembles the anchor: score_j = -cos(k_j, mu).
//
// Pure streaming work, bound by HBM (every candidate key is read twice, the
// second time from L2): two small kernels.
//   keydiff_sum_kernel    column sums of the keys of one slice of one head
//                         (fp32; a lane adds its rows in ascending order, the
//                         lanes of a channel are added in ascending order, the
//                         slices likewise afterwards: a fixed order throughout)
//   keydiff_score_kernel  folds the slices into mu, then four lanes per key:
//                         dot(k, mu) and |k|^2 over a quarter of the channels
//                         each, added across the four lanes
// The scores go where the scoring pass of the query-aware strategy leaves its
// single partial, so the selection that follows is the same.
#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kThreads = 256;
constexpr int kSliceKeys = kKeydiffSliceKeys;   // keys per workgroup of the sum kernel

// candidate kv of KV head hk of layer li of the group: a cache entry or a block key
__device__ __forceinline__ const u16* key_row(const KeydiffArgs& a, int li, int hk, int kv, int D) {
  return kv < a.c ? a.k_cache + (long long)li * a.g.kv_stride + ((size_t)hk * a.budget + kv) * D
                  : a.g.k_new[li] + ((size_t)(kv - a.c) * a.n_kv_heads + hk) * D;
}

__device__ __forceinline__ void add8(float (&acc)[8], const uint4 w) {
  acc[0] += __uint_as_float(w.x << 16); acc[1] += __uint_as_float(w.x & 0xFFFF0000u);
  acc[2] += __uint_as_float(w.y << 16); acc[3] += __uint_as_float(w.y & 0xFFFF0000u);
  acc[4] += __uint_as_float(w.z << 16); acc[5] += __uint_as_float(w.z & 0xFFFF0000u);
  acc[6] += __uint_as_float(w.w << 16); acc[7] += __uint_as_float(w.w & 0xFFFF0000u);
}

// grid (slices, Hkv, layers of the group); thread t: the 16-byte piece t % (D / 8) of rows t / (D / 8) + k * kRowsAtOnce.
// All loads of a thread are independent and issued together: one trip to memory per workgroup.
template <int D>
__global__ void __launch_bounds__(kThreads)
keydiff_sum_kernel(const KeydiffArgs a) {
  constexpr int kPieces = D / 8, kRowsAtOnce = kThreads / kPieces, kLoads = kSliceKeys / kRowsAtOnce;
  __shared__ float s_part[kRowsAtOnce][D];
  const int slice = blockIdx.x, hk = blockIdx.y, li = blockIdx.z;
  const int piece = threadIdx.x % kPieces, rr = threadIdx.x / kPieces;
  const int n_cand = a.c + a.n_keys;
  const int k0 = slice * kSliceKeys;
  uint4 w[kLoads];
#pragma unroll
  for (int k = 0; k < kLoads; ++k) {
    const int kv = k0 + rr + k * kRowsAtOnce;
    w[k] = kv < n_cand ? *reinterpret_cast<const uint4*>(key_row(a, li, hk, kv, D) + 8 * piece) : uint4{0u, 0u, 0u, 0u};
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < kLoads; ++k) add8(acc, w[k]);          // rows in ascending order
#pragma unroll
  for (int e = 0; e < 8; ++e) s_part[rr][8 * piece + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < kRowsAtOnce; ++r) t += s_part[r][threadIdx.x];
    in_set_of(a.sums, a.g, li)[((size_t)hk * a.n_slices + slice) * D + threadIdx.x] = t;
  }
}

// grid (blocks of 64 keys, Hkv, layers of the group); four lanes per key, 16 keys per wave
template <int D>
__global__ void __launch_bounds__(kThreads)
keydiff_score_kernel(const KeydiffArgs a) {
  constexpr int kFold = kThreads / D;              // threads that share the fold of one channel
  __shared__ __align__(16) float s_mu[D];
  __shared__ float s_fold[kFold][D];
  __shared__ float s_mu2;
  const int hk = blockIdx.y, li = blockIdx.z;
  const float* const sums = in_set_of(a.sums, a.g, li);
  const int n_cand = a.c + a.n_keys;
  // this thread's piece of its key first: the load is on its way while the anchor is folded
  constexpr int kPer = D / 4;                      // channels per lane: a quarter of a key
  const int kv = blockIdx.x * a.keys_per_block + (threadIdx.x >> 2);
  const int quarter = threadIdx.x & 3;
  uint4 kw[kPer / 8];
  if (kv < n_cand) {
    const u16* row = key_row(a, li, hk, kv, D) + kPer * quarter;
#pragma unroll
    for (int i = 0; i < kPer / 8; ++i) kw[i] = *reinterpret_cast<const uint4*>(row + 8 * i);
  }
  {
    // slices folded in ascending order within a thread, threads in ascending order afterwards
    const int ch = threadIdx.x % D, part = threadIdx.x / D;
    const int per = (a.n_slices + kFold - 1) / kFold;
    const int s0 = part * per, s1 = min(a.n_slices, s0 + per);
    float t = 0.f;
#pragma unroll 8
    for (int s2 = s0; s2 < s1; ++s2) t += sums[((size_t)hk * a.n_slices + s2) * D + ch];
    s_fold[part][ch] = t;
  }
  __syncthreads();
  if (threadIdx.x < D) {
    float t = 0.f;
#pragma unroll
    for (int p = 0; p < kFold; ++p) t += s_fold[p][threadIdx.x];
    s_mu[threadIdx.x] = t / (float)n_cand;
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    float m2 = 0.f;
    for (int i = threadIdx.x; i < D; i += 64) m2 += s_mu[i] * s_mu[i];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) m2 += __shfl_xor(m2, off, 64);
    if (threadIdx.x == 0) s_mu2 = m2;
  }
  __syncthreads();
  float dot = 0.f, k2 = 0.f;
  if (kv < n_cand) {
#pragma unroll
    for (int i = 0; i < kPer / 8; ++i) {
      const unsigned ws[4] = {kw[i].x, kw[i].y, kw[i].z, kw[i].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float lo = __uint_as_float(ws[j] << 16), hi = __uint_as_float(ws[j] & 0xFFFF0000u);
        const float m0 = s_mu[kPer * quarter + 8 * i + 2 * j], m1 = s_mu[kPer * quarter + 8 * i + 2 * j + 1];
        dot = __builtin_fmaf(lo, m0, dot); dot = __builtin_fmaf(hi, m1, dot);
        k2 = __builtin_fmaf(lo, lo, k2); k2 = __builtin_fmaf(hi, hi, k2);
      }
    }
  }
  dot += __shfl_xor(dot, 1, 64); k2 += __shfl_xor(k2, 1, 64);
  dot += __shfl_xor(dot, 2, 64); k2 += __shfl_xor(k2, 2, 64);
  if (quarter == 0 && kv < n_cand)
    in_set_of(a.scores, a.g, li)[(size_t)hk * a.cand_stride + kv] = -dot / (sqrtf(k2) * sqrtf(s_mu2));
}

}  // namespace

hipError_t launch_keydiff(KeydiffArgs a, int head_dim, hipStream_t s) {
  const int n_cand = a.c + a.n_keys;
  a.n_slices = keydiff_slices(n_cand);
  a.keys_per_block = 64;
  if (a.g.n_layers < 1 || a.g.n_layers > kMaxGroupLayers) return hipErrorInvalidValue;
  const dim3 g1(a.n_slices, a.n_kv_heads, a.g.n_layers);
  const dim3 g2((n_cand + a.keys_per_block - 1) / a.keys_per_block, a.n_kv_heads, a.g.n_layers);
  if (head_dim == 128) {
    hipLaunchKernelGGL(keydiff_sum_kernel<128>, g1, dim3(kThreads), 0, s, a);
    hipLaunchKernelGGL(keydiff_score_kernel<128>, g2, dim3(kThreads), 0, s, a);
  } else {
    hipLaunchKernelGGL(keydiff_sum_kernel<64>, g1, dim3(kThreads), 0, s, a);
    hipLaunchKernelGGL(keydiff_score_kernel<64>, g2, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace kvp

// One decode step of one layer (Eq. 1 with a single query row per head, Sec. 2.1):
// the current token's queries attend over the layer's cache entries and over the
// keys and values of the tokens generated so far, the current one included (the
// "tail", which the caller keeps).
//
// Bound by HBM: every cached K and V row is read once per KV head and serves
// the G query heads of its group.  A single query row gives the block attention
// kernel nothing to spread, so the keys are spread instead: a workgroup takes
// 64 keys of one KV head at a time.  Its 256 threads fetch the 64 K rows and the
// 64 V rows with fully coalesced 16-byte loads, all in flight at once (a thread
// holds one 8-channel piece of 64 * 8 / 256 rows of each), so a tile costs one
// trip to memory.  Then
//   scores   each thread dots its pieces with the G queries; the pieces of a row
//            sit in neighbouring lanes and are added by butterflies;
//   softmax  one wave per query head: maximum and sum over the 64 keys, merged
//            into the running statistics of the workgroup (kept in LDS);
//   values   each thread scales its V pieces by the weights of its rows.
// After its last tile the workgroup adds the threads' pieces (butterflies, then
// LDS across waves) and leaves (max, sum, unnormalised output) per query head; a
// second small kernel folds the workgroups' partials in a fixed order and rounds
// once to bfloat16.
#include <mutex>

#include "kvp_internal.h"

// Scratch of kvp_decode_step_static (the entry point for callers that cannot allocate): the
// partial results of the step, KVP_STATIC_SCRATCH_BYTES per GPU, held until the process ends.
static __device__ __align__(256) float scratch[KVP_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace kvp {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kTile = kDecodeTile;   // keys per workgroup step
constexpr int kGroupLimit = kDecodeGroupLimit;   // query heads per KV head
constexpr int kMaxSplits = kDecodeMaxSplits;

__device__ __forceinline__ float bf16_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(unsigned x) { return __uint_as_float(x & 0xFFFF0000u); }
__device__ __forceinline__ void unpack8(const uint4 w, float (&x)[8]) {
  x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
  x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
}

// key j of the list: cache slot j for j < c, then the tail rows
__device__ __forceinline__ const u16* row_of(const u16* cache, const u16* tail, int hk, int n_kv_heads, int j, int c,
                                             int budget, int D) {
  return j < c ? cache + ((size_t)hk * budget + j) * D : tail + ((size_t)(j - c) * n_kv_heads + hk) * D;
}

// grid (n_splits, Hkv).  G = query heads per KV head, at most GM (the compiled bound, which
// sizes the register arrays; queries beyond G read as zero and their results are dropped).
template <int D, int GM>
__global__ void __launch_bounds__(kThreads)
decode_kernel(const DecodeArgs a) {
  constexpr int kPieces = D / 8;                 // 16-byte pieces per row
  constexpr int kRowsPerLoad = kThreads / kPieces;
  constexpr int kLoads = kTile / kRowsPerLoad;   // rows of a tile a thread holds a piece of
  __shared__ float s_s[GM][kTile];               // logits of the tile, then its weights
  __shared__ float s_m[GM], s_l[GM], s_f[GM];    // running maximum, running sum, rescale factor of this tile
  __shared__ float s_o[kWaves][GM][D];
  const int split = blockIdx.x, hk = blockIdx.y;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int piece = tid % kPieces, sub = tid / kPieces;
  const int n_keys = a.c + a.n_tail;
  const int n_tiles = (n_keys + kTile - 1) / kTile;

  if (tid < GM) { s_m[tid] = -INFINITY; s_l[tid] = 0.f; }
  float o[GM][8];
#pragma unroll
  for (int g = 0; g < GM; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) o[g][e] = 0.f;

  for (int tile = split; tile < n_tiles; tile += a.n_splits) {
    // ---- fetch: every K and V piece of the tile, all loads in flight together
    uint4 kw[kLoads], vw[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const int j = min(tile * kTile + kRowsPerLoad * i + sub, n_keys - 1);
      kw[i] = *reinterpret_cast<const uint4*>(row_of(a.k_cache, a.k_tail, hk, a.n_kv_heads, j, a.c, a.budget, D) + 8 * piece);
      vw[i] = *reinterpret_cast<const uint4*>(row_of(a.v_cache, a.v_tail, hk, a.n_kv_heads, j, a.c, a.budget, D) + 8 * piece);
    }
    // ---- scores
    float s[kLoads][GM];
#pragma unroll
    for (int i = 0; i < kLoads; ++i)
#pragma unroll
      for (int g = 0; g < GM; ++g) s[i][g] = 0.f;
#pragma unroll
    for (int g = 0; g < GM; ++g) {
      if (g < G) {
        float qx[8];
        unpack8(*reinterpret_cast<const uint4*>(a.q + ((size_t)hk * G + g) * D + 8 * piece), qx);
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
          float kx[8];
          unpack8(kw[i], kx);
#pragma unroll
          for (int e = 0; e < 8; ++e) s[i][g] = __builtin_fmaf(kx[e], qx[e], s[i][g]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < kLoads; ++i)
#pragma unroll
      for (int g = 0; g < GM; ++g) {
#pragma unroll
        for (int off = 1; off < kPieces; off <<= 1) s[i][g] += __shfl_xor(s[i][g], off, 64);
      }
    if (piece == 0) {
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const int r = kRowsPerLoad * i + sub;
        const bool live = tile * kTile + r < n_keys;
#pragma unroll
        for (int g = 0; g < GM; ++g) s_s[g][r] = live ? s[i][g] : -INFINITY;
      }
    }
    __syncthreads();
    // ---- softmax statistics: wave w takes query heads w, w + 4, ...
    for (int g = wave; g < G; g += kWaves) {
      const float x = s_s[g][lane];
      float mx = x;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float m_old = s_m[g];
      const float m_new = fmaxf(m_old, mx);            // finite: a tile holds at least one key
      const float p = __builtin_amdgcn_exp2f((x - m_new) * a.scale_log2);   // 0 for a key past the end
      float sum = p;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) sum += __shfl_xor(sum, off, 64);
      const float f = __builtin_amdgcn_exp2f((m_old - m_new) * a.scale_log2);   // 0 on the first tile
      s_s[g][lane] = p;
      if (lane == 0) { s_m[g] = m_new; s_l[g] = s_l[g] * f + sum; s_f[g] = f; }
    }
    __syncthreads();
    // ---- values
#pragma unroll
    for (int g = 0; g < GM; ++g) {
      if (g < G) {
        const float f = s_f[g];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] *= f;
      }
    }
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      float vx[8];
      unpack8(vw[i], vx);
      const int r = kRowsPerLoad * i + sub;
#pragma unroll
      for (int g = 0; g < GM; ++g) {
        if (g < G) {
          const float p = s_s[g][r];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[g][e] = __builtin_fmaf(p, vx[e], o[g][e]);
        }
      }
    }
    // the next tile's logits overwrite s_s only after its own barrier-free score phase:
    // every thread must be done reading the weights first
    __syncthreads();
  }
  // ---- add the pieces: rows of one wave by butterflies, waves through LDS
#pragma unroll
  for (int g = 0; g < GM; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int off = kPieces; off < 64; off <<= 1) o[g][e] += __shfl_xor(o[g][e], off, 64);
    }
  if (lane < kPieces) {
#pragma unroll
    for (int g = 0; g < GM; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) s_o[wave][g][8 * piece + e] = o[g][e];
  }
  __syncthreads();
  for (int i = tid; i < G * D; i += kThreads) {
    const int g = i / D, ch = i % D;
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) sum += s_o[w][g][ch];
    float* part = a.partial + (((size_t)hk * G + g) * a.n_splits + split) * (D + 2);
    part[ch] = sum;
    if (ch == 0) { part[D] = s_m[g]; part[D + 1] = s_l[g]; }
  }
}

// grid (Hq); kFoldLanes threads per channel, each folding every kFoldLanes-th partial, so
// that the loads of a thread do not depend on one another and a handful are in flight at once
constexpr int kFoldLanes = 4;
template <int D>
__global__ void __launch_bounds__(kFoldLanes * D)
decode_fold_kernel(const DecodeArgs a) {
  __shared__ float s_w[kMaxSplits];            // rescale factor of every partial
  __shared__ float s_mm[kMaxSplits];
  __shared__ float s_acc[kFoldLanes][D + 1];   // per lane group: channels, then the sum
  const int h = blockIdx.x, tid = threadIdx.x;
  const int ch = tid % D, grp = tid / D;
  const float* part = a.partial + (size_t)h * a.n_splits * (D + 2);
  if (tid < a.n_splits) s_mm[tid] = part[(size_t)tid * (D + 2) + D];
  __syncthreads();
  float mm = -INFINITY;
  for (int s = 0; s < a.n_splits; ++s) mm = fmaxf(mm, s_mm[s]);
  if (tid < a.n_splits) s_w[tid] = __builtin_amdgcn_exp2f((s_mm[tid] - mm) * a.scale_log2);
  __syncthreads();
  float oo = 0.f, ll = 0.f;
#pragma unroll 8
  for (int s = grp; s < a.n_splits; s += kFoldLanes) {
    oo = __builtin_fmaf(part[(size_t)s * (D + 2) + ch], s_w[s], oo);
    if (ch == 0) ll = __builtin_fmaf(part[(size_t)s * (D + 2) + D + 1], s_w[s], ll);
  }
  s_acc[grp][ch] = oo;
  if (ch == 0) s_acc[grp][D] = ll;
  __syncthreads();
  if (grp == 0) {
    float o_sum = 0.f, l_sum = 0.f;
#pragma unroll
    for (int g = 0; g < kFoldLanes; ++g) { o_sum += s_acc[g][ch]; l_sum += s_acc[g][D]; }
    const float r = o_sum / l_sum;
    unsigned u = __float_as_uint(r);          // round to nearest even
    u += 0x7FFFu + ((u >> 16) & 1u);
    a.out[(size_t)h * D + ch] = (u16)(u >> 16);
  }
}

template <int D>
hipError_t launch_for(const DecodeArgs& a, hipStream_t s) {
  const dim3 grid(a.n_splits, a.n_kv_heads);
  const int group = a.n_q_heads / a.n_kv_heads;
  if (group <= 4) hipLaunchKernelGGL((decode_kernel<D, 4>), grid, dim3(kThreads), 0, s, a);
  else if (group <= 8) hipLaunchKernelGGL((decode_kernel<D, 8>), grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL((decode_kernel<D, 16>), grid, dim3(kThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_fold_kernel<D>, dim3(a.n_q_heads), dim3(kFoldLanes * D), 0, s, a);
  return hipGetLastError();
}

// ---- kvp_decode_step_static: the partial results live in a file-scope device array instead of
// the cache's scratch set.  Every GPU the library runs on holds its own copy of the array, at its
// own address, until the process ends; host code never uses the array's name as an address, only
// the pointer hipGetSymbolAddress gave for the device in question.
constexpr size_t kStaticScratchFloats = sizeof(scratch) / sizeof(float);
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

}  // namespace

// Looks the array's address up for the CURRENT device (once per device) and returns it.
hipError_t decode_static_scratch(float** ptr, size_t* n_floats) {
  *ptr = nullptr;
  *n_floats = kStaticScratchFloats;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

hipError_t launch_decode(const DecodeArgs& a, int head_dim, hipStream_t s) {
  if (a.n_q_heads / a.n_kv_heads > kGroupLimit || a.n_splits < 1 || a.c + a.n_tail < 1) return hipErrorInvalidValue;
  return head_dim == 128 ? launch_for<128>(a, s) : launch_for<64>(a, s);
}

}  // namespace kvp

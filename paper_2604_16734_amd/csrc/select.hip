// Per-head selection of the M candidates to keep (Alg. 1 lines 8-11, with the
// rule of Sec. 3.2 that the lowest importance scores leave first), the slot
// assignment of the kept block tokens, and the grid-neighbour merge plan.
//
// One workgroup of 1024 threads per KV head; everything lives in LDS.
//   * order: 64-bit key = (score as order-preserving u32) << 32 | ~token, so
//     "higher score first, equal scores by lower token index" is "larger key
//     first" and all keys are distinct: the kept set is unique.
//   * the M-th largest key is found by an 8-bit radix select from the top
//     byte down (at most 8 passes, early exit once the chosen bin holds one
//     key).  Float scores share their top bits, so each histogram bin is
//     replicated 32 times, indexed by lane, to spread LDS atomic contention.
//   * block-wide prefix sums rank the free slots and the kept block tokens;
//     the k-th kept block token (ascending token index) gets the k-th free slot.
//   * merge plan: a token -> position hash table over the cached tokens (block
//     tokens map directly); every evicted visual candidate looks at its grid
//     neighbours and takes the kept one with the largest key; every kept
//     candidate then collects the sources that chose it.
#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxItems = KVP_MAX_CANDIDATES / kThreads;   // 8
constexpr int kCopies = 32;                                // histogram replicas
constexpr unsigned kNone16 = 0xFFFFu;

__device__ __forceinline__ unsigned order_bits(float x) {
  if (x == 0.f) x = 0.f;   // -0 and +0 rank equal
  const unsigned u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long make_key(unsigned ob, int tok) {
  return ((unsigned long long)ob << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)tok);
}

__device__ __forceinline__ unsigned hash_tok(int tok, unsigned mask) {
  unsigned x = (unsigned)tok * 0x9E3779B1u;
  x ^= x >> 15;
  return x & mask;
}

struct Lds {
  unsigned* sc;       // [cand_pad] order-preserving score bits
  int* tok;           // [cand_pad]
  unsigned short* free_list;  // [cand_pad]
  unsigned short* dst;        // [cand_pad]
  unsigned char* keep;        // [cand_pad]
  unsigned* shared;   // histogram (256 x 32 u32) or hash table (table_size u16), whichever is larger
};

__device__ __forceinline__ void table_insert(unsigned* words, unsigned mask, int tok, unsigned pos) {
  unsigned h = hash_tok(tok, mask);
  for (;;) {
    unsigned* word = words + (h >> 1);
    const unsigned sh = (h & 1u) * 16u;
    unsigned old = *word;
    while (((old >> sh) & 0xFFFFu) == kNone16) {
      const unsigned nv = (old & ~(0xFFFFu << sh)) | (pos << sh);
      const unsigned prev = atomicCAS(word, old, nv);
      if (prev == old) return;
      old = prev;
    }
    h = (h + 1) & mask;
  }
}

// position of token `tok` among the candidates, or -1
__device__ __forceinline__ int find_pos(const Lds& l, unsigned mask, int tok, int c, int n, int t0) {
  if (tok >= t0 && tok < t0 + n) return c + (tok - t0);
  unsigned h = hash_tok(tok, mask);
  for (;;) {
    const unsigned e = (l.shared[h >> 1] >> ((h & 1u) * 16u)) & 0xFFFFu;
    if (e == kNone16) return -1;
    if (l.tok[e] == tok) return (int)e;
    h = (h + 1) & mask;
  }
}

// grid neighbours of a visual token: left, right, up, down, previous plane, next plane
__device__ __forceinline__ int neighbours(const Seg* segs, int n_segs, int tok, int* out) {
  for (int s = 0; s < n_segs; ++s) {
    const Seg sg = segs[s];
    if (tok < sg.begin || tok >= sg.begin + sg.n) continue;
    if (sg.kind != KVP_VISUAL) return -1;
    const int u = tok - sg.begin;
    const int per = sg.gh * sg.gw;
    const int plane = u / per, rem = u % per;
    const int y = rem / sg.gw, x = rem % sg.gw;
    int k = 0;
    if (x > 0) out[k++] = tok - 1;
    if (x + 1 < sg.gw) out[k++] = tok + 1;
    if (y > 0) out[k++] = tok - sg.gw;
    if (y + 1 < sg.gh) out[k++] = tok + sg.gw;
    if (sg.temporal) {
      if (plane > 0) out[k++] = tok - per;
      if (plane + 1 < sg.planes) out[k++] = tok + per;
    }
    return k;
  }
  return -1;
}

__global__ void __launch_bounds__(kThreads)
select_kernel(const SelectArgs a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ unsigned long long s_threshold;
  __shared__ unsigned s_digit, s_want, s_bin_count, s_n_dst;
  __shared__ unsigned s_bin[256];
  __shared__ unsigned s_wave_tot[kWaves];
  __shared__ Seg s_segs[KVP_MAX_SEGMENTS];

  const int hk = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = a.c, n = a.n, n_cand = c + n, budget = a.budget;
  const int items = a.items;
  const int cand_pad = items * kThreads;

  Lds l;
  {
    unsigned char* p = lds_raw;
    l.sc = reinterpret_cast<unsigned*>(p); p += (size_t)cand_pad * 4;
    l.tok = reinterpret_cast<int*>(p); p += (size_t)cand_pad * 4;
    l.free_list = reinterpret_cast<unsigned short*>(p); p += (size_t)cand_pad * 2;
    l.dst = reinterpret_cast<unsigned short*>(p); p += (size_t)cand_pad * 2;
    l.keep = p; p += (size_t)cand_pad;
    l.shared = reinterpret_cast<unsigned*>(p);
  }

  // ---- scores (sum of the partial column sums in a fixed order) and token indices
  float* scores = a.scores + (size_t)hk * a.cand_stride;
  for (int p = tid; p < n_cand; p += kThreads) {
    float sc;
    if (a.score_override) {
      sc = a.score_override[(size_t)hk * n_cand + p];
    } else {
      sc = 0.f;
      const float* part = a.partial + (size_t)hk * a.n_partials * a.cand_stride + p;
      for (int j = 0; j < a.n_partials; ++j) sc += part[(size_t)j * a.cand_stride];
    }
    scores[p] = sc;
    l.sc[p] = order_bits(sc);
    l.tok[p] = p < c ? a.token_idx[(size_t)hk * budget + p] : a.t0 + (p - c);
  }
  if (tid < a.n_segs) s_segs[tid] = a.segs[tid];
  if (tid == 0) s_n_dst = 0;
  __syncthreads();

  // ---- own candidates, blocked: thread t owns positions [t * items, (t + 1) * items)
  unsigned long long key[kMaxItems];
  bool valid[kMaxItems];
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    valid[i] = i < items && p < n_cand;
    key[i] = valid[i] ? make_key(l.sc[p], l.tok[p]) : 0ull;
  }

  // ---- radix select of the budget-th largest key
  unsigned long long prefix = 0;
  unsigned want = (unsigned)budget;
  bool found_unique = false;
  for (int pass = 0; pass < 8 && !found_unique; ++pass) {
    const int shift = 56 - 8 * pass;
    for (int i = tid; i < 256 * kCopies; i += kThreads) l.shared[i] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) {
      if (!valid[i]) continue;
      const bool match = pass == 0 || (key[i] >> (shift + 8)) == (prefix >> (shift + 8));
      if (match) atomicAdd(&l.shared[(unsigned)((key[i] >> shift) & 255u) * kCopies + (lane & (kCopies - 1))], 1u);
    }
    __syncthreads();
    {  // bin totals: 4 threads per bin, 8 replicas each
      const int bin = tid >> 2, part = tid & 3;
      unsigned t = 0;
#pragma unroll
      for (int k = 0; k < kCopies / 4; ++k) t += l.shared[bin * kCopies + part * (kCopies / 4) + k];
      t += __shfl_xor(t, 1, 64);
      t += __shfl_xor(t, 2, 64);
      if (part == 0) s_bin[bin] = t;
    }
    __syncthreads();
    if (wave == 0) {
      // lane L owns bins 4L .. 4L+3; suffix sums count the keys in higher bins
      unsigned cnt[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) cnt[b] = s_bin[4 * lane + b];
      const unsigned mine = cnt[0] + cnt[1] + cnt[2] + cnt[3];
      unsigned suf = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned v = __shfl_down(suf, off, 64);
        if (lane + off < 64) suf += v;
      }
      unsigned above = suf - mine;
#pragma unroll
      for (int b = 3; b >= 0; --b) {
        if (above < want && want <= above + cnt[b]) {
          s_digit = 4 * lane + b;
          s_want = want - above;
          s_bin_count = cnt[b];
        }
        above += cnt[b];
      }
    }
    __syncthreads();
    prefix |= (unsigned long long)s_digit << shift;
    want = s_want;
    if (s_bin_count == 1) {
      // the bin holds exactly the key we are after
#pragma unroll
      for (int i = 0; i < kMaxItems; ++i)
        if (valid[i] && (key[i] >> shift) == (prefix >> shift)) s_threshold = key[i];
      found_unique = true;
    }
    __syncthreads();
  }
  const unsigned long long threshold = found_unique ? s_threshold : prefix;

  // ---- keep flags; rank free slots and kept block tokens
  bool keep[kMaxItems];
  unsigned n_free = 0, n_new = 0;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    keep[i] = valid[i] && key[i] >= threshold;
    if (valid[i]) {
      l.keep[p] = keep[i];
      l.dst[p] = kNone16;
      a.keep[(size_t)hk * a.cand_stride + p] = keep[i];
      a.dst[(size_t)hk * a.cand_stride + p] = -1;
      if (p < budget && (p >= c || !keep[i])) ++n_free;
      if (p >= c && keep[i]) ++n_new;
    }
  }
  unsigned packed = n_free | (n_new << 16);
  unsigned incl = packed;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned v = __shfl_up(incl, off, 64);
    if (lane >= off) incl += v;
  }
  if (lane == 63) s_wave_tot[wave] = incl;
  __syncthreads();
  unsigned base = incl - packed;
  unsigned total = 0;
  for (int w2 = 0; w2 < kWaves; ++w2) {
    const unsigned t = s_wave_tot[w2];
    if (w2 < wave) base += t;
    total += t;
  }
  unsigned base_free = base & 0xFFFFu, base_new = base >> 16;
  const unsigned total_new = total >> 16;
  int rank_new[kMaxItems];
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    rank_new[i] = -1;
    if (valid[i]) {
      if (p < budget && (p >= c || !keep[i])) l.free_list[base_free++] = (unsigned short)p;
      if (p >= c && keep[i]) rank_new[i] = (int)base_new++;
    }
  }
  __syncthreads();
  MoveEntry* moves = a.moves + (size_t)hk * a.chunk_max;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    if (rank_new[i] >= 0) {
      MoveEntry e;
      e.pos = tid * items + i;
      e.slot = l.free_list[rank_new[i]];
      e.stage = -1;
      e.pad = 0;
      moves[rank_new[i]] = e;
    }
  }
  if (tid == 0) a.counts[hk].n_moves = (int)total_new;

  if (!a.merge) {
    if (tid == 0) a.counts[hk].n_dst = 0;
    return;
  }

  // ---- merge plan
  const unsigned mask = (unsigned)a.table_size - 1u;
  for (int i = tid; i < a.table_size / 2; i += kThreads) l.shared[i] = 0xFFFFFFFFu;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    if (valid[i] && p < c) table_insert(l.shared, mask, l.tok[p], (unsigned)p);
  }
  __syncthreads();
  // every evicted visual candidate picks its best kept neighbour
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    if (!valid[i] || keep[i]) continue;
    const int p = tid * items + i;
    int nb[kNeighbours];
    const int k = neighbours(s_segs, a.n_segs, l.tok[p], nb);
    unsigned long long best_key = 0;
    int best = -1;
    for (int j = 0; j < k; ++j) {
      const int r = find_pos(l, mask, nb[j], c, n, a.t0);
      if (r < 0 || !l.keep[r]) continue;
      const unsigned long long kr = make_key(l.sc[r], l.tok[r]);
      if (best < 0 || kr > best_key) { best = r; best_key = kr; }
    }
    if (best >= 0) {
      l.dst[p] = (unsigned short)best;
      a.dst[(size_t)hk * a.cand_stride + p] = best;
    }
  }
  __syncthreads();
  // every kept visual candidate collects the sources that chose it
  DstEntry* dsts = a.dsts + (size_t)hk * a.chunk_max;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    if (!valid[i] || !keep[i]) continue;
    const int p = tid * items + i;
    int nb[kNeighbours];
    const int k = neighbours(s_segs, a.n_segs, l.tok[p], nb);
    DstEntry e;
    e.pos = p;
    e.n_src = 0;
#pragma unroll
    for (int j = 0; j < kNeighbours; ++j) e.src[j] = -1;
    for (int j = 0; j < k; ++j) {
      const int r = find_pos(l, mask, nb[j], c, n, a.t0);
      if (r >= 0 && !l.keep[r] && l.dst[r] == (unsigned short)p) e.src[e.n_src++] = r;
    }
    if (e.n_src > 0) {
      const unsigned j = atomicAdd(&s_n_dst, 1u);
      dsts[j] = e;
      if (rank_new[i] >= 0) moves[rank_new[i]].stage = (int)j;
    }
  }
  __syncthreads();
  if (tid == 0) a.counts[hk].n_dst = (int)s_n_dst;
}

}  // namespace

size_t select_lds_bytes(int /*n_cand*/, int items, int table_size) {
  const size_t cand_pad = (size_t)items * kThreads;
  size_t shared = (size_t)256 * kCopies * 4;
  const size_t table = (size_t)table_size * 2;
  if (table > shared) shared = table;
  return cand_pad * (4 + 4 + 2 + 2 + 1) + shared;
}

hipError_t launch_select(const SelectArgs& a, int n_kv_heads, hipStream_t s) {
  const size_t lds = select_lds_bytes(a.c + a.n, a.items, a.table_size);
  static size_t attr_bytes = 0;
  if (lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  hipLaunchKernelGGL(select_kernel, dim3(n_kv_heads), dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

}  // namespace kvp

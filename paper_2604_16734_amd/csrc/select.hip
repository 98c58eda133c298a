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
//     neighbours, takes the kept one with the largest key and counts itself in
//     at that destination; a prefix sum numbers the destinations that were
//     chosen, and the sources then write themselves into their destination's
//     entry (the merge kernel sorts each entry, so the order they arrive in
//     does not matter).
#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kThreads = kSelectThreads;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxItemsAny = KVP_MAX_CANDIDATES / kThreads;   // 8
constexpr int kCopies = kSelectCopies;                     // histogram replicas
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
  unsigned* sc;       // [cand_pad] order-preserving score bits; later the ordinal of a merge destination
  int* tok;           // [cand_pad]
  unsigned char* keep;        // [cand_pad]; reused as per-destination fill counters
  // one region, two lives: the radix histogram (256 x kCopies u32), then the compaction lists
  unsigned* hist;
  unsigned short* evicted;    // [cand_pad] positions of the evicted candidates, ascending
  unsigned short* free_dst;   // [cand_pad] free slots by rank; then the destination of the e-th evicted
  unsigned* cnt;              // [cand_pad / 4] one byte per candidate: sources that chose it
  unsigned* table;    // token -> position of the cached tokens: table_size u16, open addressing
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

__device__ __forceinline__ unsigned table_entry(const Lds& l, unsigned h) {
  return (l.table[h >> 1] >> ((h & 1u) * 16u)) & 0xFFFFu;
}

// position of cached token `tok`, or -1, when its home slot `h` holds `e` and that is not it
__device__ __forceinline__ int probe_on(const Lds& l, unsigned mask, int tok, unsigned h, unsigned e) {
  for (;;) {
    if (e == kNone16) return -1;
    if (l.tok[e] == tok) return (int)e;
    h = (h + 1) & mask;
    e = table_entry(l, h);
  }
}

struct SegL {          // a prefix segment in LDS, with reciprocals for the coordinate split
  int begin, n, kind, gh, gw, planes, temporal, per;
  float inv_per, inv_gw;
};

// u / d and u % d for 0 <= u < 2^24, d >= 1, with a float reciprocal and one fix-up step
__device__ __forceinline__ void div_mod(int u, int d, float inv_d, int& q, int& r) {
  q = (int)((float)u * inv_d);
  r = u - q * d;
  if (r < 0) { r += d; --q; }
  if (r >= d) { r -= d; ++q; }
}

// grid neighbours of a visual token: left, right, up, down, previous plane, next plane;
// out[j] = -1 where there is none.  Returns false for a text token.
__device__ __forceinline__ bool neighbours(const SegL* segs, int n_segs, int tok, int (&out)[kNeighbours]) {
#pragma unroll
  for (int j = 0; j < kNeighbours; ++j) out[j] = -1;
  for (int s = 0; s < n_segs; ++s) {
    const int begin = segs[s].begin;
    if (tok < begin || tok >= begin + segs[s].n) continue;
    const SegL sg = segs[s];
    if (sg.kind != KVP_VISUAL) return false;
    int plane, rem, y, x;
    div_mod(tok - sg.begin, sg.per, sg.inv_per, plane, rem);
    div_mod(rem, sg.gw, sg.inv_gw, y, x);
    if (x > 0) out[0] = tok - 1;
    if (x + 1 < sg.gw) out[1] = tok + 1;
    if (y > 0) out[2] = tok - sg.gw;
    if (y + 1 < sg.gh) out[3] = tok + sg.gw;
    if (sg.temporal) {
      if (plane > 0) out[4] = tok - sg.per;
      if (plane + 1 < sg.planes) out[5] = tok + sg.per;
    }
    return true;
  }
  return false;
}

// kMaxItems: candidates a thread can own (4 covers up to 4096 candidates and halves the registers
// of the batched loads; 8 covers the limit)
template <int kMaxItems>
__global__ void __launch_bounds__(kThreads)
select_kernel(const SelectArgs a_first) {
  // grid (KV heads, layers of the group): this workgroup's layer
  SelectArgs a = a_first;
  {
    const int li = blockIdx.y;
    a.partial = in_set_of(a.partial, a.g, li);
    a.scores = in_set_of(a.scores, a.g, li);
    a.keep = in_set_of(a.keep, a.g, li);
    a.dst = in_set_of(a.dst, a.g, li);
    a.counts = in_set_of(a.counts, a.g, li);
    a.moves = in_set_of(a.moves, a.g, li);
    a.dsts = in_set_of(a.dsts, a.g, li);
    a.token_idx += (long long)li * a.g.meta_stride;
  }
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ unsigned long long s_threshold;
  __shared__ unsigned s_digit, s_want, s_bin_count;
  __shared__ unsigned s_bin[256];
  __shared__ unsigned s_wave_tot[kWaves], s_wave_ev[kWaves];
  __shared__ unsigned s_wave_diff[2 * kWaves];
  __shared__ SegL s_segs[KVP_MAX_SEGMENTS];

  const int hk = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = a.c, n = a.n, n_cand = c + n, budget = a.budget;
  const int items = a.items;
  const int cand_pad = items * kThreads;
  const unsigned mask = (unsigned)a.table_size - 1u;

  Lds l;
  {
    unsigned char* p = lds_raw;
    l.sc = reinterpret_cast<unsigned*>(p); p += (size_t)cand_pad * 4;
    l.tok = reinterpret_cast<int*>(p); p += (size_t)cand_pad * 4;
    l.keep = p; p += (size_t)cand_pad;
    l.hist = reinterpret_cast<unsigned*>(p);
    l.evicted = reinterpret_cast<unsigned short*>(p);
    l.free_dst = reinterpret_cast<unsigned short*>(p + (size_t)cand_pad * 2);
    l.cnt = reinterpret_cast<unsigned*>(p + (size_t)cand_pad * 4);
    p += select_region_bytes(cand_pad);
    l.table = reinterpret_cast<unsigned*>(p);
  }

  // ---- token indices, the token -> position table of the cached ones, and the scores (sum of
  // the partial column sums in a fixed order).  Thread t takes candidates t, t + 1024, ...; the
  // loads of a batch of partials of all of them are in flight together, and the first batch is
  // on its way while the table is filled.
  float* scores = a.scores + (size_t)hk * a.cand_stride;
  {
    int tokv[kMaxItems];
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) {
      const int p = tid + i * kThreads;
      tokv[i] = 0;
      if (i < items && p < n_cand) tokv[i] = p < c ? a.token_idx[(size_t)hk * budget + p] : a.t0 + (p - c);
    }
    float acc[kMaxItems];
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) acc[i] = 0.f;
    const float* part = a.partial + (size_t)hk * a.n_partials * a.cand_stride;
    constexpr int kBatch = kMaxItems <= 4 ? 8 : 4;             // partials fetched together
    const int n_rounds = a.score_override ? 0 : (a.n_partials + kBatch - 1) / kBatch;
    float v[kBatch][kMaxItems];
    auto fetch = [&](int round) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int j = min(kBatch * round + u, a.n_partials - 1);      // a surplus slot repeats the last partial
#pragma unroll
        for (int i = 0; i < kMaxItems; ++i)
          if (i < items) v[u][i] = part[(size_t)j * a.cand_stride + min(tid + i * kThreads, n_cand - 1)];
      }
    };
    auto add = [&](int round) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
#pragma unroll
        for (int i = 0; i < kMaxItems; ++i)
          if (i < items && kBatch * round + u < a.n_partials) acc[i] += v[u][i];
    };
    if (n_rounds > 0) fetch(0);
    if (a.score_override) {
#pragma unroll
      for (int i = 0; i < kMaxItems; ++i) {
        const int p = tid + i * kThreads;
        if (i < items && p < n_cand) acc[i] = a.score_override[(size_t)hk * n_cand + p];
      }
    }
    for (int i = tid; i < a.table_size / 2; i += kThreads) l.table[i] = 0xFFFFFFFFu;
    if (tid < a.n_segs) {
      const Seg g = a.segs[tid];
      SegL sl;
      sl.begin = g.begin; sl.n = g.n; sl.kind = g.kind; sl.gh = g.gh; sl.gw = g.gw;
      sl.planes = g.planes; sl.temporal = g.temporal;
      sl.per = g.gh * g.gw;
      sl.inv_per = sl.per > 0 ? 1.f / (float)sl.per : 0.f;
      sl.inv_gw = g.gw > 0 ? 1.f / (float)g.gw : 0.f;
      s_segs[tid] = sl;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) {
      const int p = tid + i * kThreads;
      if (i < items && p < n_cand) {
        l.tok[p] = tokv[i];
        if (a.merge && p < c) table_insert(l.table, mask, tokv[i], (unsigned)p);
      }
    }
    for (int round = 0; round < n_rounds; ++round) {
      add(round);
      if (round + 1 < n_rounds) fetch(round + 1);
    }
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) {
      const int p = tid + i * kThreads;
      if (i < items && p < n_cand) {
        scores[p] = acc[i];
        l.sc[p] = order_bits(acc[i]);
      }
    }
  }
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

  // ---- radix select of the budget-th largest key, eight bits at a time, starting at the highest
  // bit in which any two keys differ (float scores share their sign and most of the exponent,
  // and digits spent on a common prefix would tell nothing apart)
  // (the bits in which some key differs from candidate 0 are the bits in which any two differ)
  const unsigned long long ref = make_key(l.sc[0], l.tok[0]);
  unsigned diff_hi = 0, diff_lo = 0;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i)
    if (valid[i]) {
      diff_hi |= (unsigned)((key[i] ^ ref) >> 32);
      diff_lo |= (unsigned)(key[i] ^ ref);
    }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    diff_hi |= __shfl_xor(diff_hi, off, 64);
    diff_lo |= __shfl_xor(diff_lo, off, 64);
  }
  if (lane == 0) { s_wave_diff[2 * wave] = diff_hi; s_wave_diff[2 * wave + 1] = diff_lo; }
  __syncthreads();
#pragma unroll
  for (int w2 = 0; w2 < kWaves; ++w2) { diff_hi |= s_wave_diff[2 * w2]; diff_lo |= s_wave_diff[2 * w2 + 1]; }
  const unsigned long long diff = ((unsigned long long)diff_hi << 32) | diff_lo;
  int top = diff ? 64 - __builtin_clzll(diff) : 0;             // bits [0, top) are still undecided
  unsigned long long prefix = top >= 64 ? 0ull : (ref >> top) << top;
  unsigned want = (unsigned)budget;
  bool found_unique = false;
  while (top > 0 && !found_unique) {
    const int width = top < 8 ? top : 8;
    const int lo = top - width;
    for (int i = tid; i < 256 * kCopies; i += kThreads) l.hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) {
      if (!valid[i]) continue;
      const bool match = top >= 64 || (key[i] >> top) == (prefix >> top);
      if (match)
        atomicAdd(&l.hist[(unsigned)((key[i] >> lo) & ((1u << width) - 1u)) * kCopies + (lane & (kCopies - 1))], 1u);
    }
    __syncthreads();
    {  // bin totals: 4 threads per bin, 8 replicas each, taken in an order that keeps the 64 lanes
       // of a wave on 64 different banks (bin b, replica r is word 32 b + r)
      const int bin = tid >> 2, part = tid & 3;
      unsigned t = 0;
#pragma unroll
      for (int k = 0; k < kCopies / 4; ++k)
        t += l.hist[bin * kCopies + ((4 * (bin >> 1) + part + 4 * k) & (kCopies - 1))];
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
    prefix |= (unsigned long long)s_digit << lo;
    want = s_want;
    if (s_bin_count == 1) {
      // the bin holds exactly the key we are after
#pragma unroll
      for (int i = 0; i < kMaxItems; ++i)
        if (valid[i] && (key[i] >> lo) == (prefix >> lo)) s_threshold = key[i];
      found_unique = true;
    }
    __syncthreads();
    top = lo;
  }
  const unsigned long long threshold = found_unique ? s_threshold : prefix;

  // ---- keep flags; rank the free slots, the kept block tokens and the evicted candidates.
  // (The histogram is dead from here on: its memory now holds the lists.)
  bool keep[kMaxItems];
  unsigned n_free = 0, n_new = 0, n_ev = 0;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    keep[i] = valid[i] && key[i] >= threshold;
    if (valid[i]) {
      l.keep[p] = keep[i];
      a.keep[(size_t)hk * a.cand_stride + p] = keep[i];
      a.dst[(size_t)hk * a.cand_stride + p] = -1;
      if (p < budget && (p >= c || !keep[i])) ++n_free;
      if (p >= c && keep[i]) ++n_new;
      if (!keep[i]) ++n_ev;
    }
  }
  unsigned packed = n_free | (n_new << 16);
  unsigned incl = packed, incl_ev = n_ev;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned v = __shfl_up(incl, off, 64);
    const unsigned ve = __shfl_up(incl_ev, off, 64);
    if (lane >= off) { incl += v; incl_ev += ve; }
  }
  if (lane == 63) { s_wave_tot[wave] = incl; s_wave_ev[wave] = incl_ev; }
  for (int i = tid; i < cand_pad / 4; i += kThreads) l.cnt[i] = 0u;
  __syncthreads();
  unsigned base = incl - packed, base_ev = incl_ev - n_ev;
  unsigned total = 0, total_ev = 0;
  for (int w2 = 0; w2 < kWaves; ++w2) {
    const unsigned t = s_wave_tot[w2], te = s_wave_ev[w2];
    if (w2 < wave) { base += t; base_ev += te; }
    total += t; total_ev += te;
  }
  unsigned base_free = base & 0xFFFFu, base_new = base >> 16;
  const unsigned total_new = total >> 16;
  int rank_new[kMaxItems];
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    rank_new[i] = -1;
    if (valid[i]) {
      if (p < budget && (p >= c || !keep[i])) l.free_dst[base_free++] = (unsigned short)p;
      if (p >= c && keep[i]) rank_new[i] = (int)base_new++;
      if (!keep[i]) l.evicted[base_ev++] = (unsigned short)p;
    }
  }
  __syncthreads();
  MoveEntry* moves = a.moves + (size_t)hk * a.chunk_max;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    if (rank_new[i] >= 0) {
      MoveEntry e;
      e.pos = tid * items + i;
      e.slot = l.free_dst[rank_new[i]];
      e.stage = -1;
      e.pad = 0;
      moves[rank_new[i]] = e;
    }
  }
  if (tid == 0) {
    a.counts[hk].n_moves = (int)total_new;
    atomicAdd(&a.totals[KVP_T_EVICTING_HEADS], 1ull);
    atomicAdd(&a.totals[KVP_T_MOVED_ROWS], (unsigned long long)total_new);
  }

  if (!a.merge) {
    if (tid == 0) a.counts[hk].n_dst = 0;
    return;
  }
  __syncthreads();                       // the free list has been consumed: it now takes destinations

  // ---- merge plan: the e-th evicted candidate (thread e, e + 1024, ...) picks its best kept
  // grid neighbour and counts itself in there
  for (unsigned e = tid; e < total_ev; e += kThreads) {
    const int p = l.evicted[e];
    const int tokp = l.tok[p];
    int best = -1;
    int nb[kNeighbours];
    if (neighbours(s_segs, a.n_segs, tokp, nb)) {
      // first probe of all neighbours at once; a token of the block sits at a known position
      unsigned h[kNeighbours], ent[kNeighbours];
      bool in_block[kNeighbours];
#pragma unroll
      for (int j = 0; j < kNeighbours; ++j) {
        in_block[j] = nb[j] >= a.t0 && nb[j] < a.t0 + n;
        h[j] = hash_tok(nb[j] < 0 ? 0 : nb[j], mask);
        ent[j] = table_entry(l, h[j]);
      }
      int r[kNeighbours];
      int tk[kNeighbours];
#pragma unroll
      for (int j = 0; j < kNeighbours; ++j) {
        r[j] = in_block[j] ? c + (nb[j] - a.t0) : (ent[j] == kNone16 ? -1 : (int)ent[j]);
        tk[j] = r[j] >= 0 ? l.tok[r[j]] : -1;
      }
#pragma unroll
      for (int j = 0; j < kNeighbours; ++j) {
        if (nb[j] < 0) r[j] = -1;
        else if (!in_block[j] && r[j] >= 0 && tk[j] != nb[j]) r[j] = probe_on(l, mask, nb[j], h[j], ent[j]);
      }
      unsigned kp[kNeighbours], sc[kNeighbours];
#pragma unroll
      for (int j = 0; j < kNeighbours; ++j) {
        kp[j] = r[j] >= 0 ? l.keep[r[j]] : 0u;
        sc[j] = r[j] >= 0 ? l.sc[r[j]] : 0u;
      }
      unsigned long long best_key = 0;
#pragma unroll
      for (int j = 0; j < kNeighbours; ++j) {
        if (!kp[j]) continue;
        const unsigned long long kr = make_key(sc[j], nb[j]);
        if (best < 0 || kr > best_key) { best = r[j]; best_key = kr; }
      }
    }
    l.free_dst[e] = best >= 0 ? (unsigned short)best : (unsigned short)kNone16;
    if (best >= 0) {
      a.dst[(size_t)hk * a.cand_stride + p] = best;
      atomicAdd(&l.cnt[best >> 2], 1u << (8 * (best & 3)));
    }
  }
  __syncthreads();
  // number the destinations that were chosen, in candidate order; the ordinal of a destination
  // goes where its score bits were (nobody reads those any more)
  unsigned* fill = reinterpret_cast<unsigned*>(l.keep);     // the keep flags have been consumed
  unsigned n_mine = 0;
  unsigned cnt_of[kMaxItems];
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    const int p = tid * items + i;
    cnt_of[i] = valid[i] ? (l.cnt[p >> 2] >> (8 * (p & 3))) & 0xFFu : 0u;
    n_mine += cnt_of[i] ? 1u : 0u;
  }
  unsigned incl2 = n_mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned v = __shfl_up(incl2, off, 64);
    if (lane >= off) incl2 += v;
  }
  if (lane == 63) s_wave_tot[wave] = incl2;
  for (int i = tid; i < cand_pad / 4; i += kThreads) fill[i] = 0u;
  __syncthreads();
  unsigned ord = incl2 - n_mine, n_dst = 0;
  for (int w2 = 0; w2 < kWaves; ++w2) {
    const unsigned t = s_wave_tot[w2];
    if (w2 < wave) ord += t;
    n_dst += t;
  }
  DstEntry* dsts = a.dsts + (size_t)hk * a.chunk_max;
#pragma unroll
  for (int i = 0; i < kMaxItems; ++i) {
    if (!cnt_of[i]) continue;
    const int p = tid * items + i;
    l.sc[p] = ord;
    dsts[ord].pos = p;
    dsts[ord].n_src = (int)cnt_of[i];
    if (rank_new[i] >= 0) moves[rank_new[i]].stage = (int)ord;
    ++ord;
  }
  __syncthreads();
  // every source writes itself into its destination's entry
  unsigned n_src_mine = 0;
  for (unsigned e = tid; e < total_ev; e += kThreads) {
    const unsigned d = l.free_dst[e];
    if (d == kNone16) continue;
    const unsigned old = atomicAdd(&fill[d >> 2], 1u << (8 * (d & 3)));
    const unsigned k = (old >> (8 * (d & 3))) & 0xFFu;
    dsts[l.sc[d]].src[k] = l.evicted[e];
    ++n_src_mine;
  }
  if (tid == 0) a.counts[hk].n_dst = (int)n_dst;
  // running totals for the benchmark's byte counts (integer atomics: the order does not matter)
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) n_src_mine += __shfl_xor(n_src_mine, off, 64);
  if (lane == 0 && n_src_mine) atomicAdd(&a.totals[KVP_T_MERGE_SOURCES], (unsigned long long)n_src_mine);
  if (tid == 0) atomicAdd(&a.totals[KVP_T_MERGE_DESTINATIONS], (unsigned long long)n_dst);
}

}  // namespace

hipError_t launch_select(const SelectArgs& a, int n_kv_heads, hipStream_t s) {
  const size_t lds = select_lds_bytes(a.c + a.n, a.items, a.table_size);
  const dim3 grid(n_kv_heads, a.g.n_layers);
  if (a.items <= 4) hipLaunchKernelGGL(select_kernel<4>, grid, dim3(kThreads), lds, s, a);
  else hipLaunchKernelGGL(select_kernel<kMaxItemsAny>, grid, dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

// Allows both kernels the dynamic LDS of the largest head they can be given (the attribute
// belongs to the function on the current device: called at cache creation).
hipError_t prepare_select() {
  const int sizes[2] = {4, kMaxItemsAny};
  const void* fns[2] = {reinterpret_cast<const void*>(select_kernel<4>),
                        reinterpret_cast<const void*>(select_kernel<kMaxItemsAny>)};
  for (int i = 0; i < 2; ++i) {
    int ts = 2;
    while (ts < 2 * sizes[i] * kThreads) ts <<= 1;
    const size_t lds = select_lds_bytes(sizes[i] * kThreads, sizes[i], ts);
    hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace kvp

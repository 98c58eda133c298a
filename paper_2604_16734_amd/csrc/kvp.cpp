// Host side of libkvp: validation, the per-layer state machine of Alg. 1,
// carving of the caller's device buffer, and kernel sequencing.  No device
// memory is allocated and no stream is synchronised anywhere in this file
// except kvp_profile_read, which waits for its own events.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kvp_internal.h"

using namespace kvp;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  // persistent, per layer strides in bytes
  size_t k_off, v_off, idx_off, w_off;
  size_t kv_layer_bytes, meta_layer_elems;
  size_t persistent_bytes;
  // global
  size_t segs_off, totals_off;
  // scratch, per set
  size_t set_off, set_bytes;
  size_t lse_off, partial_off, scores_off, keep_off, dst_off, counts_off, moves_off, dsts_off,
      stage_k_off, stage_v_off, stage_w_off;
  int cand_stride, max_partials, n_sets;
  size_t total_bytes;
};

bool valid_config(const kvp_config* c) {
  if (!c) return false;
  if (c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return false;
  if (c->n_q_heads % c->n_kv_heads) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->budget < 1 || c->chunk_max < 1) return false;
  if ((long long)c->budget + c->chunk_max > KVP_MAX_CANDIDATES) return false;
  if (c->merge != 0 && c->merge != 1) return false;
  if (c->scratch_sets < 0 || c->scratch_sets > c->n_layers) return false;
  if (c->flags & ~KVP_FLAG_DRY_RUN) return false;
  if (!(c->softmax_scale >= 0.f) || std::isinf(c->softmax_scale)) return false;
  return true;
}

Layout make_layout(const kvp_config& c) {
  Layout L{};
  const size_t L_ = c.n_layers, H = c.n_kv_heads, M = c.budget, D = c.head_dim, B = c.chunk_max;
  L.kv_layer_bytes = H * M * D * 2;
  L.meta_layer_elems = H * M;
  size_t off = 0;
  L.k_off = off; off = align_up(off + L_ * L.kv_layer_bytes);
  L.v_off = off; off = align_up(off + L_ * L.kv_layer_bytes);
  L.idx_off = off; off = align_up(off + L_ * L.meta_layer_elems * 4);
  L.w_off = off; off = align_up(off + L_ * L.meta_layer_elems * 4);
  L.persistent_bytes = off;
  L.segs_off = off; off = align_up(off + KVP_MAX_SEGMENTS * sizeof(Seg));
  L.totals_off = off; off = align_up(off + KVP_T_COUNT * sizeof(unsigned long long));
  L.n_sets = c.scratch_sets ? c.scratch_sets : 1;
  L.cand_stride = (int)((M + B + 63) / 64 * 64);
  // partial score arrays per KV head: what the separate column-sum kernel needs, or, when the
  // attention kernel leaves the scores itself, one per workgroup of a KV head (query heads of the
  // group x row tiles), as long as that stays modest
  L.max_partials = colsum_max_partials(c.n_q_heads / c.n_kv_heads, c.chunk_max);
  {
    const int fused = attention_max_partials(c.n_q_heads / c.n_kv_heads, c.n_q_heads, c.chunk_max);
    if (fused <= kMaxFusedPartials && fused > L.max_partials) L.max_partials = fused;
  }
  size_t s = 0;
  L.lse_off = s; s = align_up(s + (size_t)c.n_q_heads * B * 4);
  // The partial score arrays and the staging rows of the compaction share their memory: the
  // selection has read the last partial before the merge kernel (launched after it, on the same
  // stream) writes the first staged row, and the next block's scoring pass writes partials only
  // after the move kernel has read the last one (the scratch set is the layer's until then).
  const size_t partial_bytes = align_up(H * L.max_partials * L.cand_stride * 4);
  const size_t stage_bytes = align_up(H * B * D * 2);
  L.partial_off = s;
  L.stage_k_off = s;
  L.stage_v_off = s + stage_bytes;
  s += partial_bytes > 2 * stage_bytes ? partial_bytes : 2 * stage_bytes;
  L.scores_off = s; s = align_up(s + H * L.cand_stride * 4);
  L.keep_off = s; s = align_up(s + H * L.cand_stride);
  L.dst_off = s; s = align_up(s + H * L.cand_stride * 4);
  L.counts_off = s; s = align_up(s + H * sizeof(HeadCounts));
  L.moves_off = s; s = align_up(s + H * B * sizeof(MoveEntry));
  L.dsts_off = s; s = align_up(s + H * B * sizeof(DstEntry));
  L.stage_w_off = s; s = align_up(s + H * B * 4);
  L.set_bytes = s;
  L.set_off = off;
  off += L.set_bytes * L.n_sets;
  L.total_bytes = off;
  return L;
}

enum LayerState { READY = 0, PENDING = 1 };
enum { kScoreOwn = 0, kScoreProxy = 1, kScoreKeydiff = 2 };

struct Layer {
  int state = READY;
  int count = 0;        // entries per head
  int next_token = 0;
  // the pending block
  int t0 = 0, n = 0;
  int n_partials = 0;   // partial score arrays the scoring pass of the pending block left
  const u16* k = nullptr;
  const u16* v = nullptr;
  // a scoring pass (proxy queries, or the keys alone) that is still to be launched:
  // kvp_prefill_block launches it for a group of layers at once; a layer in this state cannot be
  // compacted yet
  const u16* q_obs = nullptr;
  int n_obs = 0;
  int unscored = 0;     // 0, kScoreProxy or kScoreKeydiff
  // last block, for kvp_debug_last
  int last_cand = 0;
  bool has_last = false;
};

struct ProfEvent {
  int kind;
  int layers;           // layers the launch covered
  hipEvent_t start, stop;
};

}  // namespace

struct kvp_cache {
  kvp_config cfg;
  Layout lay;
  unsigned char* base;
  int n_tokens;                       // prefix length from the segments
  std::vector<Seg> segs;
  std::vector<Layer> layers;
  std::vector<int> set_owner;         // layer holding each scratch set, or -1
  float scale;
  bool dry;
  int attn_shape = -1;                // kvp_set_attention_shape; < 0: chosen per launch
  bool fused_scores = true;           // kvp_set_score_sweep: scores out of the attention launch itself
  bool deferred_scoring = false;      // kvp_set_deferred_scoring: proxy and key-only scoring at the compaction
  float* static_scratch = nullptr;    // the file-scope scratch array on this cache's device
  size_t static_scratch_floats = 0;
  bool profiling = false;
  std::vector<ProfEvent> events;      // recorded, not yet read
  std::vector<hipEvent_t> pool;       // idle events
  // kvp_prefill_block with two streams works in groups of layers.  Per group, in a ring:
  // "attention and scoring of the group enqueued" (main stream) and "its compactions
  // enqueued" (side stream).  Groups are numbered from 0 for the life of the cache.
  std::vector<hipEvent_t> attended, compacted;
  std::vector<long long> set_last_group;   // per scratch set: the last group that used it, or -1
  long long n_groups = 0;                  // groups enqueued so far
  long long waited_group = -1;             // the main stream already waits for groups up to this one

  u16* k_cache(int l) const { return reinterpret_cast<u16*>(base + lay.k_off + (size_t)l * lay.kv_layer_bytes); }
  u16* v_cache(int l) const { return reinterpret_cast<u16*>(base + lay.v_off + (size_t)l * lay.kv_layer_bytes); }
  int32_t* idx(int l) const { return reinterpret_cast<int32_t*>(base + lay.idx_off) + (size_t)l * lay.meta_layer_elems; }
  float* weight(int l) const { return reinterpret_cast<float*>(base + lay.w_off) + (size_t)l * lay.meta_layer_elems; }
  Seg* dev_segs() const { return reinterpret_cast<Seg*>(base + lay.segs_off); }
  unsigned long long* totals() const { return reinterpret_cast<unsigned long long*>(base + lay.totals_off); }
  unsigned char* set(int l) const { return base + lay.set_off + (size_t)(l % lay.n_sets) * lay.set_bytes; }
};

namespace {

// Runs one launch, bracketed by events when profiling.
template <class F>
int launch(kvp_cache* c, int kind, int layers, hipStream_t s, F&& f) {
  if (c->dry) return KVP_OK;
  ProfEvent pe{kind, layers, nullptr, nullptr};
  if (c->profiling) {
    for (hipEvent_t* e : {&pe.start, &pe.stop}) {
      if (!c->pool.empty()) {
        *e = c->pool.back();
        c->pool.pop_back();
      } else if (hipEventCreate(e) != hipSuccess) {
        return KVP_EDEVICE;
      }
    }
    if (hipEventRecord(pe.start, s) != hipSuccess) return KVP_EDEVICE;
  }
  if (f() != hipSuccess) return KVP_EDEVICE;
  if (c->profiling) {
    if (hipEventRecord(pe.stop, s) != hipSuccess) return KVP_EDEVICE;
    c->events.push_back(pe);
  }
  return KVP_OK;
}

// `count` consecutive layers from `first` on, each with its pending block, as the kernels see them
LayerGroup make_group(const kvp_cache* c, int first, int count) {
  const Layout& lay = c->lay;
  LayerGroup g{};
  g.n_layers = count;
  g.first_set = first % lay.n_sets;
  g.n_sets = lay.n_sets;
  g.set_stride = (long long)lay.set_bytes;
  g.kv_stride = (long long)(lay.kv_layer_bytes / 2);
  g.meta_stride = (long long)lay.meta_layer_elems;
  for (int i = 0; i < count; ++i) {
    g.k_new[i] = c->layers[first + i].k;
    g.v_new[i] = c->layers[first + i].v;
  }
  return g;
}

// Alg. 1 lines 7-11 for `count` consecutive layers that hold the same block (same entries in the
// cache, same tokens pending): one launch of each compaction kernel for all of them.
int run_compact(kvp_cache* c, int first, int count, const float* scores_override, hipStream_t s) {
  Layer& L = c->layers[first];
  const kvp_config& cfg = c->cfg;
  const Layout& lay = c->lay;
  unsigned char* set = c->set(first);
  const int cnt = L.count, n = L.n, M = cfg.budget;

  const LayerGroup g = make_group(c, first, count);

  CompactArgs ca{};
  ca.g = g;
  ca.k_cache = c->k_cache(first);
  ca.v_cache = c->v_cache(first);
  ca.token_idx = c->idx(first);
  ca.weight = c->weight(first);
  ca.counts = reinterpret_cast<HeadCounts*>(set + lay.counts_off);
  ca.moves = reinterpret_cast<MoveEntry*>(set + lay.moves_off);
  ca.dsts = reinterpret_cast<DstEntry*>(set + lay.dsts_off);
  ca.stage_k = reinterpret_cast<u16*>(set + lay.stage_k_off);
  ca.stage_v = reinterpret_cast<u16*>(set + lay.stage_v_off);
  ca.stage_w = reinterpret_cast<float*>(set + lay.stage_w_off);
  ca.c = cnt; ca.n = n; ca.t0 = L.t0; ca.budget = M;
  ca.n_kv_heads = cfg.n_kv_heads; ca.head_dim = cfg.head_dim; ca.chunk_max = cfg.chunk_max;
  const int rpb = rows_per_compact_block(cfg.head_dim);

  if (cnt + n <= M) {
    // Alg. 1 line 8 is false: plain append
    ca.identity = 1;
    ca.blocks_per_head = (n + rpb - 1) / rpb;
    return launch(c, KVP_K_MOVE, count, s, [&] { return launch_move(ca, s); });
  }

  SelectArgs sa{};
  sa.g = g;
  sa.partial = scores_override ? nullptr : reinterpret_cast<const float*>(set + lay.partial_off);
  sa.score_override = scores_override;
  sa.scores = reinterpret_cast<float*>(set + lay.scores_off);
  sa.keep = set + lay.keep_off;
  sa.dst = reinterpret_cast<int32_t*>(set + lay.dst_off);
  sa.token_idx = c->idx(first);
  sa.counts = reinterpret_cast<HeadCounts*>(set + lay.counts_off);
  sa.moves = reinterpret_cast<MoveEntry*>(set + lay.moves_off);
  sa.dsts = reinterpret_cast<DstEntry*>(set + lay.dsts_off);
  sa.segs = c->dev_segs();
  sa.totals = c->totals();
  sa.n_segs = (int)c->segs.size();
  sa.c = cnt; sa.n = n; sa.t0 = L.t0; sa.budget = M;
  sa.cand_stride = lay.cand_stride; sa.chunk_max = cfg.chunk_max;
  sa.n_partials = L.n_partials;
  sa.merge = cfg.merge;
  sa.items = (cnt + n + 1023) / 1024;
  int ts = 2;
  while (ts < 2 * (cnt + n)) ts <<= 1;
  sa.table_size = ts;
  int rc = launch(c, KVP_K_SELECT, count, s, [&] { return launch_select(sa, cfg.n_kv_heads, s); });
  if (rc) return rc;

  ca.identity = 0;
  const int n_evict = cnt + n - M;
  if (cfg.merge) {
    const int max_dst = n_evict < cfg.chunk_max ? n_evict : cfg.chunk_max;
    ca.blocks_per_head = (max_dst + rpb - 1) / rpb;
    rc = launch(c, KVP_K_MERGE, count, s, [&] { return launch_merge(ca, s); });
    if (rc) return rc;
  }
  ca.blocks_per_head = (n + rpb - 1) / rpb;
  return launch(c, KVP_K_MOVE, count, s, [&] { return launch_move(ca, s); });
}

// kvp_compact for layers [first, first + count): one group launch when they hold the same block,
// one layer at a time otherwise.  Every layer must be PENDING.
int compact_layers(kvp_cache* c, int first, int count, const float* scores_override, hipStream_t s) {
  // (a scoring pass that was put off is the caller's to launch first: score_deferred_layers)
  for (int i = 0; i < count; ++i)
    if (c->layers[first + i].state != PENDING || c->layers[first + i].unscored != 0) return KVP_ESTATE;
  bool same = count <= kMaxGroupLayers && (scores_override == nullptr || count == 1);
  const Layer& A = c->layers[first];
  for (int i = 1; i < count && same; ++i) {
    const Layer& B = c->layers[first + i];
    same = B.count == A.count && B.n == A.n && B.t0 == A.t0 && B.n_partials == A.n_partials;
  }
  if (!same) {
    if (scores_override != nullptr) return KVP_EINVAL;
    for (int i = 0; i < count; ++i) {
      const int rc = compact_layers(c, first + i, 1, nullptr, s);
      if (rc) return rc;
    }
    return KVP_OK;
  }
  const int rc = run_compact(c, first, count, scores_override, s);
  if (rc) return rc;
  for (int i = 0; i < count; ++i) {
    Layer& L = c->layers[first + i];
    L.count = L.count + L.n <= c->cfg.budget ? L.count + L.n : c->cfg.budget;
    L.state = READY;
    L.next_token = L.t0 + L.n;
    c->set_owner[(first + i) % c->lay.n_sets] = -1;
  }
  return KVP_OK;
}

}  // namespace

extern "C" {

const char* kvp_strerror(int code) {
  switch (code) {
    case KVP_OK: return "ok";
    case KVP_EINVAL: return "invalid argument";
    case KVP_ESTATE: return "call out of order for this layer";
    case KVP_ENOMEM: return "buffer too small or out of host memory";
    case KVP_EDEVICE: return "HIP runtime error";
    default: return "unknown kvp error";
  }
}

const char* kvp_kernel_name(int32_t kind) {
  switch (kind) {
    case KVP_K_ATTENTION: return "attention";
    case KVP_K_COLSUM: return "colsum";
    case KVP_K_SELECT: return "select";
    case KVP_K_MERGE: return "merge";
    case KVP_K_MOVE: return "move";
    case KVP_K_ROWSTAT: return "rowstat";
    case KVP_K_KEYDIFF: return "keydiff";
    case KVP_K_DECODE: return "decode";
    default: return "?";
  }
}

size_t kvp_cache_bytes(const kvp_config* cfg) {
  if (!valid_config(cfg)) return 0;
  return make_layout(*cfg).total_bytes;
}

size_t kvp_persistent_bytes(const kvp_config* cfg) {
  if (!valid_config(cfg)) return 0;
  return make_layout(*cfg).persistent_bytes;
}

int kvp_init_cache(const kvp_config* cfg, const kvp_segment* segs, int32_t n_segs, void* device_buf,
                   size_t device_bytes, void* stream, kvp_cache** out) {
  if (!out) return KVP_EINVAL;
  *out = nullptr;
  if (!valid_config(cfg) || !segs || n_segs < 1 || n_segs > KVP_MAX_SEGMENTS) return KVP_EINVAL;
  const bool dry = cfg->flags & KVP_FLAG_DRY_RUN;
  if (!dry && (!device_buf || (reinterpret_cast<uintptr_t>(device_buf) % kAlign))) return KVP_EINVAL;
  long long t = 0;
  for (int i = 0; i < n_segs; ++i) {
    const kvp_segment& s = segs[i];
    if (s.token_begin != t || s.n_tokens < 1) return KVP_EINVAL;
    if (s.kind == KVP_VISUAL) {
      if (s.grid_h < 1 || s.grid_w < 1 || s.n_planes < 1) return KVP_EINVAL;
      if ((long long)s.grid_h * s.grid_w * s.n_planes != s.n_tokens) return KVP_EINVAL;
      if (s.temporal != 0 && s.temporal != 1) return KVP_EINVAL;
    } else if (s.kind != KVP_TEXT) {
      return KVP_EINVAL;
    }
    t += s.n_tokens;
    if (t > (1 << 24)) return KVP_EINVAL;   // the select kernel splits token indices with fp32 reciprocals
  }
  const Layout lay = make_layout(*cfg);
  if (!dry && device_bytes < lay.total_bytes) return KVP_ENOMEM;

  kvp_cache* c = new (std::nothrow) kvp_cache();
  if (!c) return KVP_ENOMEM;
  c->cfg = *cfg;
  c->lay = lay;
  c->base = static_cast<unsigned char*>(device_buf);
  c->n_tokens = (int)t;
  c->dry = dry;
  c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.f / std::sqrt((float)cfg->head_dim);
  for (int i = 0; i < n_segs; ++i)
    c->segs.push_back(Seg{segs[i].token_begin, segs[i].n_tokens, segs[i].kind, segs[i].grid_h,
                          segs[i].grid_w, segs[i].n_planes, segs[i].temporal});
  c->layers.resize(cfg->n_layers);
  c->set_owner.assign(lay.n_sets, -1);
  if (!dry) {
    const size_t slots = (size_t)cfg->n_layers * lay.meta_layer_elems;
    hipError_t e = prepare_attention();
    if (e == hipSuccess) e = prepare_select();
    if (e == hipSuccess) e = decode_static_scratch(&c->static_scratch, &c->static_scratch_floats);
    if (e == hipSuccess)
      e = launch_init(c->idx(0), c->weight(0), slots, c->segs.data(), n_segs, c->dev_segs(),
                      c->totals(), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
      delete c;
      return KVP_EDEVICE;
    }
  }
  *out = c;
  return KVP_OK;
}

namespace {


// A short list of proxy queries would leave the attention kernel with a handful of workgroups that
// each walk all keys: rowstat_kernel spreads the keys instead.  Its per-block partials borrow the
// memory of the column-sum partials, which the scoring pass only writes afterwards.
static bool proxy_by_rowstat(const kvp_cache* c, int n_cand, int n_obs) {
  const kvp_config& cfg = c->cfg;
  const Layout& lay = c->lay;
  const int n_kb = rowstat_key_blocks(n_cand);
  const size_t need = (size_t)cfg.n_q_heads * n_obs * n_kb * 2 * sizeof(float);
  const size_t have = (size_t)cfg.n_kv_heads * lay.max_partials * lay.cand_stride * sizeof(float);
  return (long long)n_obs * cfg.n_q_heads < 128 * 64 && need <= have;
}

// The scoring kernels' arguments for `layer` (the first layer of a group, or the only one) with
// `count` entries in its cache and a block of `n_tokens`; the group and the queries are the caller's.
static RowstatArgs rowstat_args(kvp_cache* c, int layer, int count, int n_tokens, int n_obs) {
  const kvp_config& cfg = c->cfg;
  const Layout& lay = c->lay;
  unsigned char* set = c->set(layer);
  RowstatArgs ra{};
  ra.k_cache = c->k_cache(layer);
  ra.lse2 = reinterpret_cast<float*>(set + lay.lse_off);
  ra.part_m = reinterpret_cast<float*>(set + lay.partial_off);
  ra.part_l = ra.part_m + (size_t)cfg.n_q_heads * n_obs * rowstat_key_blocks(count + n_tokens);
  ra.n = n_obs; ra.c = count; ra.n_keys = n_tokens;
  ra.n_q_heads = cfg.n_q_heads; ra.n_kv_heads = cfg.n_kv_heads;
  ra.budget = cfg.budget; ra.lse_stride = cfg.chunk_max;
  ra.scale_log2 = c->scale * 1.4426950408889634f;
  return ra;
}

static ColsumArgs colsum_args(kvp_cache* c, int layer, int count, int n_tokens, int n_rows, int shift) {
  const kvp_config& cfg = c->cfg;
  const Layout& lay = c->lay;
  unsigned char* set = c->set(layer);
  ColsumArgs cs{};
  cs.k_cache = c->k_cache(layer);
  cs.lse2 = reinterpret_cast<float*>(set + lay.lse_off);
  cs.partial = reinterpret_cast<float*>(set + lay.partial_off);
  cs.n = n_rows; cs.c = count;
  cs.n_keys = n_tokens; cs.shift = shift;
  cs.n_q_heads = cfg.n_q_heads; cs.n_kv_heads = cfg.n_kv_heads;
  cs.budget = cfg.budget; cs.lse_stride = cfg.chunk_max; cs.cand_stride = lay.cand_stride;
  cs.scale_log2 = c->scale * 1.4426950408889634f;
  plan_colsum(cs, cfg.head_dim);
  return cs;
}

static KeydiffArgs keydiff_args(kvp_cache* c, int layer, int count, int n_tokens) {
  const kvp_config& cfg = c->cfg;
  const Layout& lay = c->lay;
  KeydiffArgs ka{};
  ka.k_cache = c->k_cache(layer);
  ka.scores = reinterpret_cast<float*>(c->set(layer) + lay.partial_off);          // the one "partial"
  ka.sums = ka.scores + (size_t)cfg.n_kv_heads * lay.cand_stride;
  ka.c = count; ka.n_keys = n_tokens; ka.n_kv_heads = cfg.n_kv_heads;
  ka.budget = cfg.budget; ka.cand_stride = lay.cand_stride;
  return ka;
}

// The scoring pass (proxy queries: row statistics, then column sums; or the keys alone) for `count`
// consecutive layers whose blocks went through prefill_impl with `defer`: one launch of each
// kernel for up to kMaxGroupLayers layers in the same state, else layer by layer.
static int score_deferred_layers(kvp_cache* c, int first, int count, hipStream_t s) {
  const kvp_config& cfg = c->cfg;
  for (int done = 0; done < count;) {
    Layer& A = c->layers[first + done];
    if (A.unscored == 0) {          // scored inside prefill_impl already (nothing to evict, or a long list)
      ++done;
      continue;
    }
    int m = 1;
    while (done + m < count && m < kMaxGroupLayers) {
      const Layer& B = c->layers[first + done + m];
      if (B.unscored != A.unscored || B.count != A.count || B.n != A.n || B.t0 != A.t0 || B.n_obs != A.n_obs) break;
      ++m;
    }
    const int layer = first + done;
    const LayerGroup g = make_group(c, layer, m);
    int n_partials = 1;
    if (A.unscored == kScoreKeydiff) {
      KeydiffArgs ka = keydiff_args(c, layer, A.count, A.n);
      ka.g = g;
      const int rc = launch(c, KVP_K_KEYDIFF, m, s, [&] { return launch_keydiff(ka, cfg.head_dim, s); });
      if (rc) return rc;
    } else {
      RowstatArgs ra = rowstat_args(c, layer, A.count, A.n, A.n_obs);
      ColsumArgs cs = colsum_args(c, layer, A.count, A.n, A.n_obs, A.n);
      ra.g = g;
      cs.g = g;
      for (int i = 0; i < m; ++i) ra.q_layer[i] = cs.q_layer[i] = c->layers[layer + i].q_obs;
      int rc = launch(c, KVP_K_ROWSTAT, m, s, [&] { return launch_rowstat(ra, cfg.head_dim, s); });
      if (rc) return rc;
      rc = launch(c, KVP_K_COLSUM, m, s, [&] { return launch_colsum(cs, cfg.head_dim, s); });
      if (rc) return rc;
      n_partials = cs.n_partials;
    }
    for (int i = 0; i < m; ++i) {
      Layer& L = c->layers[layer + i];
      L.n_partials = n_partials;
      L.unscored = 0;
    }
    done += m;
  }
  return KVP_OK;
}

// kvp_prefill_chunk and its variants: attention for the block; the scores come from the block's
// own queries, from proxy queries, or from the keys alone
// `defer`: leave the scoring pass of proxy queries or of the keys alone to score_deferred_layers,
// which launches it for a group of layers at once (kvp_prefill_block); the layer is PENDING and
// `unscored` until then.
static int prefill_impl(kvp_cache* c, int32_t layer, int32_t token_begin, int32_t n_tokens, const void* q,
                 const void* k, const void* v, void* out, const void* q_obs, int32_t n_obs, int mode,
                 void* stream, bool defer = false) {
  const bool proxy = mode == kScoreProxy;
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  if (n_tokens < 1 || n_tokens > c->cfg.chunk_max) return KVP_EINVAL;
  if (!c->dry && (!q || !k || !v || !out)) return KVP_EINVAL;
  if (proxy && (n_obs < 1 || n_obs > c->cfg.chunk_max || (!c->dry && !q_obs))) return KVP_EINVAL;
  Layer& L = c->layers[layer];
  if (L.state != READY) return KVP_ESTATE;
  if (token_begin != L.next_token) return KVP_ESTATE;
  if ((long long)token_begin + n_tokens > c->n_tokens) return KVP_EINVAL;
  const int set_i = layer % c->lay.n_sets;
  if (c->set_owner[set_i] != -1) return KVP_ESTATE;   // another layer's block is still pending there

  const kvp_config& cfg = c->cfg;
  const Layout& lay = c->lay;
  unsigned char* set = c->set(layer);
  hipStream_t s = static_cast<hipStream_t>(stream);

  AttnArgs aa{};
  aa.q = static_cast<const u16*>(q);
  aa.k_new = static_cast<const u16*>(k);
  aa.v_new = static_cast<const u16*>(v);
  aa.out = static_cast<u16*>(out);
  aa.k_cache = c->k_cache(layer);
  aa.v_cache = c->v_cache(layer);
  aa.lse2 = reinterpret_cast<float*>(set + lay.lse_off);
  aa.n = n_tokens; aa.c = L.count;
  aa.n_keys = n_tokens; aa.shift = 0;
  aa.n_q_heads = cfg.n_q_heads; aa.n_kv_heads = cfg.n_kv_heads;
  aa.budget = cfg.budget; aa.lse_stride = cfg.chunk_max;
  aa.scale_log2 = c->scale * 1.4426950408889634f;
  plan_attention(aa, cfg.head_dim, c->attn_shape);
  // The scores decide an eviction; a block that fits into the cache as it is needs none.  Scored
  // by its own queries, the block's attention launch leaves the column sums itself (a second
  // sweep inside the kernel), one partial array per workgroup of a KV head.
  const bool evicts = L.count + n_tokens > cfg.budget;
  const int own_partials = (cfg.n_q_heads / cfg.n_kv_heads) * aa.n_row_tiles;
  const bool fused = evicts && mode == kScoreOwn && own_partials <= lay.max_partials && c->fused_scores;
  if (fused) {
    aa.partial = reinterpret_cast<float*>(set + lay.partial_off);
    aa.n_partials = own_partials;
    aa.cand_stride = lay.cand_stride;
  }
  int rc = launch(c, KVP_K_ATTENTION, 1, s, [&] { return launch_attention(aa, cfg.head_dim, s); });
  if (rc) return rc;
  aa.partial = nullptr;
  L.unscored = 0;
  if (fused) {
    L.n_partials = own_partials;
  } else if (evicts) {
    // the block as the scoring kernels see it: this layer alone
    LayerGroup one{};
    one.n_layers = 1;
    one.first_set = set_i; one.n_sets = lay.n_sets;
    one.k_new[0] = aa.k_new; one.v_new[0] = aa.v_new;
    bool deferred = false;
    if (proxy) {
      // row statistics of the proxy queries over all candidates (nothing hidden, no output);
      // they replace the block's own in the scratch set
      aa.q = static_cast<const u16*>(q_obs);
      aa.out = nullptr;
      aa.n = n_obs;
      aa.shift = n_tokens;
      if (proxy_by_rowstat(c, L.count + n_tokens, n_obs)) {
        if (defer) {
          deferred = true;
        } else {
          RowstatArgs ra = rowstat_args(c, layer, L.count, n_tokens, n_obs);
          ra.g = one;
          ra.q_layer[0] = aa.q;
          rc = launch(c, KVP_K_ROWSTAT, 1, s, [&] { return launch_rowstat(ra, cfg.head_dim, s); });
        }
      } else {
        plan_attention(aa, cfg.head_dim, c->attn_shape);
        rc = launch(c, KVP_K_ATTENTION, 1, s, [&] { return launch_attention(aa, cfg.head_dim, s); });
      }
      if (rc) return rc;
    }
    if (deferred) {
      L.q_obs = aa.q;
      L.n_obs = n_obs;
      L.unscored = kScoreProxy;
    } else if (mode == kScoreKeydiff && defer) {
      L.unscored = kScoreKeydiff;
    } else if (mode == kScoreKeydiff) {
      KeydiffArgs ka = keydiff_args(c, layer, L.count, n_tokens);
      ka.g = one;
      rc = launch(c, KVP_K_KEYDIFF, 1, s, [&] { return launch_keydiff(ka, cfg.head_dim, s); });
      if (rc) return rc;
      L.n_partials = 1;
    } else {
      ColsumArgs cs = colsum_args(c, layer, L.count, n_tokens, aa.n, aa.shift);
      cs.g = one;
      cs.q_layer[0] = aa.q;
      rc = launch(c, KVP_K_COLSUM, 1, s, [&] { return launch_colsum(cs, cfg.head_dim, s); });
      if (rc) return rc;
      L.n_partials = cs.n_partials;
    }
  }

  L.state = PENDING;
  L.t0 = token_begin; L.n = n_tokens;
  L.k = aa.k_new; L.v = aa.v_new;
  L.last_cand = L.count + n_tokens;
  L.has_last = true;
  c->set_owner[set_i] = layer;
  return KVP_OK;
}

}  // namespace

int kvp_prefill_chunk(kvp_cache* c, int32_t layer, int32_t token_begin, int32_t n_tokens, const void* q,
                      const void* k, const void* v, void* out, void* stream) {
  return prefill_impl(c, layer, token_begin, n_tokens, q, k, v, out, nullptr, 0, kScoreOwn, stream);
}

int kvp_prefill_chunk_proxy(kvp_cache* c, int32_t layer, int32_t token_begin, int32_t n_tokens, const void* q,
                            const void* k, const void* v, void* out, const void* q_obs, int32_t n_obs,
                            void* stream) {
  return prefill_impl(c, layer, token_begin, n_tokens, q, k, v, out, q_obs, n_obs, kScoreProxy, stream,
                      c && c->deferred_scoring);
}

int kvp_prefill_chunk_keydiff(kvp_cache* c, int32_t layer, int32_t token_begin, int32_t n_tokens, const void* q,
                              const void* k, const void* v, void* out, void* stream) {
  return prefill_impl(c, layer, token_begin, n_tokens, q, k, v, out, nullptr, 0, kScoreKeydiff, stream,
                      c && c->deferred_scoring);
}

int kvp_compact(kvp_cache* c, int32_t layer, const float* scores_override, void* stream) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  if (c->layers[layer].state != PENDING) return KVP_ESTATE;
  // a scoring pass that was put off (kvp_set_deferred_scoring) comes first
  const int rc = score_deferred_layers(c, layer, 1, static_cast<hipStream_t>(stream));
  if (rc) return rc;
  return compact_layers(c, layer, 1, scores_override, static_cast<hipStream_t>(stream));
}

int kvp_compact_layers(kvp_cache* c, int32_t first_layer, int32_t n_layers, void* stream) {
  if (!c || first_layer < 0 || n_layers < 1 || n_layers > c->cfg.n_layers || first_layer > c->cfg.n_layers - n_layers)
    return KVP_EINVAL;
  for (int i = 0; i < n_layers; ++i)
    if (c->layers[first_layer + i].state != PENDING) return KVP_ESTATE;
  {
    // scoring passes that were put off (kvp_set_deferred_scoring) come first, grouped like the rest
    const int rc = score_deferred_layers(c, first_layer, n_layers, static_cast<hipStream_t>(stream));
    if (rc) return rc;
  }
  for (int done = 0; done < n_layers; done += kMaxGroupLayers) {
    const int count = n_layers - done < kMaxGroupLayers ? n_layers - done : kMaxGroupLayers;
    const int rc = compact_layers(c, first_layer + done, count, nullptr, static_cast<hipStream_t>(stream));
    if (rc) return rc;
  }
  return KVP_OK;
}

int kvp_prefill_block(kvp_cache* c, int32_t token_begin, int32_t n_tokens, const void* const* q,
                      const void* const* k, const void* const* v, void* const* out, int32_t scoring,
                      const void* const* q_obs, int32_t n_obs, void* stream, void* side_stream) {
  if (!c || !q || !k || !v || !out) return KVP_EINVAL;
  if (scoring < KVP_SCORE_OWN || scoring > KVP_SCORE_KEYDIFF) return KVP_EINVAL;
  if (scoring == KVP_SCORE_PROXY && !q_obs) return KVP_EINVAL;
  const int n_layers = c->cfg.n_layers, n_sets = c->lay.n_sets;
  const bool two = side_stream != nullptr && side_stream != stream && !c->dry;
  if (two && n_sets < 2) return KVP_EINVAL;      // compaction beside the next layer needs a second scratch set
  hipStream_t main = static_cast<hipStream_t>(stream), side = static_cast<hipStream_t>(side_stream);
  // With two streams the layers go in groups of half the scratch sets: the attention and
  // scoring of a group on the main stream, one event, its compactions on the side stream, one
  // event.  The streams so exchange two events per group instead of two per layer (a record
  // costs the main stream about 4 us, a wait about 6 us), and while the side stream compacts
  // one group the main stream has the other half of the sets for the next.
  // On one stream a group may take every scratch set: its compactions then go out as one launch
  // of each kernel for the whole group.
  const int group = std::min(kMaxGroupLayers, two ? std::max(1, n_sets / 2) : n_sets);
  const size_t ring = (size_t)n_sets + 2;        // more than the groups any set can still refer to
  if (two && c->attended.empty()) {
    for (std::vector<hipEvent_t>* list : {&c->attended, &c->compacted})
      for (size_t i = 0; i < ring; ++i) {
        hipEvent_t e;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventReleaseToDevice) != hipSuccess) return KVP_EDEVICE;
        list->push_back(e);
      }
    c->set_last_group.assign(n_sets, -1);
  }
  const int mode = scoring == KVP_SCORE_PROXY ? kScoreProxy : scoring == KVP_SCORE_KEYDIFF ? kScoreKeydiff : kScoreOwn;
  for (int first = 0; first < n_layers; first += group) {
    int last = std::min(n_layers, first + group);
    if (two) {
      // A scratch set must have been released by the compaction that used it last; the side
      // stream is in order, so the latest such group covers the others, and with them the
      // compaction of each layer's previous block (which used that layer's own set).
      long long dep = -1;
      for (int layer = first; layer < last; ++layer) dep = std::max(dep, c->set_last_group[layer % n_sets]);
      if (dep > c->waited_group) {
        if (hipStreamWaitEvent(main, c->compacted[dep % ring], 0) != hipSuccess) return KVP_EDEVICE;
        c->waited_group = dep;
      }
    }
    int rc = KVP_OK;
    for (int layer = first; layer < last; ++layer) {
      rc = prefill_impl(c, layer, token_begin, n_tokens, q[layer], k[layer], v[layer], out[layer],
                        mode == kScoreProxy ? q_obs[layer] : nullptr, n_obs, mode, stream, mode != kScoreOwn);
      if (rc) {
        last = layer;                            // the layers before it still get their compaction
        break;
      }
    }
    if (mode != kScoreOwn && last > first) {
      const int rc3 = score_deferred_layers(c, first, last - first, main);
      if (rc3) return rc3;
    }
    const size_t slot = (size_t)(c->n_groups % ring);
    if (two && last > first) {
      if (hipEventRecord(c->attended[slot], main) != hipSuccess) return KVP_EDEVICE;
      if (hipStreamWaitEvent(side, c->attended[slot], 0) != hipSuccess) return KVP_EDEVICE;
    }
    if (last > first) {
      const int rc2 = compact_layers(c, first, last - first, nullptr, two ? side : main);
      if (rc2) return rc2;
    }
    if (two && last > first) {
      if (hipEventRecord(c->compacted[slot], side) != hipSuccess) return KVP_EDEVICE;
      for (int layer = first; layer < last; ++layer) c->set_last_group[layer % n_sets] = c->n_groups;
      ++c->n_groups;
    }
    if (rc) return rc;
  }
  return KVP_OK;
}

int kvp_prefill_join(kvp_cache* c, void* stream, void* side_stream) {
  if (!c) return KVP_EINVAL;
  if (c->dry || !side_stream || side_stream == stream || c->n_groups == 0) return KVP_OK;
  // the side stream is in order: its last event covers every compaction before it
  const size_t slot = (size_t)((c->n_groups - 1) % (long long)c->compacted.size());
  if (hipStreamWaitEvent(static_cast<hipStream_t>(stream), c->compacted[slot], 0) != hipSuccess) return KVP_EDEVICE;
  c->waited_group = c->n_groups - 1;
  return KVP_OK;
}

int kvp_decode_ready(kvp_cache* c, int32_t layer, kvp_view* out) {
  if (!c || !out || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  const Layer& L = c->layers[layer];
  if (L.state != READY) return KVP_ESTATE;
  out->k = c->k_cache(layer);
  out->v = c->v_cache(layer);
  out->token_idx = c->idx(layer);
  out->weight = c->weight(layer);
  out->count = L.count;
  out->budget = c->cfg.budget;
  out->next_token = L.next_token;
  return KVP_OK;
}

int kvp_decode_step(kvp_cache* c, int32_t layer, const void* q, const void* k_tail, const void* v_tail,
                    int32_t n_tail, void* out, void* stream) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  if (n_tail < 1 || n_tail > (1 << 20)) return KVP_EINVAL;
  if (!c->dry && (!q || !k_tail || !v_tail || !out)) return KVP_EINVAL;
  const kvp_config& cfg = c->cfg;
  if (cfg.n_q_heads / cfg.n_kv_heads > decode_max_group()) return KVP_EINVAL;
  const Layer& L = c->layers[layer];
  if (L.state != READY) return KVP_ESTATE;
  if (c->set_owner[layer % c->lay.n_sets] != -1) return KVP_ESTATE;
  const Layout& lay = c->lay;
  DecodeArgs da{};
  da.q = static_cast<const u16*>(q);
  da.k_tail = static_cast<const u16*>(k_tail);
  da.v_tail = static_cast<const u16*>(v_tail);
  da.out = static_cast<u16*>(out);
  da.k_cache = c->k_cache(layer);
  da.v_cache = c->v_cache(layer);
  da.partial = reinterpret_cast<float*>(c->set(layer) + lay.partial_off);
  da.c = L.count; da.n_tail = n_tail;
  da.n_q_heads = cfg.n_q_heads; da.n_kv_heads = cfg.n_kv_heads; da.budget = cfg.budget;
  da.scale_log2 = c->scale * 1.4426950408889634f;
  const size_t have = (size_t)cfg.n_kv_heads * lay.max_partials * lay.cand_stride;   // floats
  da.n_splits = decode_splits((long long)L.count + n_tail, cfg.head_dim, have, cfg.n_q_heads);
  if (da.n_splits < 1) return KVP_ENOMEM;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return launch(c, KVP_K_DECODE, 1, s, [&] { return launch_decode(da, cfg.head_dim, s); });
}

int kvp_decode_step_static(kvp_cache* c, int32_t layer, const void* q, const void* k_tail, const void* v_tail,
                           int32_t n_tail, void* out, void* stream) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  if (n_tail < 1 || n_tail > (1 << 20)) return KVP_EINVAL;
  if (!c->dry && (!q || !k_tail || !v_tail || !out)) return KVP_EINVAL;
  const kvp_config& cfg = c->cfg;
  if (cfg.n_q_heads / cfg.n_kv_heads > decode_max_group()) return KVP_EINVAL;
  const Layer& L = c->layers[layer];
  if (L.state != READY) return KVP_ESTATE;
  // the partial results must fit the static array with enough workgroups per KV head to be worth
  // running: all the step wants, or KVP_STATIC_MIN_SPLITS of them
  const size_t have = KVP_STATIC_SCRATCH_BYTES / sizeof(float);
  const int want = decode_splits_wanted((long long)L.count + n_tail);
  const int splits = decode_splits((long long)L.count + n_tail, cfg.head_dim, have, cfg.n_q_heads);
  if (splits < (want < KVP_STATIC_MIN_SPLITS ? want : KVP_STATIC_MIN_SPLITS)) return KVP_ENOMEM;
  if (c->dry) return KVP_OK;
  if (!c->static_scratch || c->static_scratch_floats < have) return KVP_EDEVICE;
  DecodeArgs da{};
  da.q = static_cast<const u16*>(q);
  da.k_tail = static_cast<const u16*>(k_tail);
  da.v_tail = static_cast<const u16*>(v_tail);
  da.out = static_cast<u16*>(out);
  da.k_cache = c->k_cache(layer);
  da.v_cache = c->v_cache(layer);
  da.partial = c->static_scratch;       // the looked-up device address, never the array's name
  da.c = L.count; da.n_tail = n_tail;
  da.n_q_heads = cfg.n_q_heads; da.n_kv_heads = cfg.n_kv_heads; da.budget = cfg.budget;
  da.scale_log2 = c->scale * 1.4426950408889634f;
  da.n_splits = splits;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return launch(c, KVP_K_DECODE, 1, s, [&] { return launch_decode(da, cfg.head_dim, s); });
}

int kvp_set_state(kvp_cache* c, int32_t layer, int32_t count, int32_t next_token) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  if (count < 0 || count > c->cfg.budget) return KVP_EINVAL;
  if (next_token < 0 || next_token > c->n_tokens || count > next_token) return KVP_EINVAL;
  Layer& L = c->layers[layer];
  const int set_i = layer % c->lay.n_sets;
  if (L.state == PENDING && c->set_owner[set_i] == layer) c->set_owner[set_i] = -1;
  L.state = READY;
  L.unscored = 0;
  L.count = count;
  L.next_token = next_token;
  L.has_last = false;
  return KVP_OK;
}

int kvp_set_attention_shape(kvp_cache* c, int32_t shape) {
  if (!c || shape < -1 || shape > 2) return KVP_EINVAL;
  c->attn_shape = shape;
  return KVP_OK;
}

int kvp_set_deferred_scoring(kvp_cache* c, int32_t on) {
  if (!c || (on != 0 && on != 1)) return KVP_EINVAL;
  c->deferred_scoring = on != 0;
  return KVP_OK;
}

int kvp_set_score_sweep(kvp_cache* c, int32_t fused) {
  if (!c || (fused != 0 && fused != 1)) return KVP_EINVAL;
  c->fused_scores = fused != 0;
  return KVP_OK;
}

int kvp_debug_last(kvp_cache* c, int32_t layer, const float** scores, const uint8_t** keep,
                   const int32_t** dst, int32_t* n_cand, int32_t* stride) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVP_EINVAL;
  const Layer& L = c->layers[layer];
  if (!L.has_last) return KVP_ESTATE;
  unsigned char* set = c->set(layer);
  if (scores) *scores = reinterpret_cast<const float*>(set + c->lay.scores_off);
  if (keep) *keep = set + c->lay.keep_off;
  if (dst) *dst = reinterpret_cast<const int32_t*>(set + c->lay.dst_off);
  if (n_cand) *n_cand = L.last_cand;
  if (stride) *stride = c->lay.cand_stride;
  return KVP_OK;
}

int kvp_debug_totals(kvp_cache* c, const uint64_t** totals) {
  if (!c || !totals) return KVP_EINVAL;
  *totals = c->dry ? nullptr : reinterpret_cast<const uint64_t*>(c->totals());
  return KVP_OK;
}

int kvp_profile_enable(kvp_cache* c, int32_t on) {
  if (!c) return KVP_EINVAL;
  c->profiling = on != 0 && !c->dry;
  return KVP_OK;
}

int kvp_profile_read(kvp_cache* c, kvp_kernel_stat* stats) {
  if (!c || !stats) return KVP_EINVAL;
  for (int i = 0; i < KVP_K_COUNT; ++i) stats[i] = kvp_kernel_stat{0, 0, 0.0};
  int rc = KVP_OK;
  for (ProfEvent& pe : c->events) {
    float ms = 0.f;
    if (hipEventSynchronize(pe.stop) != hipSuccess || hipEventElapsedTime(&ms, pe.start, pe.stop) != hipSuccess) {
      rc = KVP_EDEVICE;
    } else {
      stats[pe.kind].launches += 1;
      stats[pe.kind].layers += pe.layers;
      stats[pe.kind].total_ms += ms;
    }
    c->pool.push_back(pe.start);
    c->pool.push_back(pe.stop);
  }
  c->events.clear();
  return rc;
}

void kvp_free_cache(kvp_cache* c) {
  if (!c) return;
  for (ProfEvent& pe : c->events) {
    (void)hipEventDestroy(pe.start);
    (void)hipEventDestroy(pe.stop);
  }
  for (hipEvent_t e : c->pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->attended) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->compacted) (void)hipEventDestroy(e);
  delete c;
}

}  // extern "C"

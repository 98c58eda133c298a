// Drives the C ABI of the host-only sanitized build through the dry-run cases of the Python host
// tests: configuration and segment validation, sizes, the per-layer state machine over all five
// workloads and all three ways of scoring, kvp_prefill_block in groups, the decode entry points
// and their limits.  Exits 0 when every check holds; the sanitizers abort on any invalid access.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "kvp.h"

#define CHECK(cond)                                                            \
  do {                                                                         \
    if (!(cond)) {                                                             \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                            \
    }                                                                          \
  } while (0)

struct Shape {
  const char* name;
  int layers, hq, hkv, d, chunk, budget, gh, gw, planes, temporal, n_text;
};
static const Shape kShapes[] = {
    {"tiny", 1, 4, 4, 64, 64, 128, 24, 24, 1, 0, 32},
    {"single_image", 4, 32, 32, 128, 128, 256, 24, 24, 1, 0, 64},
    {"tiled_image", 8, 28, 4, 128, 256, 512, 24, 24, 5, 0, 128},
    {"video", 16, 28, 4, 128, 512, 1024, 14, 14, 32, 1, 128},
    {"long_video", 32, 32, 8, 128, 1024, 2048, 16, 16, 64, 1, 256},
    {"limit", 2, 16, 1, 64, 2048, 6144, 16, 16, 47, 1, 256},        // 8192 candidates, 16 heads per KV head
};

static kvp_config config_of(const Shape& s, int sets) {
  kvp_config c{};
  c.n_layers = s.layers; c.n_q_heads = s.hq; c.n_kv_heads = s.hkv; c.head_dim = s.d;
  c.budget = s.budget; c.chunk_max = s.chunk; c.merge = 1; c.scratch_sets = sets;
  c.flags = KVP_FLAG_DRY_RUN; c.softmax_scale = 0.f;
  return c;
}

static std::vector<kvp_segment> segments_of(const Shape& s) {
  const int nvis = s.gh * s.gw * s.planes;
  return {kvp_segment{0, nvis, KVP_VISUAL, s.gh, s.gw, s.planes, s.temporal},
          kvp_segment{nvis, s.n_text, KVP_TEXT, 0, 0, 0, 0}};
}

int main() {
  CHECK(kvp_strerror(KVP_OK) && kvp_strerror(-77));
  for (const Shape& s : kShapes) {
    const std::vector<kvp_segment> segs = segments_of(s);
    const int n_tokens = segs[0].n_tokens + segs[1].n_tokens;
    for (int sets : {1, 2, s.layers}) {
      if (sets > s.layers) continue;
      kvp_config cfg = config_of(s, sets);
      CHECK(kvp_cache_bytes(&cfg) > kvp_persistent_bytes(&cfg));
      CHECK(kvp_persistent_bytes(&cfg) >= (size_t)2 * s.layers * s.hkv * s.d * 2 * s.budget);
      kvp_cache* c = nullptr;
      CHECK(kvp_init_cache(&cfg, segs.data(), 2, nullptr, 0, nullptr, &c) == KVP_OK && c);
      // per-layer calls, every way of scoring in turn
      int count = 0, block = 0;
      for (int t0 = 0; t0 < n_tokens; t0 += s.chunk, ++block) {
        const int n = t0 + s.chunk <= n_tokens ? s.chunk : n_tokens - t0;
        for (int l = 0; l < s.layers; ++l) {
          int rc;
          if (block % 3 == 0) rc = kvp_prefill_chunk(c, l, t0, n, nullptr, nullptr, nullptr, nullptr, nullptr);
          else if (block % 3 == 1) rc = kvp_prefill_chunk_keydiff(c, l, t0, n, nullptr, nullptr, nullptr, nullptr, nullptr);
          else rc = kvp_prefill_chunk_proxy(c, l, t0, n, nullptr, nullptr, nullptr, nullptr, nullptr, 1 + block % s.chunk, nullptr);
          CHECK(rc == KVP_OK);
          CHECK(kvp_prefill_chunk(c, l, t0 + n, 1, nullptr, nullptr, nullptr, nullptr, nullptr) == KVP_ESTATE);
          kvp_view vw{};
          CHECK(kvp_decode_ready(c, l, &vw) == KVP_ESTATE);
          CHECK(kvp_compact(c, l, nullptr, nullptr) == KVP_OK);
          CHECK(kvp_compact(c, l, nullptr, nullptr) == KVP_ESTATE);
          CHECK(kvp_decode_ready(c, l, &vw) == KVP_OK);
          const int want = count + n < s.budget ? count + n : s.budget;
          CHECK(vw.count == want && vw.next_token == t0 + n && vw.budget == s.budget);
          if (s.hq / s.hkv <= 16) {
            CHECK(kvp_decode_step(c, l, nullptr, nullptr, nullptr, 1 + block, nullptr, nullptr) == KVP_OK);
            const int rcs = kvp_decode_step_static(c, l, nullptr, nullptr, nullptr, 1 + block, nullptr, nullptr);
            CHECK(rcs == KVP_OK || rcs == KVP_ENOMEM);
          }
        }
        count = count + n < s.budget ? count + n : s.budget;
      }
      CHECK(kvp_prefill_chunk(c, 0, n_tokens, 1, nullptr, nullptr, nullptr, nullptr, nullptr) == KVP_EINVAL);
      // the whole prefix again through kvp_prefill_block (groups of layers), after a restore
      for (int l = 0; l < s.layers; ++l) CHECK(kvp_set_state(c, l, 0, 0) == KVP_OK);
      std::vector<const void*> in(s.layers, nullptr);
      std::vector<void*> out(s.layers, nullptr);
      int blk = 0;
      for (int t0 = 0; t0 < n_tokens; t0 += s.chunk, ++blk) {
        const int n = t0 + s.chunk <= n_tokens ? s.chunk : n_tokens - t0;
        // the three ways of scoring in turn: the proxy and key-only passes go out for a group of layers
        const int scoring = blk % 3 == 0 ? KVP_SCORE_OWN : blk % 3 == 1 ? KVP_SCORE_PROXY : KVP_SCORE_KEYDIFF;
        CHECK(kvp_prefill_block(c, t0, n, in.data(), in.data(), in.data(), out.data(), scoring,
                                scoring == KVP_SCORE_PROXY ? in.data() : nullptr, 1 + blk % s.chunk,
                                nullptr, nullptr) == KVP_OK);
      }
      CHECK(kvp_prefill_join(c, nullptr, nullptr) == KVP_OK);
      // and once more layer by layer with one kvp_compact_layers per block, as far as the scratch
      // sets allow layers to be pending together
      for (int l = 0; l < s.layers; ++l) CHECK(kvp_set_state(c, l, 0, 0) == KVP_OK);
      CHECK(kvp_compact_layers(c, 0, s.layers + 1, nullptr) == KVP_EINVAL);
      CHECK(kvp_compact_layers(c, 0, 1, nullptr) == KVP_ESTATE);
      for (int t0 = 0; t0 < n_tokens; t0 += s.chunk) {
        const int n = t0 + s.chunk <= n_tokens ? s.chunk : n_tokens - t0;
        const int together = sets < s.layers ? sets : s.layers;
        for (int first = 0; first < s.layers; first += together) {
          const int count = first + together <= s.layers ? together : s.layers - first;
          for (int l = first; l < first + count; ++l)
            CHECK(kvp_prefill_chunk(c, l, t0, n, nullptr, nullptr, nullptr, nullptr, nullptr) == KVP_OK);
          CHECK(kvp_compact_layers(c, first, count, nullptr) == KVP_OK);
        }
      }
      for (int l = 0; l < s.layers; ++l) {
        kvp_view vw{};
        CHECK(kvp_decode_ready(c, l, &vw) == KVP_OK && vw.next_token == n_tokens);
      }
      CHECK(kvp_set_attention_shape(c, 3) == KVP_EINVAL && kvp_set_attention_shape(c, 1) == KVP_OK);
      CHECK(kvp_set_score_sweep(c, 2) == KVP_EINVAL && kvp_set_score_sweep(c, 0) == KVP_OK);
      const uint64_t* totals = reinterpret_cast<const uint64_t*>(1);
      CHECK(kvp_debug_totals(c, &totals) == KVP_OK && totals == nullptr);
      kvp_kernel_stat stats[KVP_K_COUNT];
      CHECK(kvp_profile_enable(c, 1) == KVP_OK && kvp_profile_read(c, stats) == KVP_OK);
      kvp_free_cache(c);
    }
  }
  // refused configurations and layouts
  {
    kvp_config bad = config_of(kShapes[0], 1);
    bad.head_dim = 96;
    CHECK(kvp_cache_bytes(&bad) == 0);
    kvp_config big = config_of(kShapes[0], 1);
    big.budget = 8190;
    CHECK(kvp_cache_bytes(&big) == 0);
    kvp_config ok = config_of(kShapes[0], 1);
    kvp_cache* c = nullptr;
    kvp_segment gap[2] = {{0, 10, KVP_VISUAL, 2, 5, 1, 0}, {11, 5, KVP_TEXT, 0, 0, 0, 0}};
    CHECK(kvp_init_cache(&ok, gap, 2, nullptr, 0, nullptr, &c) == KVP_EINVAL && !c);
    CHECK(kvp_init_cache(&ok, gap, 0, nullptr, 0, nullptr, &c) == KVP_EINVAL);
    CHECK(kvp_init_cache(&ok, nullptr, 1, nullptr, 0, nullptr, &c) == KVP_EINVAL);
    CHECK(kvp_compact(nullptr, 0, nullptr, nullptr) == KVP_EINVAL);
    kvp_free_cache(nullptr);
  }
  std::puts("host state machine under the sanitizers: ok");
  return 0;
}

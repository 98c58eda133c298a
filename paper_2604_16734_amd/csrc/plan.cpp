// Host-side planning of the launches: workgroup shapes, grids, splits and scratch sizes.  Nothing
// here touches the device; the file is also part of the host-only build that runs the state
// machine under the address and undefined-behaviour sanitizers.
#include "kvp_internal.h"

namespace kvp {

// ---- attention
// eight waves x 32 rows (two waves per SIMD) when 128-row workgroups fill the chip, otherwise four
// waves x 32 rows over 64-row workgroups
static int shape_for(int n, int n_q_heads) { return ((n + 127) / 128) * n_q_heads >= 192 ? 2 : 1; }

// The most partial score arrays per KV head (query heads of the group x row tiles) that a block of
// up to chunk_max rows leaves when the library picks the shape itself.  A forced shape may need
// more; such a launch then scores with the separate kernel.
int attention_max_partials(int group, int n_q_heads, int chunk_max) {
  int most = 0;
  for (int n = 1; n <= chunk_max; ++n) {
    const int rows = kAttnRowsOfShape[shape_for(n, n_q_heads)];
    const int tiles = (n + rows - 1) / rows;
    most = tiles > most ? tiles : most;
  }
  return group * most;
}

void plan_attention(AttnArgs& a, int /*head_dim*/, int forced_shape) {
  a.variant = shape_for(a.n, a.n_q_heads);
  if (forced_shape >= 0 && forced_shape <= 2) a.variant = forced_shape;      // kvp_set_attention_shape
  const int rows = kAttnRowsOfShape[a.variant];
  a.n_row_tiles = (a.n + rows - 1) / rows;
  a.total_work = a.n_row_tiles * a.n_q_heads;
  a.work_per_xcd = (a.total_work + kXcds - 1) / kXcds;
}


// ---- column sums
int colsum_max_partials(int /*group*/, int /*chunk_max*/) { return kColsumMaxRowSplits; }

void plan_colsum(ColsumArgs& a, int /*head_dim*/) {
  const int n_cand = a.c + a.n_keys;
  const int n_qt = (a.n + 31) / 32;
  // 64 keys per wave, or 32 when that is what it takes to spread a small launch over the chip
  int nt = 2;
  {
    const int blocks = (n_cand + 64 * kColsumWaves - 1) / (64 * kColsumWaves);
    const int splits = n_qt < kColsumMaxRowSplits ? n_qt : kColsumMaxRowSplits;
    if (a.n_kv_heads * blocks * splits < kColsumTargetWorkgroups / 2) nt = 1;
  }
  a.subtiles = nt;
  const int block_keys = 32 * nt * kColsumWaves;
  a.n_kv_blocks = (n_cand + block_keys - 1) / block_keys;
  // tiles per workgroup: the fewest that keep the launch within one round (and the row splits of
  // a block within the partial count)
  int tau = (n_qt + kColsumMaxRowSplits - 1) / kColsumMaxRowSplits;
  for (;; ++tau) {
    int total = 0, most = 0;
    for (int k = 0; k < a.n_kv_blocks; ++k) {
      const int blk0 = k * block_keys;
      const int first_tile = blk0 - a.c > a.shift ? (blk0 - a.c - a.shift) / 32 : 0;
      const int visible = n_qt - first_tile > 0 ? n_qt - first_tile : 1;
      const int splits = (visible + tau - 1) / tau;
      a.split_prefix[k] = total;
      total += splits;
      most = splits > most ? splits : most;
    }
    a.split_prefix[a.n_kv_blocks] = total;
    a.wgs_per_head = total;
    a.n_partials = most;
    if (total * a.n_kv_heads <= kColsumTargetWorkgroups || tau >= n_qt) break;
  }
  a.total_work = a.wgs_per_head * a.n_kv_heads;
  a.work_per_xcd = (a.total_work + kXcds - 1) / kXcds;
}


// ---- selection
size_t select_lds_bytes(int /*n_cand*/, int items, int table_size) {
  const size_t cand_pad = (size_t)items * kSelectThreads;
  return cand_pad * (4 + 4 + 1) + select_region_bytes(cand_pad) + (size_t)table_size * 2;
}

// ---- compaction: row pairs (K row and V row of a slot, 16 bytes per lane) a workgroup carries
int rows_per_compact_block(int head_dim) { return kCompactThreads / (2 * head_dim / 8); }

// ---- proxy row statistics, key-only scores
int rowstat_key_blocks(int n_cand) { return (n_cand + kRowstatBlockKeys - 1) / kRowstatBlockKeys; }
int keydiff_slices(int n_cand) { return (n_cand + kKeydiffSliceKeys - 1) / kKeydiffSliceKeys; }

// ---- decode step
int decode_max_group() { return kDecodeGroupLimit; }

// workgroups per KV head the step would like: one per 64-key tile, kDecodeMaxSplits at most
int decode_splits_wanted(long long n_keys) {
  const long long want = (n_keys + kDecodeTile - 1) / kDecodeTile;
  return (int)(want > kDecodeMaxSplits ? kDecodeMaxSplits : want);
}

// workgroups per KV head: as many as wanted while their partial results fit the scratch
// (every workgroup then has at least one tile)
int decode_splits(long long n_keys, int head_dim, size_t scratch_floats, int n_q_heads) {
  long long want = decode_splits_wanted(n_keys);
  const long long fit = (long long)(scratch_floats / ((size_t)n_q_heads * (head_dim + 2)));
  if (want > fit) want = fit;
  return want < 1 ? 0 : (int)want;
}

}  // namespace kvp

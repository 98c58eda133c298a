// Internal declarations shared by the host state machine and the kernel
// launchers of libkvp.  Not part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvp.h"

namespace kvp {

typedef unsigned short u16;  // one bfloat16 bit pattern

constexpr int kXcds = 8;            // MI355X: 8 accelerator dies, each with its own L2
constexpr int kNeighbours = 6;      // 4 in the plane + 2 in time

// One block of one layer attending over cache U block (Eq. 1).
struct AttnArgs {
  const u16* q;        // [n, Hq, D]
  const u16* k_new;    // [n, Hkv, D]
  const u16* v_new;    // [n, Hkv, D]
  u16* out;            // [n, Hq, D], or null: only the row statistics are wanted
  const u16* k_cache;  // this layer: [Hkv, M, D]
  const u16* v_cache;
  float* lse2;         // [Hq, lse_stride]  log2-domain log-sum-exp of every row
  int n, c, n_q_heads, n_kv_heads, budget, lse_stride;
  int n_keys;          // block keys (k_new, v_new rows); the query rows are n
  int shift;           // row r sees block key j iff j <= r + shift (0: causal block; >= n_keys: all)
  int n_row_tiles, work_per_xcd, total_work;
  int variant;         // tile shape, chosen by plan_attention
  float scale_log2;    // softmax scale times log2(e)
};

// Column sums of the softmax matrix (Eq. 4 summed over rows and over the query
// heads of a KV group), one partial array per row split.
constexpr int kColsumMaxKvBlocks = 64;
struct ColsumArgs {
  const u16* q;
  const u16* k_new;
  const u16* k_cache;
  const float* lse2;
  float* partial;      // [Hkv, n_partials, cand_stride]
  int n, c, n_q_heads, n_kv_heads, budget, lse_stride, cand_stride;
  int n_keys, shift;   // as in AttnArgs
  int n_kv_blocks;     // blocks of 256 * subtiles keys
  int n_partials;      // the most row splits any key block has; every key gets that many partials
  int subtiles;        // 32-key subtiles per wave, chosen by plan_colsum
  int wgs_per_head;    // = split_prefix[n_kv_blocks]
  int work_per_xcd, total_work;
  float scale_log2;
  // workgroups [split_prefix[k], split_prefix[k + 1]) of a head share key block k and split the
  // 32-row query tiles that see it evenly among themselves
  int split_prefix[kColsumMaxKvBlocks + 1];
};

// Row statistics of a short list of proxy queries over all candidates (rowstat.hip).
struct RowstatArgs {
  const u16* q;        // [n, Hq, D] proxy queries
  const u16* k_new;    // [n_keys, Hkv, D]
  const u16* k_cache;  // this layer: [Hkv, M, D]
  float* lse2;         // [Hq, lse_stride] out
  float* part_m;       // [Hq, n, n_kv_blocks] scratch: row maximum per key block (raw logits)
  float* part_l;       // [Hq, n, n_kv_blocks] scratch: sum of exp2 against that maximum
  int n, c, n_keys, n_q_heads, n_kv_heads, budget, lse_stride;
  int n_kv_blocks;     // set by launch_rowstat
  float scale_log2;
};
int rowstat_key_blocks(int n_cand);
hipError_t launch_rowstat(RowstatArgs a, int head_dim, hipStream_t s);

// Query-agnostic scores of all candidates (keydiff.hip).
struct KeydiffArgs {
  const u16* k_new;    // [n_keys, Hkv, D]
  const u16* k_cache;  // this layer: [Hkv, M, D]
  float* sums;         // [Hkv, n_slices, D] scratch: column sums of the keys, one per slice
  float* scores;       // [Hkv, cand_stride] out
  int c, n_keys, n_kv_heads, budget, cand_stride;
  int n_slices, keys_per_block;   // set by launch_keydiff
};
int keydiff_slices(int n_cand);
hipError_t launch_keydiff(KeydiffArgs a, int head_dim, hipStream_t s);

// One decode step of one layer (decode.hip).
struct DecodeArgs {
  const u16* q;        // [Hq, D]
  const u16* k_tail;   // [n_tail, Hkv, D]
  const u16* v_tail;
  u16* out;            // [Hq, D]
  const u16* k_cache;  // this layer: [Hkv, M, D]
  const u16* v_cache;
  float* partial;      // [Hq, n_splits, D + 2] scratch: unnormalised output, maximum, sum
  int c, n_tail, n_q_heads, n_kv_heads, budget, n_splits;
  float scale_log2;
};
int decode_max_group();
int decode_splits(long long n_keys, int head_dim, size_t scratch_floats, int n_q_heads);
int decode_splits_wanted(long long n_keys);
hipError_t launch_decode(const DecodeArgs& a, int head_dim, hipStream_t s);
// address and size of the file-scope scratch array on the current device (kvp_decode_step_static)
hipError_t decode_static_scratch(float** ptr, size_t* n_floats);

// Device copy of one prefix segment.
struct Seg {
  int begin, n, kind, gh, gw, planes, temporal;
};

// Per-head outputs of the select kernel, inputs of merge and move.
struct HeadCounts {
  int n_moves;   // kept block tokens = free slots filled
  int n_dst;     // merge destinations that have at least one source
  int pad0, pad1;
};
struct MoveEntry {
  int pos;    // candidate position (>= c) of the kept block token
  int slot;   // cache slot it goes to
  int stage;  // index into the staging rows if the token is a merge destination, else -1
  int pad;
};
struct DstEntry {
  int pos;                  // candidate position of the destination
  int n_src;
  int src[kNeighbours];     // candidate positions of its sources
};

struct SelectArgs {
  const float* partial;         // [Hkv, n_partials, cand_stride] or null when override is set
  const float* score_override;  // [Hkv, n_cand] or null
  float* scores;                // [Hkv, cand_stride]   scores actually used
  uint8_t* keep;                // [Hkv, cand_stride]
  int32_t* dst;                 // [Hkv, cand_stride]
  const int32_t* token_idx;     // this layer: [Hkv, M]
  HeadCounts* counts;           // [Hkv]
  MoveEntry* moves;             // [Hkv, chunk_max]
  DstEntry* dsts;               // [Hkv, chunk_max]
  const Seg* segs;
  int n_segs;
  int c, n, t0, budget, cand_stride, chunk_max, n_partials, merge;
  int items;                    // candidates per thread
  int table_size;               // power of two >= 2 * (c + n)
};

struct CompactArgs {
  u16* k_cache;            // this layer
  u16* v_cache;
  int32_t* token_idx;
  float* weight;
  const u16* k_new;
  const u16* v_new;
  const HeadCounts* counts;
  const MoveEntry* moves;
  const DstEntry* dsts;
  u16* stage_k;            // [Hkv, chunk_max, D]
  u16* stage_v;
  float* stage_w;          // [Hkv, chunk_max]
  int c, n, t0, budget, n_kv_heads, head_dim, chunk_max;
  int identity;            // 1: plain append of all n tokens to slots c..c+n-1
  int blocks_per_head;
};

// launchers (each returns the hipError_t of the launch)
hipError_t launch_attention(const AttnArgs& a, int head_dim, hipStream_t s);
hipError_t launch_colsum(const ColsumArgs& a, int head_dim, hipStream_t s);
hipError_t launch_select(const SelectArgs& a, int n_kv_heads, hipStream_t s);
hipError_t launch_merge(const CompactArgs& a, hipStream_t s);
hipError_t launch_move(const CompactArgs& a, hipStream_t s);
hipError_t launch_init(int32_t* token_idx, float* weight, size_t n_slots, const Seg* host_segs,
                       int n_segs, Seg* dev_segs, hipStream_t s);
int rows_per_compact_block();

// host-side planning shared by launchers and the state machine
void plan_attention(AttnArgs& a, int head_dim, int forced_shape);   // forced_shape < 0: chosen from the launch size
hipError_t prepare_attention();   // function attributes on the current device; once per cache creation
hipError_t prepare_select();
void plan_colsum(ColsumArgs& a, int head_dim);
int colsum_max_partials(int group, int chunk_max);
size_t select_lds_bytes(int n_cand, int items, int table_size);

}  // namespace kvp

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

// Sizes that the kernels and the host-side planning (plan.cpp) must agree on.
constexpr int kAttnRowsOfShape[3] = {128, 64, 128};   // query rows per workgroup of the three attention shapes
constexpr int kColsumWaves = 4;                 // waves per workgroup of the column-sum kernel
constexpr int kColsumTargetWorkgroups = 512;    // two per CU, all resident: the launch is a single round
constexpr int kColsumMaxRowSplits = 16;
constexpr int kSelectThreads = 1024;
constexpr int kSelectCopies = 32;               // histogram replicas of the radix select
constexpr int kRowstatBlockKeys = 256;          // keys per workgroup of the proxy row-statistics kernel
constexpr int kKeydiffSliceKeys = 64;           // keys per workgroup of the key-sum kernel
constexpr int kDecodeTile = 64;                 // keys per workgroup step of the decode kernel
constexpr int kDecodeMaxSplits = 128;
constexpr int kDecodeGroupLimit = 16;           // query heads per KV head the decode kernel is built for
constexpr int kCompactThreads = 256;
constexpr int kCompactTargetWorkgroups = 4096;  // a merge or move launch is capped at about this many workgroups

// bytes of the select kernel's region that is first the radix histogram and then the compaction lists
constexpr size_t select_region_bytes(size_t cand_pad) {
  const size_t hist = (size_t)256 * kSelectCopies * 4, lists = cand_pad * 5;
  return (hist > lists ? hist : lists + 15) / 16 * 16;
}

// One block of one layer attending over cache U block (Eq. 1).
struct AttnArgs {
  const u16* q;        // [n, Hq, D]
  const u16* k_new;    // [n, Hkv, D]
  const u16* v_new;    // [n, Hkv, D]
  u16* out;            // [n, Hq, D], or null: only the row statistics are wanted
  const u16* k_cache;  // this layer: [Hkv, M, D]
  const u16* v_cache;
  float* lse2;         // [Hq, lse_stride]  log2-domain log-sum-exp of every row
  float* partial;      // null, or [Hkv, n_partials, cand_stride]: the launch also leaves the column sums
                       // of its softmax matrix (Eq. 4), one array per workgroup of a KV head
  int n_partials, cand_stride;   // n_partials = query heads per KV head x n_row_tiles
  int n, c, n_q_heads, n_kv_heads, budget, lse_stride;
  int n_keys;          // block keys (k_new, v_new rows); the query rows are n
  int shift;           // row r sees block key j iff j <= r + shift (0: causal block; >= n_keys: all)
  int n_row_tiles, work_per_xcd, total_work;
  int variant;         // tile shape, chosen by plan_attention
  float scale_log2;    // softmax scale times log2(e)
};

// A launch of the selection and compaction kernels covers a group of consecutive layers that hold
// the same block (same c, n, t0).  The pointers in SelectArgs and CompactArgs are those of the
// group's FIRST layer; layer i of the group is reached through the strides below.
constexpr int kMaxGroupLayers = 16;
struct LayerGroup {
  int n_layers;
  int first_set, n_sets;        // layer i uses scratch set (first_set + i) % n_sets
  long long set_stride;         // bytes between scratch sets
  long long kv_stride;          // bf16 elements between the K (or V) caches of consecutive layers
  long long meta_stride;        // elements between their token_idx (or weight) arrays
  const u16* k_new[kMaxGroupLayers];   // the block's keys and values of every layer of the group
  const u16* v_new[kMaxGroupLayers];
};

#if defined(__HIPCC__)
// the same pointer in scratch set (first_set + li) % n_sets instead of set first_set
template <class T>
__device__ __forceinline__ T* in_set_of(T* p, const LayerGroup& g, int li) {
  if (p == nullptr) return p;
  const long long sets = (long long)((g.first_set + li) % g.n_sets) - g.first_set;
  return reinterpret_cast<T*>(reinterpret_cast<uintptr_t>(p) + (uintptr_t)(sets * g.set_stride));
}
#endif

// Column sums of the softmax matrix (Eq. 4 summed over rows and over the query
// heads of a KV group), one partial array per row split.
constexpr int kColsumMaxKvBlocks = 64;
struct ColsumArgs {
  // One launch scores a group of layers (grid y = layer): layer i of the group reads its queries
  // from q_layer[i], the block's keys from g.k_new[i], the cache g.kv_stride elements further on
  // per layer, and its statistics and partials from scratch set (g.first_set + i) % g.n_sets.
  LayerGroup g;
  const u16* q_layer[kMaxGroupLayers];
  const u16* k_cache;  // of the group's first layer
  const float* lse2;   // in the first layer's scratch set, like partial
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
  LayerGroup g;        // a group of layers per launch, as in ColsumArgs; g.k_new[i]: [n_keys, Hkv, D]
  const u16* q_layer[kMaxGroupLayers];   // [n, Hq, D] proxy queries of every layer of the group
  const u16* k_cache;  // the group's first layer: [Hkv, M, D]
  float* lse2;         // [Hq, lse_stride] out
  float* part_m;       // [Hq, n, n_kv_blocks] scratch: row maximum per key block (raw logits)
  float* part_l;       // [Hq, n, n_kv_blocks] scratch: sum of exp2 against that maximum
  int n, c, n_keys, n_q_heads, n_kv_heads, budget, lse_stride;
  int n_kv_blocks;     // set by launch_rowstat, like the next two
  int items_per_wg;    // (query head, 32-row tile) items a workgroup takes
  int item_splits;     // workgroups that share the items of a KV head
  float scale_log2;
};
int rowstat_key_blocks(int n_cand);
hipError_t launch_rowstat(RowstatArgs a, int head_dim, hipStream_t s);

// Query-agnostic scores of all candidates (keydiff.hip).
struct KeydiffArgs {
  LayerGroup g;        // a group of layers per launch (grid z); g.k_new[i]: [n_keys, Hkv, D]
  const u16* k_cache;  // the group's first layer: [Hkv, M, D]
  float* sums;         // [Hkv, n_slices, D] scratch: column sums of the keys, one per slice
  float* scores;       // [Hkv, cand_stride] out (both in the first layer's scratch set)
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
  LayerGroup g;
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
  unsigned long long* totals;   // [KVP_T_COUNT] running totals of the cache (kvp_debug_totals)
  int n_segs;
  int c, n, t0, budget, cand_stride, chunk_max, n_partials, merge;
  int items;                    // candidates per thread
  int table_size;               // power of two >= 2 * (c + n)
};

struct CompactArgs {
  LayerGroup g;
  u16* k_cache;            // the group's first layer
  u16* v_cache;
  int32_t* token_idx;
  float* weight;
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
hipError_t launch_select(const SelectArgs& a, int n_kv_heads, hipStream_t s);   // grid: heads x a.g.n_layers
hipError_t launch_merge(const CompactArgs& a, hipStream_t s);
hipError_t launch_move(const CompactArgs& a, hipStream_t s);
hipError_t launch_init(int32_t* token_idx, float* weight, size_t n_slots, const Seg* host_segs,
                       int n_segs, Seg* dev_segs, unsigned long long* totals, hipStream_t s);
int rows_per_compact_block(int head_dim);

// host-side planning shared by launchers and the state machine
void plan_attention(AttnArgs& a, int head_dim, int forced_shape);   // forced_shape < 0: chosen from the launch size
int attention_max_partials(int group, int n_q_heads, int chunk_max);   // most partial score arrays per KV head a launch leaves
constexpr int kMaxFusedPartials = 64;                   // beyond that the separate column-sum kernel scores
hipError_t prepare_attention();   // function attributes on the current device; once per cache creation
hipError_t prepare_select();
void plan_colsum(ColsumArgs& a, int head_dim);
int colsum_max_partials(int group, int chunk_max);
size_t select_lds_bytes(int n_cand, int items, int table_size);

}  // namespace kvp

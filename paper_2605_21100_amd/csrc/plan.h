// Internal definitions shared by the host planner, the launchers and the kernels.
#pragma once
#include <cstdint>
#include <vector>

#include "nanocp.h"

namespace nanocp {

enum Variant : int32_t { kGeneric = 0, kGqaMfmaBf16 = 1, kGqaMfmaFp8 = 2, kMlaMfmaBf16 = 3 };
int pick_variant(const nanocp_attn_desc& d);  // which tile kernel handles this problem shape
nanocp_status check_desc(const nanocp_attn_desc& d);  // shape / dtype checks shared by the host entry points

// Reduction segment: the tile partials of one (shard, kv head).  Only segments with
// n_parts != 1 exist (0 parts = empty shard, filled with O = 0 / LSE = -inf).
struct Seg {
  int32_t shard;
  int32_t kv_head;
  int32_t slot_begin;
  int32_t n_parts;
  int32_t final_row;  // >= 0: the shard is the only partial of this output row (see nanocp_plan_set_final_rows)
};

constexpr int kThreads = 256;       // every kernel here runs 4 wavefronts per workgroup

// Device-side tile record (the public nanocp_tile plus what the fused reduction needs).
struct DevTile {
  int32_t q_row, bt_row, kv_head, shard;
  int32_t tok_begin, tok_end;
  int32_t dst;         // partial slot, or -1 = write the final (shard, head) rows directly
  int32_t seg;         // index of the (shard, head)'s arrival counter (valid if dst >= 0)
  int32_t n_parts;     // tiles of this (shard, head)
  int32_t slot_begin;  // first partial slot of this (shard, head)
  int32_t final_row;   // >= 0: output row this shard alone produces (written in its final form), else -1
  int32_t lse_shard;   // row of out_lse the (shard, head)'s LSE goes to: the shard itself, or the first shard of its group
};

// sync words owned by the plan (zero between launches): [0] work-queue head, [1] finished workgroups,
// [kSyncSegBase + i] arrivals at reduction segment i
constexpr int kSyncSegBase = 2;

// Arguments of the tile kernels (passed by value).
struct KParams {
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const float* k_scale;
  const float* v_scale;
  const int32_t* block_table;
  float* out_o;
  float* out_lse;
  float* ws_o;    // [num_slots, G, Dv]
  float* ws_lse;  // [num_slots, G]
  const DevTile* tiles;
  const int32_t* chunk_offsets;
  int32_t* sync;         // plan-owned counters (see kSyncSegBase)
  int32_t num_chunks;
  const Seg* segs;       // segments without a tile of their own kernel pass (the fused variants fill the empty ones)
  int32_t num_segs;
  const int32_t* header;  // null, or the counts on the device (plan image): they then override num_chunks / num_segs
  uint64_t* tile_clock;   // may be null
  void* final_out;       // [num_out, Hq, Dv] float, bf16 or fp8; null = every shard writes out_o / out_lse
  float* final_lse;      // [num_out, Hq], may be null
  int32_t final_kind;    // nanocp_dtype of final_out
  float out_inv_scale;   // fp8 final rows: code of value * out_inv_scale
  int32_t variant;       // the tile kernel this launch runs (checked against a plan image's header)
  int32_t Hq, Hkv, G, Dk, Dv, ps, max_blocks, kind;
  float scale;
};

// Plan image: the device-side part of a plan as one relocatable block whose layout depends only on the bucket's
// capacities, so that launches recorded once (HIP graph) serve every plan that fits the bucket.
// header words: [0] chunks, [1] reduction segments (separate kernel), [2] fused segments, [3] partial slots
constexpr int kHeaderWords = 64;
struct ImageLayout {
  size_t header, sync, chunk_offsets, tiles, segs, total;
};
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline ImageLayout image_layout(const nanocp_bucket& b) {
  ImageLayout L;
  L.header = 0;
  L.sync = align256(kHeaderWords * sizeof(int32_t));
  L.chunk_offsets = L.sync + align256((size_t)(kSyncSegBase + b.max_segs) * sizeof(int32_t));
  L.tiles = L.chunk_offsets + align256((size_t)(b.max_chunks + 1) * sizeof(int32_t));
  L.segs = L.tiles + align256((size_t)b.max_tiles * sizeof(DevTile));
  L.total = L.segs + align256((size_t)b.max_segs * sizeof(Seg));
  return L;
}

}  // namespace nanocp

struct nanocp_plan {
  nanocp_attn_desc desc;
  int32_t num_shards, num_q_rows, num_bt_rows, max_blocks;
  int32_t variant;
  int32_t num_chunks;
  int32_t num_slots;
  size_t workspace_bytes;
  std::vector<nanocp_tile> tiles;       // grouped by chunk, in execution order
  std::vector<int32_t> chunk_offsets;   // [num_chunks + 1]
  std::vector<nanocp::DevTile> dev_tiles;
  std::vector<nanocp::Seg> segs;        // segments the separate reduce kernel handles
  int32_t num_multi_segs;               // (shard, head) pairs with more than one tile
  int32_t launch_blocks;                // workgroups to launch
  int32_t num_final_rows = 0;           // rows of the final output (0 = nanocp_plan_set_final_rows not called)
  bool grouped = false;                 // some output row is fed by several local shards reduced as one segment
  bool dynamic;                         // workgroups pull chunks from a queue
  bool fused;                           // ... and reduce the tile partials of a (shard, head) themselves
  // device copy
  int device = -1;
  nanocp::DevTile* d_tiles = nullptr;
  int32_t* d_chunk_offsets = nullptr;
  nanocp::Seg* d_segs = nullptr;
  int32_t* d_sync = nullptr;
};

// Host planner: builds the split-KV tile work-list (nanocp_plan_create and friends).
//
// The flattened list of pages of all (shard, kv head) pairs is cut into spans of near-equal
// cost, one span ("chunk") per workgroup.  A span that ends inside a (shard, head) leaves that
// pair with several tiles whose partials are reduced afterwards; pairs that fall entirely
// inside one span write their result directly.  This is the one-GPU analogue of the paper's
// balance objective (Dual-balanced Scheduling / WaterFill: minimise the peak load).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>

#include "plan.h"

using namespace nanocp;

namespace {

int elem_bytes(int dt) { return dt == NANOCP_F32 ? 4 : dt == NANOCP_BF16 ? 2 : 1; }

}  // namespace

nanocp_status nanocp::check_desc(const nanocp_attn_desc& d) {
  if (d.kind != NANOCP_GQA && d.kind != NANOCP_MLA) return NANOCP_EINVAL;
  if (d.q_dtype < 0 || d.q_dtype > 2 || d.kv_dtype < 0 || d.kv_dtype > 2) return NANOCP_EINVAL;
  if (d.num_q_heads <= 0 || d.num_kv_heads <= 0 || d.head_dim_qk <= 0 || d.head_dim_v <= 0 || d.page_size <= 0)
    return NANOCP_EINVAL;
  if (!(d.softmax_scale == d.softmax_scale)) return NANOCP_EINVAL;
  if (d.num_q_heads % d.num_kv_heads) return NANOCP_ESHAPE;
  const int x = 16 / elem_bytes(d.kv_dtype);
  if (d.kind == NANOCP_MLA) {
    if (d.num_kv_heads != 1 || d.head_dim_v > d.head_dim_qk) return NANOCP_ESHAPE;
    if (d.head_dim_qk % x) return NANOCP_ESHAPE;
  } else {
    if (d.head_dim_qk % x || d.page_size % (4 * x)) return NANOCP_ESHAPE;  // V is laid out in groups of 4x tokens
  }
  const bool combo = (d.q_dtype == NANOCP_F32 && d.kv_dtype == NANOCP_F32) ||
                     (d.q_dtype == NANOCP_BF16 && d.kv_dtype == NANOCP_BF16) ||
                     (d.q_dtype == NANOCP_BF16 && d.kv_dtype == NANOCP_FP8_E4M3);
  if (!combo) return NANOCP_EUNSUPPORTED;
  if (d.kind == NANOCP_MLA && d.kv_dtype == NANOCP_FP8_E4M3) return NANOCP_EUNSUPPORTED;
  if (d.head_dim_qk > 576 || d.head_dim_v > 512) return NANOCP_EUNSUPPORTED;  // generic kernel's LDS/register budget
  return NANOCP_OK;
}

int nanocp::pick_variant(const nanocp_attn_desc& d) {
  const int G = d.num_q_heads / d.num_kv_heads;
  if (d.kind == NANOCP_GQA && d.q_dtype == NANOCP_BF16 && G == 16 && d.head_dim_qk == 128 && d.head_dim_v == 128) {
    if (d.kv_dtype == NANOCP_BF16 && d.page_size == 64) return kGqaMfmaBf16;
    if (d.kv_dtype == NANOCP_FP8_E4M3 && d.page_size == 64) return kGqaMfmaFp8;
  }
  if (d.kind == NANOCP_MLA && d.q_dtype == NANOCP_BF16 && d.kv_dtype == NANOCP_BF16 && (d.num_q_heads == 128 || d.num_q_heads == 64) &&
      d.head_dim_qk == 576 && d.head_dim_v == 512 && d.page_size == 64 &&
      d.softmax_scale > 0.f && d.softmax_scale < 3.0e38f)  // the kernel takes maxima over unscaled scores
    return kMlaMfmaBf16;
  return kGeneric;
}

namespace {

// Planner constants.  Only a build with -DNANOCP_TUNING reads overrides from the environment (integers, clamped);
// the product build uses the values below whatever the process environment holds.
int knob(const char* name, int dflt, int lo, int hi) {
#ifdef NANOCP_TUNING
  const char* v = std::getenv(name);
  if (v && *v) {
    char* end = nullptr;
    const long x = std::strtol(v, &end, 10);
    if (end != v) return (int)std::min<long>(hi, std::max<long>(lo, x));
  }
#else
  (void)name, (void)lo, (void)hi;
#endif
  return dflt;
}

// Partial slots and reduction segments.  A segment is the set of tiles whose partials combine into one result:
// the tiles of one (shard, kv head), or -- when final_row names the same output row for several shards (all the
// partials of that row are local) -- of all those shards together, so that the row needs no merge afterwards.
// A segment with one tile writes its result directly (dst = -1); otherwise its tiles get consecutive slots.
void assign_segments(nanocp_plan* p, const int32_t* final_row) {
  const int Hkv = p->desc.num_kv_heads;
  const int G = p->desc.num_q_heads / Hkv;
  const int S = p->num_shards;
  // group id of a shard: the first shard naming the same output row, or itself
  std::vector<int> group(S), first_of_row;
  for (int s = 0; s < S; ++s) {
    group[s] = s;
    if (final_row && final_row[s] >= 0) {
      if ((size_t)final_row[s] >= first_of_row.size()) first_of_row.resize(final_row[s] + 1, -1);
      if (first_of_row[final_row[s]] < 0) first_of_row[final_row[s]] = s;
      group[s] = first_of_row[final_row[s]];
    }
  }
  std::vector<int> count((size_t)S * Hkv, 0), slot0((size_t)S * Hkv, 0), seg_id((size_t)S * Hkv, -1), next((size_t)S * Hkv, 0);
  for (const nanocp_tile& t : p->tiles) count[(size_t)group[t.shard] * Hkv + t.kv_head]++;
  p->num_slots = 0;
  p->num_multi_segs = 0;
  p->segs.clear();
  p->grouped = false;
  for (int s = 0; s < S; ++s) {
    if (group[s] != s) {
      p->grouped = true;
      continue;
    }
    for (int h = 0; h < Hkv; ++h) {
      const size_t key = (size_t)s * Hkv + h;
      const int n = count[key];
      const int fr = final_row ? final_row[s] : -1;
      if (n > 1) {
        slot0[key] = p->num_slots;
        p->num_slots += n;
        seg_id[key] = p->num_multi_segs++;
        if (!p->fused) p->segs.push_back(nanocp::Seg{s, h, slot0[key], n, fr});
      } else if (n == 0) {
        p->segs.push_back(nanocp::Seg{s, h, 0, 0, fr});  // nothing to attend to: O = 0, LSE = -inf
      }
    }
  }
  // members of a group that are not its first shard have no result of their own; an empty one that is alone is
  // covered above (it is its own group)
  for (size_t i = 0; i < p->tiles.size(); ++i) {
    nanocp_tile& t = p->tiles[i];
    const size_t key = (size_t)group[t.shard] * Hkv + t.kv_head;
    const int n = count[key];
    t.dst = n > 1 ? slot0[key] + next[key]++ : -1;
    p->dev_tiles[i] = nanocp::DevTile{t.q_row, t.bt_row, t.kv_head, t.shard, t.tok_begin, t.tok_end, t.dst,
                                      seg_id[key], n, slot0[key], final_row ? final_row[t.shard] : -1, group[t.shard]};
  }
  // workspace: o partials [slots, G, Dv] then lse partials [slots, G], each 256-byte aligned
  const size_t o_bytes = ((size_t)p->num_slots * G * p->desc.head_dim_v * sizeof(float) + 255) & ~(size_t)255;
  const size_t l_bytes = ((size_t)p->num_slots * G * sizeof(float) + 255) & ~(size_t)255;
  p->workspace_bytes = p->num_slots ? o_bytes + l_bytes : 0;
}

}  // namespace

namespace {

void free_device_copy(nanocp_plan* plan) {
  if (plan->d_tiles) (void)hipFree(plan->d_tiles);
  if (plan->d_chunk_offsets) (void)hipFree(plan->d_chunk_offsets);
  if (plan->d_segs) (void)hipFree(plan->d_segs);
  if (plan->d_sync) (void)hipFree(plan->d_sync);
  plan->d_tiles = nullptr;
  plan->d_chunk_offsets = nullptr;
  plan->d_segs = nullptr;
  plan->d_sync = nullptr;
}

}  // namespace

extern "C" {

nanocp_status nanocp_plan_create(const nanocp_attn_desc* desc, const nanocp_shard* shards, int32_t num_shards,
                                 int32_t num_q_rows, int32_t num_bt_rows, int32_t max_blocks_per_row,
                                 int32_t tile_tokens, int32_t num_cus, nanocp_plan** out) {
  if (!desc || !out || (num_shards > 0 && !shards)) return NANOCP_EINVAL;
  *out = nullptr;
  if (num_shards < 0 || num_q_rows < 0 || num_bt_rows < 0 || max_blocks_per_row < 0 || tile_tokens < 0 || num_cus < 0)
    return NANOCP_EINVAL;
  nanocp_status st = check_desc(*desc);
  if (st != NANOCP_OK) return st;
  const int ps = desc->page_size;
  const int64_t row_tokens = (int64_t)max_blocks_per_row * ps;
  for (int s = 0; s < num_shards; ++s) {
    const nanocp_shard& sh = shards[s];
    if (sh.kv_begin < 0 || sh.kv_end < sh.kv_begin) return NANOCP_EINVAL;
    if (sh.q_row < 0 || sh.q_row >= num_q_rows || sh.bt_row < 0 || sh.bt_row >= num_bt_rows) return NANOCP_EBOUNDS;
    if ((int64_t)sh.kv_end > row_tokens) return NANOCP_EBOUNDS;
  }
  if (num_cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NANOCP_EHIP;
    num_cus = prop.multiProcessorCount;
  }

  nanocp_plan* p = new (std::nothrow) nanocp_plan();
  if (!p) return NANOCP_ENOMEM;
  try {
    p->desc = *desc;
    p->num_shards = num_shards;
    p->num_q_rows = num_q_rows;
    p->num_bt_rows = num_bt_rows;
    p->max_blocks = max_blocks_per_row;
    p->variant = nanocp::pick_variant(*desc);
    const int Hkv = desc->num_kv_heads;
    const int G = desc->num_q_heads / Hkv;
    p->dynamic = p->variant != kGeneric;
    p->fused = p->variant == kGqaMfmaBf16 || p->variant == kGqaMfmaFp8;  // reduce inside the tile kernel
    // An MLA tile is expensive (144 KB of Q in, a 256 KB partial out and back in through the reduction) and its
    // pages cost the same compute everywhere, so the queue is all equal chunks; the GQA kernels are bandwidth-bound
    // with timing that varies, so they keep a self-scheduled tail.  (Measured on the benchmark workloads.)
    const bool mla = p->variant == kMlaMfmaBf16;
    const int c0 = knob("NANOCP_PLAN_OVERHEAD_PAGES", mla ? 6 : 2, 0, 64);  // cost of a tile's Q load, combine, write-back
    const int min_pages = knob("NANOCP_PLAN_MIN_PAGES", 8, 1, 1 << 20);
    const double static_frac = knob("NANOCP_PLAN_STATIC_PCT", mla ? 100 : 85, 1, 100) / 100.0;
    const int gss_k = knob("NANOCP_PLAN_GSS_K", 2, 1, 64);
    const int snap_pct = knob("NANOCP_PLAN_SNAP_PCT", 12, 0, 50);  // measured: fewer tiles, same balance
    const int64_t M = std::max<int64_t>(1, (int64_t)num_cus * knob("NANOCP_PLAN_WGS_PER_CU", 1, 1, 16));

    // longest shards first: the big, statically sized chunks at the head of the queue then hold the long
    // shards, and the small chunks at its tail are mostly whole short requests (no partials to reduce)
    std::vector<int> order;
    int64_t units = 0;  // total cost in page units
    for (int s = 0; s < num_shards; ++s) {
      const nanocp_shard& sh = shards[s];
      if (sh.kv_end == sh.kv_begin) continue;
      order.push_back(s);
      const int64_t np = (sh.kv_end - 1) / ps - sh.kv_begin / ps + 1;
      units += (np + c0) * Hkv;
    }
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
      return shards[a].kv_end - shards[a].kv_begin > shards[b].kv_end - shards[b].kv_begin;
    });

    const bool fixed = tile_tokens > 0;
    const int64_t cap_fixed = std::max<int64_t>(1, tile_tokens / ps) + c0;
    const int64_t cap_static =
        std::max<int64_t>((int64_t)(static_frac * (double)units / (double)M + 0.999), c0 + min_pages);
    const int64_t whole_max = std::max<int64_t>(c0 + min_pages, cap_static / knob("NANOCP_PLAN_WHOLE_DIV", 2, 1, 64));
    int64_t consumed = 0;
    auto open_cap = [&](int chunk_idx) -> int64_t {
      if (fixed) return cap_fixed;
      if (!p->dynamic) return std::max<int64_t>((units + M - 1) / M, c0 + min_pages);  // one chunk per workgroup
      if (chunk_idx < M) return cap_static;
      // guided self-scheduling over what is left: ever smaller chunks even out the finish times
      return std::max<int64_t>(c0 + min_pages, (units - consumed) / (gss_k * M));
    };

    {
      int chunk = 0;
      int64_t used = 0, cap = open_cap(0);
      for (int s : order) {
        const nanocp_shard& sh = shards[s];
        const int pb = sh.kv_begin / ps, pe = (sh.kv_end - 1) / ps + 1;
        for (int h = 0; h < Hkv; ++h) {
          int pg = pb;
          while (pg < pe) {
            // tail of the queue: a short (shard, head) is kept whole so that it needs no partials
            const bool whole = !fixed && p->dynamic && chunk >= M && pg == pb && (pe - pb) + c0 <= whole_max;
            // Snapping: a cut that would leave a sliver (of the chunk, or of the (shard, head)) costs a tile and a
            // partial for little balance; within `snap` pages the cut moves to the nearer boundary instead.
            const int64_t snap = (fixed || !p->dynamic) ? 0 : cap * snap_pct / 100;
            const int64_t need = whole ? (pe - pb) + c0 : c0 + 1 + std::min<int64_t>(snap, pe - pg - 1);
            if (used > 0 && cap - used < need) {
              ++chunk;
              used = 0;
              cap = open_cap(chunk);
            }
            int take = whole ? pe - pb : (int)std::min<int64_t>(pe - pg, cap - used - c0);
            if (!whole && (pe - pg) - take <= snap) take = pe - pg;  // the rest is a sliver: keep it in this chunk

            nanocp_tile t;
            t.shard = s;
            t.kv_head = h;
            t.q_row = sh.q_row;
            t.bt_row = sh.bt_row;
            t.tok_begin = std::max(sh.kv_begin, pg * ps);
            t.tok_end = std::min(sh.kv_end, (pg + take) * ps);
            t.dst = -1;
            t.chunk = chunk;
            p->tiles.push_back(t);
            used += c0 + take;
            consumed += c0 + take;
            pg += take;
          }
        }
      }
      p->num_chunks = p->tiles.empty() ? 0 : chunk + 1;
    }
    p->launch_blocks = p->dynamic ? (int32_t)std::min<int64_t>(p->num_chunks, M) : p->num_chunks;

    p->dev_tiles.resize(p->tiles.size());
    assign_segments(p, nullptr);

    // Queue order: the statically sized chunks first, then the rest by decreasing cost (longest
    // processing time first), so that the very last chunks taken are the smallest ones.
    if (p->dynamic && !fixed && p->num_chunks > M) {
      std::vector<int64_t> cost(p->num_chunks, 0);
      for (const nanocp_tile& t : p->tiles) cost[t.chunk] += (t.tok_end - 1) / ps - t.tok_begin / ps + 1 + c0;
      std::vector<int> perm(p->num_chunks);
      for (int c = 0; c < p->num_chunks; ++c) perm[c] = c;
      std::stable_sort(perm.begin() + M, perm.end(), [&](int a, int b) { return cost[a] > cost[b]; });
      std::vector<int> new_id(p->num_chunks);
      for (int c = 0; c < p->num_chunks; ++c) new_id[perm[c]] = c;
      std::vector<size_t> idx(p->tiles.size());
      for (size_t i = 0; i < idx.size(); ++i) idx[i] = i;
      std::stable_sort(idx.begin(), idx.end(),
                       [&](size_t a, size_t b) { return new_id[p->tiles[a].chunk] < new_id[p->tiles[b].chunk]; });
      std::vector<nanocp_tile> nt(p->tiles.size());
      std::vector<DevTile> nd(p->tiles.size());
      for (size_t i = 0; i < idx.size(); ++i) {
        nt[i] = p->tiles[idx[i]];
        nt[i].chunk = new_id[nt[i].chunk];
        nd[i] = p->dev_tiles[idx[i]];
      }
      p->tiles.swap(nt);
      p->dev_tiles.swap(nd);
    }
    p->chunk_offsets.assign(p->num_chunks + 1, 0);
    for (const nanocp_tile& t : p->tiles) p->chunk_offsets[t.chunk + 1]++;
    for (int c = 0; c < p->num_chunks; ++c) p->chunk_offsets[c + 1] += p->chunk_offsets[c];
  } catch (const std::bad_alloc&) {
    delete p;
    return NANOCP_ENOMEM;
  }
  *out = p;
  return NANOCP_OK;
}

nanocp_status nanocp_plan_query(const nanocp_plan* plan, int32_t* num_tiles, int32_t* num_chunks,
                                size_t* workspace_bytes) {
  if (!plan) return NANOCP_EINVAL;
  if (num_tiles) *num_tiles = (int32_t)plan->tiles.size();
  if (num_chunks) *num_chunks = plan->num_chunks;
  if (workspace_bytes) *workspace_bytes = plan->workspace_bytes;
  return NANOCP_OK;
}

nanocp_status nanocp_plan_tiles(const nanocp_plan* plan, const nanocp_tile** tiles, int32_t* num_tiles) {
  if (!plan || !tiles || !num_tiles) return NANOCP_EINVAL;
  *tiles = plan->tiles.data();
  *num_tiles = (int32_t)plan->tiles.size();
  return NANOCP_OK;
}

nanocp_status nanocp_plan_set_final_rows(nanocp_plan* plan, const int32_t* shard_final_row, int32_t num_out) {
  if (!plan || !shard_final_row || num_out < 0) return NANOCP_EINVAL;
  if (plan->device >= 0) return NANOCP_ESTATE;  // the device copy is immutable
  for (int s = 0; s < plan->num_shards; ++s)
    if (shard_final_row[s] < -1 || shard_final_row[s] >= num_out) return NANOCP_EBOUNDS;
  try {
    assign_segments(plan, shard_final_row);
  } catch (const std::bad_alloc&) {
    return NANOCP_ENOMEM;
  }
  plan->num_final_rows = num_out;
  return NANOCP_OK;
}

size_t nanocp_bucket_plan_bytes(const nanocp_bucket* b) {
  if (!b || b->max_tiles < 0 || b->max_chunks < 0 || b->max_segs < 0 || b->max_slots < 0) return 0;
  return nanocp::image_layout(*b).total;
}

size_t nanocp_bucket_workspace_bytes(const nanocp_attn_desc* desc, const nanocp_bucket* b) {
  if (!desc || !b || desc->num_kv_heads <= 0 || b->max_slots <= 0) return 0;
  const size_t G = (size_t)(desc->num_q_heads / desc->num_kv_heads);
  return nanocp::align256((size_t)b->max_slots * G * desc->head_dim_v * sizeof(float)) +
         nanocp::align256((size_t)b->max_slots * G * sizeof(float));
}

nanocp_status nanocp_plan_pack(const nanocp_plan* plan, const nanocp_bucket* b, void* host_image, size_t image_bytes) {
  if (!plan || !b || !host_image) return NANOCP_EINVAL;
  if (b->max_tiles < 0 || b->max_chunks < 0 || b->max_segs < 0 || b->max_slots < 0) return NANOCP_EINVAL;
  const nanocp::ImageLayout L = nanocp::image_layout(*b);
  if (image_bytes < L.total) return NANOCP_EBOUNDS;
  if ((int64_t)plan->dev_tiles.size() > b->max_tiles || plan->num_chunks > b->max_chunks ||
      (int64_t)plan->segs.size() > b->max_segs || plan->num_multi_segs > b->max_segs || plan->num_slots > b->max_slots)
    return NANOCP_EBOUNDS;
  char* img = (char*)host_image;
  std::memset(img, 0, L.chunk_offsets);  // header and counters
  int32_t* hdr = (int32_t*)(img + L.header);
  hdr[0] = plan->num_chunks;
  hdr[1] = (int32_t)plan->segs.size();
  hdr[2] = plan->num_multi_segs;
  hdr[3] = plan->num_slots;
  hdr[4] = plan->variant;
  hdr[5] = plan->grouped ? 1 : 0;
  hdr[6] = plan->num_final_rows;
  std::memcpy(img + L.chunk_offsets, plan->chunk_offsets.data(), plan->chunk_offsets.size() * sizeof(int32_t));
  std::memcpy(img + L.tiles, plan->dev_tiles.data(), plan->dev_tiles.size() * sizeof(nanocp::DevTile));
  std::memcpy(img + L.segs, plan->segs.data(), plan->segs.size() * sizeof(nanocp::Seg));
  return NANOCP_OK;
}

const char* nanocp_plan_kernel(const nanocp_plan* plan) {
  if (!plan) return "";
  switch (plan->variant) {
    case kGqaMfmaBf16: return "gqa_mfma_bf16";
    case kGqaMfmaFp8: return "gqa_mfma_fp8";
    case kMlaMfmaBf16: return "mla_mfma_bf16";
    default: return "generic";
  }
}

nanocp_status nanocp_plan_upload(nanocp_plan* plan, void* stream) {
  if (!plan) return NANOCP_EINVAL;
  if (plan->device >= 0) return NANOCP_ESTATE;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return NANOCP_EHIP;
  hipStream_t st = (hipStream_t)stream;
  auto up = [&](void** dptr, const void* src, size_t bytes) -> nanocp_status {
    if (bytes == 0) return NANOCP_OK;
    if (hipMalloc(dptr, bytes) != hipSuccess) return NANOCP_ENOMEM;
    if (hipMemcpyAsync(*dptr, src, bytes, hipMemcpyHostToDevice, st) != hipSuccess) return NANOCP_EHIP;
    return NANOCP_OK;
  };
  // On a failure part-way every buffer allocated so far is released again (after the stream has drained: a copy
  // into one of them may still be in flight) and the plan stays in its not-uploaded state.
  auto fail = [&](nanocp_status s) {
    (void)hipStreamSynchronize(st);
    free_device_copy(plan);
    return s;
  };
  nanocp_status s;
  if ((s = up((void**)&plan->d_tiles, plan->dev_tiles.data(), plan->dev_tiles.size() * sizeof(DevTile))) != NANOCP_OK) return fail(s);
  if ((s = up((void**)&plan->d_chunk_offsets, plan->chunk_offsets.data(), plan->chunk_offsets.size() * sizeof(int32_t))) != NANOCP_OK) return fail(s);
  if ((s = up((void**)&plan->d_segs, plan->segs.data(), plan->segs.size() * sizeof(Seg))) != NANOCP_OK) return fail(s);
  {
    const size_t sync_bytes = (size_t)(kSyncSegBase + plan->num_multi_segs) * sizeof(int32_t);
    if (hipMalloc((void**)&plan->d_sync, sync_bytes) != hipSuccess) return fail(NANOCP_ENOMEM);
    if (hipMemsetAsync(plan->d_sync, 0, sync_bytes, st) != hipSuccess) return fail(NANOCP_EHIP);
  }
  // the host vectors must outlive the async copies: they live as long as the plan, and destroy synchronises
  plan->device = dev;
  return NANOCP_OK;
}

void nanocp_plan_destroy(nanocp_plan* plan) {
  if (!plan) return;
  if (plan->device >= 0) {
    // synchronise and free on the device that holds the copy, whatever device is current for the caller
    int cur = -1;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    const bool switched = have_cur && cur != plan->device && hipSetDevice(plan->device) == hipSuccess;
    (void)hipDeviceSynchronize();
    free_device_copy(plan);
    if (switched) (void)hipSetDevice(cur);
  }
  delete plan;
}

const char* nanocp_status_str(nanocp_status s) {
  switch (s) {
    case NANOCP_OK: return "ok";
    case NANOCP_EINVAL: return "invalid argument";
    case NANOCP_ESHAPE: return "inconsistent shape";
    case NANOCP_EBOUNDS: return "out of bounds";
    case NANOCP_EUNSUPPORTED: return "unsupported configuration";
    case NANOCP_ENOMEM: return "out of memory";
    case NANOCP_EHIP: return "HIP runtime error";
    case NANOCP_ESTATE: return "plan in wrong state";
    default: return "unknown status";
  }
}

}  // extern "C"

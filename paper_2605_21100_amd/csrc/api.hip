// Device entry points: nanocp_decode_attn_partial(_timed), nanocp_merge_partials, and the two small
// LSE-combine kernels (intra-shard tile reduction, cross-shard merge).
// Paper: Data Plane, Phase 2 (partial attention + LSE) and Phase 4 (LSE-based merging).
#include <hip/hip_runtime.h>

#include <mutex>

#include "epilogue.h"
#include "nanocp_debug.h"
#include "plan.h"

namespace nanocp {

hipError_t launch_generic(const nanocp_attn_desc& d, const KParams& p, int num_blocks, hipStream_t st);
hipError_t launch_gqa_mfma(int variant, const KParams& p, int num_blocks, hipStream_t st);
hipError_t launch_mla_mfma(const KParams& p, int num_blocks, hipStream_t st);
hipError_t launch_mla_reduce(const KParams& p, const Seg* segs, int num_segs, hipStream_t st);

namespace {

// LSE-combine of the tile partials of one (shard, kv head): the same operator as the Phase 4 merge,
// applied inside the instance (used by the variants that do not reduce inside the tile kernel, and to
// fill empty shards).  One thread per 4 output dims; parts are taken 8 at a time with a running maximum.
__global__ __launch_bounds__(kThreads) void reduce_tiles_kernel(const Seg* __restrict__ segs,
                                                                const float* __restrict__ ws_o,
                                                                const float* __restrict__ ws_lse,
                                                                float* __restrict__ out_o, float* __restrict__ out_lse,
                                                                void* __restrict__ final_out,
                                                                float* __restrict__ final_lse, int final_kind,
                                                                float out_inv_scale,
                                                                const int32_t* __restrict__ header, int Hq, int G,
                                                                int Dv) {
  if (header && (int)blockIdx.x >= header[1]) return;  // plan image: launched for the bucket's capacity
  const Seg sg = segs[blockIdx.x];
  const int q4 = Dv >> 2;
  const int i4 = blockIdx.y * kThreads + threadIdx.x;
  if (i4 >= G * q4) return;
  const int g = i4 / q4;
  const size_t row = (size_t)G * Dv;
  float top = -INFINITY, tot = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < sg.n_parts; k0 += 8) {
    float li[8];
    float4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const size_t slot = (size_t)(sg.slot_begin + min(k0 + j, sg.n_parts - 1));
      li[j] = ws_lse[slot * G + g];
      v[j] = *(const float4*)(ws_o + slot * row + (size_t)i4 * 4);
    }
    float bm = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (k0 + j >= sg.n_parts) li[j] = -INFINITY;
      bm = fmaxf(bm, li[j]);
    }
    const float nt = fmaxf(top, bm);  // finite: tile partials are never empty
    const float sc = expf(top - nt);
    tot *= sc;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] *= sc;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool live = li[j] != -INFINITY;
      const float w = live ? expf(li[j] - nt) : 0.f;
      tot += w;
      acc[0] = fmaf(w, live ? v[j].x : 0.f, acc[0]);
      acc[1] = fmaf(w, live ? v[j].y : 0.f, acc[1]);
      acc[2] = fmaf(w, live ? v[j].z : 0.f, acc[2]);
      acc[3] = fmaf(w, live ? v[j].w : 0.f, acc[3]);
    }
    top = nt;
  }
  const bool empty = sg.n_parts == 0;
  const float inv = empty ? 0.f : 1.f / tot;
  const float lse = empty ? -INFINITY : top + logf(tot);
  if ((i4 % q4) == 0) out_lse[(size_t)sg.shard * Hq + (size_t)sg.kv_head * G + g] = lse;
  if (final_out && sg.final_row >= 0) {
    // the shard is the only partial of its output row: final form, no merge needed
    const size_t fi = ((size_t)sg.final_row * Hq + (size_t)sg.kv_head * G) * Dv + (size_t)i4 * 4;
    const float o4[4] = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
    store_final<4>(final_out, fi, final_kind, out_inv_scale, o4);
    if (final_lse && (i4 % q4) == 0) final_lse[(size_t)sg.final_row * Hq + (size_t)sg.kv_head * G + g] = lse;
    return;
  }
  float* o = out_o + ((size_t)sg.shard * Hq + (size_t)sg.kv_head * G) * Dv + (size_t)i4 * 4;
  *(float4*)o = make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
}

// Phase 4: per (output, head) merge of the partials named by the CSR lists.
// One thread per 4 consecutive output dims, so each thread has a single short chain of dependent loads.
__global__ __launch_bounds__(kThreads) void merge_kernel(const float* __restrict__ o_parts,
                                                         const float* __restrict__ lse_parts,
                                                         const int32_t* __restrict__ part_offsets,
                                                         const int32_t* __restrict__ part_index,
                                                         const int32_t* __restrict__ out_rows,
                                                         const int32_t* __restrict__ num_out_dev, void* __restrict__ out,
                                                         float* __restrict__ out_lse, int out_kind, float out_inv_scale,
                                                         int Hq, int Dv) {
  if (num_out_dev && (int)blockIdx.x >= *num_out_dev) return;  // launched for a capacity, the count is on the device
  const int b = part_offsets[blockIdx.x], e = part_offsets[blockIdx.x + 1];
  const int r = out_rows ? out_rows[blockIdx.x] : (int)blockIdx.x;  // output row of this list
  const int q4 = Dv >> 2;  // float4 groups per head (Dv % 4 == 0 is checked by the host)
  const int i4 = blockIdx.y * kThreads + threadIdx.x;
  if (i4 >= Hq * q4) return;
  const int a = i4 / q4;
  const size_t row = (size_t)Hq * Dv;
  float top = -INFINITY, tot = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (e - b == 1) {
    // a request held by one instance (the common case): its partial is the final output
    const size_t pi = part_index ? (size_t)part_index[b] : (size_t)b;
    const float li = lse_parts[pi * Hq + a];
    const float4 v = *(const float4*)(o_parts + pi * row + (size_t)i4 * 4);
    if (li != -INFINITY) {
      top = li, tot = 1.f;
      acc[0] = v.x, acc[1] = v.y, acc[2] = v.z, acc[3] = v.w;
    }
  } else {
    // One pass with a running maximum, 8 parts at a time: the index loads of a batch are issued together,
    // then its LSE and output loads, so a request with d <= 8 partials costs two memory round trips.
    for (int k0 = b; k0 < e; k0 += 8) {
      size_t pi[8];
      float li[8];
      float4 v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = min(k0 + j, e - 1);
        pi[j] = part_index ? (size_t)part_index[k] : (size_t)k;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        li[j] = lse_parts[pi[j] * Hq + a];
        v[j] = *(const float4*)(o_parts + pi[j] * row + (size_t)i4 * 4);
      }
      float bm = -INFINITY;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (k0 + j >= e) li[j] = -INFINITY;  // padding of the last batch
        bm = fmaxf(bm, li[j]);
      }
      const float nt = fmaxf(top, bm);
      if (nt != -INFINITY) {
        const float sc = expf(top - nt);  // top = -inf on the first live batch: exp(-inf) = 0
        tot *= sc;
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] *= sc;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool live = li[j] != -INFINITY;  // an empty partial's output is ignored whatever it holds
          const float w = live ? expf(li[j] - nt) : 0.f;
          tot += w;
          acc[0] = fmaf(w, live ? v[j].x : 0.f, acc[0]);
          acc[1] = fmaf(w, live ? v[j].y : 0.f, acc[1]);
          acc[2] = fmaf(w, live ? v[j].z : 0.f, acc[2]);
          acc[3] = fmaf(w, live ? v[j].w : 0.f, acc[3]);
        }
        top = nt;
      }
    }
  }
  float lse = -INFINITY;
  if (top != -INFINITY) {
    if (tot != 1.f) {
      const float inv = 1.f / tot;
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] *= inv;
    }
    lse = top + logf(tot);
  }
  const size_t oi = (size_t)r * row + (size_t)i4 * 4;
  store_final<4>(out, oi, out_kind, out_inv_scale, acc);
  if (out_lse && (i4 % q4) == 0) out_lse[(size_t)r * Hq + a] = lse;
}

// the tile kernel of the variant, then the reduction kernel over `num_segs` segments (0 = none)
nanocp_status launch_tiles_and_reduce(const nanocp_attn_desc& d, int variant, const KParams& p, int blocks,
                                      const Seg* d_segs, int num_segs, hipStream_t st) {
  if (blocks > 0) {
    hipError_t e;
    if (variant == kGeneric)
      e = launch_generic(d, p, blocks, st);
    else if (variant == kMlaMfmaBf16)
      e = launch_mla_mfma(p, blocks, st);
    else
      e = launch_gqa_mfma(variant, p, blocks, st);
    if (e != hipSuccess) return NANOCP_EHIP;
  }
  // the GQA MFMA variants reduce inside the tile kernel; their only segments are (shard, head) pairs without tokens,
  // which the tile kernel fills itself.  The MLA variant has a reduction kernel of its own (its partials are stored
  // in register order); the generic variant's segments go through reduce_tiles_kernel.
  const bool fills_own = blocks > 0 && (variant == kGqaMfmaBf16 || variant == kGqaMfmaFp8);
  if (num_segs > 0 && variant == kMlaMfmaBf16) {
    if (launch_mla_reduce(p, d_segs, num_segs, st) != hipSuccess) return NANOCP_EHIP;
  } else if (num_segs > 0 && !fills_own) {
    if (p.Dv % 4) return NANOCP_ESHAPE;
    const unsigned per_seg = (unsigned)((p.G * (p.Dv / 4) + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(reduce_tiles_kernel, dim3((unsigned)num_segs, per_seg), dim3(kThreads), 0, st, d_segs, p.ws_o,
                       p.ws_lse, p.out_o, p.out_lse, p.final_out, p.final_lse, p.final_kind, p.out_inv_scale, p.header, p.Hq, p.G, p.Dv);
    if (hipGetLastError() != hipSuccess) return NANOCP_EHIP;
  }
  return NANOCP_OK;
}

nanocp_status run_partial(const nanocp_plan* plan, const void* q, const void* k_pool, const void* v_pool,
                          const float* k_scale, const float* v_scale, const int32_t* block_table, float* out_o,
                          float* out_lse, void* workspace, size_t workspace_bytes, uint64_t* tile_clock, void* final_out,
                          int32_t final_dtype, float* final_lse, void* stream) {
  if (!plan) return NANOCP_EINVAL;
  if (final_out) {
    if (!final_dtype_ok(final_dtype)) return NANOCP_EUNSUPPORTED;
    if (plan->num_final_rows == 0) return NANOCP_ESTATE;  // nanocp_plan_set_final_rows was not called
    if ((uintptr_t)final_out & 15) return NANOCP_EINVAL;
    if (plan->desc.head_dim_v % 8) return NANOCP_ESHAPE;
  }
  if (plan->grouped && !final_out) return NANOCP_ESTATE;  // grouped shards have no per-shard result to deliver
  const nanocp_attn_desc& d = plan->desc;
  if (plan->num_shards == 0) return NANOCP_OK;
  if (!q || !k_pool || !block_table || !out_o || !out_lse) return NANOCP_EINVAL;
  if (d.kind == NANOCP_GQA && !v_pool) return NANOCP_EINVAL;
  if (d.kv_dtype == NANOCP_FP8_E4M3 && (!k_scale || !v_scale)) return NANOCP_EINVAL;
  if (plan->device < 0) return NANOCP_ESTATE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return NANOCP_EHIP;
  if (dev != plan->device) return NANOCP_ESTATE;
  if (plan->workspace_bytes > 0 && (!workspace || workspace_bytes < plan->workspace_bytes)) return NANOCP_EBOUNDS;
  if (((uintptr_t)q | (uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)workspace | (uintptr_t)out_o) & 15)
    return NANOCP_EINVAL;

  hipStream_t st = (hipStream_t)stream;
  const int G = d.num_q_heads / d.num_kv_heads;
  KParams p;
  p.q = q;
  p.k_pool = k_pool;
  p.v_pool = v_pool;
  p.k_scale = k_scale;
  p.v_scale = v_scale;
  p.block_table = block_table;
  p.out_o = out_o;
  p.out_lse = out_lse;
  const size_t o_bytes = ((size_t)plan->num_slots * G * d.head_dim_v * sizeof(float) + 255) & ~(size_t)255;
  p.ws_o = (float*)workspace;
  p.ws_lse = (float*)((char*)workspace + o_bytes);
  p.tiles = plan->d_tiles;
  p.chunk_offsets = plan->d_chunk_offsets;
  p.sync = plan->d_sync;
  p.num_chunks = plan->num_chunks;
  p.segs = plan->d_segs;
  p.num_segs = (int)plan->segs.size();
  p.header = nullptr;
  p.tile_clock = tile_clock;
  p.final_out = final_out;
  p.final_lse = final_out ? final_lse : nullptr;
  p.final_kind = final_out ? final_dtype : NANOCP_F32;
  p.out_inv_scale = out_inv_scale_of(d);
  p.variant = plan->variant;
  p.Hq = d.num_q_heads;
  p.Hkv = d.num_kv_heads;
  p.G = G;
  p.Dk = d.head_dim_qk;
  p.Dv = d.head_dim_v;
  p.ps = d.page_size;
  p.max_blocks = plan->max_blocks;
  p.kind = d.kind;
  p.scale = d.softmax_scale;

  return launch_tiles_and_reduce(d, plan->variant, p, plan->num_chunks > 0 ? plan->launch_blocks : 0, plan->d_segs,
                                 (int)plan->segs.size(), st);
}

// Phase 2 driven by a plan image on the device: every count is read from the image's header by the kernels.
nanocp_status run_image(const nanocp_attn_desc* desc, const nanocp_bucket* bucket, const void* device_image,
                        int32_t num_cus, int32_t max_blocks_per_row, const void* q, const void* k_pool,
                        const void* v_pool, const float* k_scale, const float* v_scale, const int32_t* block_table,
                        float* out_o, float* out_lse, void* workspace, size_t workspace_bytes, void* final_out,
                        int32_t final_dtype, float* final_lse, void* stream) {
  if (!desc || !bucket || !device_image || num_cus <= 0 || max_blocks_per_row < 0) return NANOCP_EINVAL;
  if (bucket->max_tiles < 0 || bucket->max_chunks < 0 || bucket->max_segs < 0 || bucket->max_slots < 0)
    return NANOCP_EINVAL;
  const nanocp_attn_desc& d = *desc;
  const nanocp_status ds = check_desc(d);  // the kernels' LDS and register arrays are sized for the checked limits
  if (ds != NANOCP_OK) return ds;
  if (d.head_dim_v % 4) return NANOCP_ESHAPE;
  if (!q || !k_pool || !block_table || !out_o || !out_lse) return NANOCP_EINVAL;
  if (d.kind == NANOCP_GQA && !v_pool) return NANOCP_EINVAL;
  if (d.kv_dtype == NANOCP_FP8_E4M3 && (!k_scale || !v_scale)) return NANOCP_EINVAL;
  if (final_out && !final_dtype_ok(final_dtype)) return NANOCP_EUNSUPPORTED;
  if (final_out && d.head_dim_v % 8) return NANOCP_ESHAPE;
  const size_t ws_need = nanocp_bucket_workspace_bytes(desc, bucket);
  if (ws_need > 0 && (!workspace || workspace_bytes < ws_need)) return NANOCP_EBOUNDS;
  if (((uintptr_t)q | (uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)workspace | (uintptr_t)out_o |
       (uintptr_t)final_out) & 15)
    return NANOCP_EINVAL;
  if ((uintptr_t)device_image & 255) return NANOCP_EINVAL;
  const int variant = pick_variant(d);
  const ImageLayout L = image_layout(*bucket);
  const char* img = (const char*)device_image;
  const int G = d.num_q_heads / d.num_kv_heads;
  KParams p;
  p.q = q;
  p.k_pool = k_pool;
  p.v_pool = v_pool;
  p.k_scale = k_scale;
  p.v_scale = v_scale;
  p.block_table = block_table;
  p.out_o = out_o;
  p.out_lse = out_lse;
  p.ws_o = (float*)workspace;
  p.ws_lse = (float*)((char*)workspace + align256((size_t)bucket->max_slots * G * d.head_dim_v * sizeof(float)));
  p.tiles = (const DevTile*)(img + L.tiles);
  p.chunk_offsets = (const int32_t*)(img + L.chunk_offsets);
  p.sync = (int32_t*)(img + L.sync);
  p.num_chunks = 0;
  p.segs = (const Seg*)(img + L.segs);
  p.num_segs = 0;
  p.header = (const int32_t*)(img + L.header);
  p.tile_clock = nullptr;
  p.final_out = final_out;
  p.final_lse = final_out ? final_lse : nullptr;
  p.final_kind = final_out ? final_dtype : NANOCP_F32;
  p.out_inv_scale = out_inv_scale_of(d);
  p.variant = variant;
  p.Hq = d.num_q_heads;
  p.Hkv = d.num_kv_heads;
  p.G = G;
  p.Dk = d.head_dim_qk;
  p.Dv = d.head_dim_v;
  p.ps = d.page_size;
  p.max_blocks = max_blocks_per_row;
  p.kind = d.kind;
  p.scale = d.softmax_scale;
  // dynamic variants: one workgroup per compute unit pulls chunks; the generic kernel runs one workgroup per chunk
  const int blocks = variant == kGeneric ? bucket->max_chunks : num_cus;
  return launch_tiles_and_reduce(d, variant, p, blocks, (const Seg*)(img + L.segs), bucket->max_segs,
                                 (hipStream_t)stream);
}

// Scratch of nanocp_decode_attn_partial_image_static: the tile partials ([slots, G, Dv] outputs, then [slots, G]
// LSEs) of one launch.  The array's name is a host-side stand-in, not a device address: the address each device
// holds its copy at is looked up once per device (with that device current) and only that pointer is handed to
// kernels.  Nothing in it has to start at zero: every slot a launch reads was written by the same launch.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

}  // namespace
}  // namespace nanocp

static __device__ __align__(256) unsigned char nanocp_static_scratch[nanocp::kStaticScratchBytes];

namespace nanocp {
namespace {

nanocp_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return NANOCP_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return NANOCP_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(nanocp_static_scratch)) != hipSuccess || !ptr) return NANOCP_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return NANOCP_OK;
}

}  // namespace
}  // namespace nanocp

extern "C" {

nanocp_status nanocp_decode_attn_partial(const nanocp_plan* plan, const void* q, const void* k_pool,
                                         const void* v_pool, const float* k_scale, const float* v_scale,
                                         const int32_t* block_table, float* out_o, float* out_lse, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  return nanocp::run_partial(plan, q, k_pool, v_pool, k_scale, v_scale, block_table, out_o, out_lse, workspace,
                             workspace_bytes, nullptr, nullptr, NANOCP_F32, nullptr, stream);
}

nanocp_status nanocp_decode_attn_partial_final(const nanocp_plan* plan, const void* q, const void* k_pool,
                                               const void* v_pool, const float* k_scale, const float* v_scale,
                                               const int32_t* block_table, float* out_o, float* out_lse,
                                               void* workspace, size_t workspace_bytes, void* final_out,
                                               int32_t final_dtype, float* final_lse, void* stream) {
  if (!final_out) return NANOCP_EINVAL;
  return nanocp::run_partial(plan, q, k_pool, v_pool, k_scale, v_scale, block_table, out_o, out_lse, workspace,
                             workspace_bytes, nullptr, final_out, final_dtype, final_lse, stream);
}

nanocp_status nanocp_decode_attn_partial_image(const nanocp_attn_desc* desc, const nanocp_bucket* bucket,
                                               const void* device_image, int32_t num_cus, int32_t max_blocks_per_row,
                                               const void* q, const void* k_pool, const void* v_pool,
                                               const float* k_scale, const float* v_scale,
                                               const int32_t* block_table, float* out_o, float* out_lse,
                                               void* workspace, size_t workspace_bytes, void* final_out,
                                               int32_t final_dtype, float* final_lse, void* stream) {
  if (num_cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NANOCP_EHIP;
    num_cus = prop.multiProcessorCount;
  }
  return nanocp::run_image(desc, bucket, device_image, num_cus, max_blocks_per_row, q, k_pool, v_pool, k_scale,
                           v_scale, block_table, out_o, out_lse, workspace, workspace_bytes, final_out, final_dtype,
                           final_lse, stream);
}

nanocp_status nanocp_decode_attn_partial_image_static(const nanocp_attn_desc* desc, const nanocp_bucket* bucket,
                                                      const void* device_image, int32_t num_cus,
                                                      int32_t max_blocks_per_row, const void* q, const void* k_pool,
                                                      const void* v_pool, const float* k_scale, const float* v_scale,
                                                      const int32_t* block_table, float* out_o, float* out_lse,
                                                      void* final_out, int32_t final_dtype, float* final_lse,
                                                      void* stream) {
  using namespace nanocp;
  if (!desc || !bucket) return NANOCP_EINVAL;
  if (num_cus <= 0) return NANOCP_EINVAL;  // no device query on this path: the caller states the launch width
  const size_t need = nanocp_bucket_workspace_bytes(desc, bucket);
  if (need > kStaticScratchBytes) return NANOCP_EBOUNDS;  // the bucket's tile partials do not fit the static scratch
  void* ws = nullptr;
  const nanocp_status s = static_scratch(&ws);
  if (s != NANOCP_OK) return s;
  return run_image(desc, bucket, device_image, num_cus, max_blocks_per_row, q, k_pool, v_pool, k_scale, v_scale,
                   block_table, out_o, out_lse, ws, kStaticScratchBytes, final_out, final_dtype, final_lse, stream);
}

nanocp_status nanocp_decode_attn_partial_timed(const nanocp_plan* plan, const void* q, const void* k_pool,
                                               const void* v_pool, const float* k_scale, const float* v_scale,
                                               const int32_t* block_table, float* out_o, float* out_lse,
                                               void* workspace, size_t workspace_bytes, uint64_t* tile_clock,
                                               void* stream) {
  if (!tile_clock) return NANOCP_EINVAL;
  return nanocp::run_partial(plan, q, k_pool, v_pool, k_scale, v_scale, block_table, out_o, out_lse, workspace,
                             workspace_bytes, tile_clock, nullptr, NANOCP_F32, nullptr, stream);
}

nanocp_status nanocp_merge_partials(const nanocp_attn_desc* desc, const float* o_parts, const float* lse_parts,
                                    const int32_t* part_offsets, const int32_t* part_index, int32_t num_out, void* out,
                                    int32_t out_dtype, float* out_lse, void* stream) {
  return nanocp_merge_partials_rows(desc, o_parts, lse_parts, part_offsets, part_index, num_out, nullptr, out, out_dtype,
                                    out_lse, stream);
}

nanocp_status nanocp_merge_partials_rows(const nanocp_attn_desc* desc, const float* o_parts, const float* lse_parts,
                                         const int32_t* part_offsets, const int32_t* part_index, int32_t num_out,
                                         const int32_t* out_rows, void* out, int32_t out_dtype, float* out_lse,
                                         void* stream) {
  return nanocp_merge_partials_dyn(desc, o_parts, lse_parts, part_offsets, part_index, num_out, nullptr, out_rows, out,
                                   out_dtype, out_lse, stream);
}

nanocp_status nanocp_merge_partials_dyn(const nanocp_attn_desc* desc, const float* o_parts, const float* lse_parts,
                                        const int32_t* part_offsets, const int32_t* part_index, int32_t num_out,
                                        const int32_t* num_out_dev, const int32_t* out_rows, void* out,
                                        int32_t out_dtype, float* out_lse, void* stream) {
  if (!desc || num_out < 0) return NANOCP_EINVAL;
  if (desc->num_q_heads <= 0 || desc->head_dim_v <= 0) return NANOCP_EINVAL;
  if (!nanocp::final_dtype_ok(out_dtype)) return NANOCP_EUNSUPPORTED;
  if (num_out == 0) return NANOCP_OK;
  if (!o_parts || !lse_parts || !part_offsets || !out) return NANOCP_EINVAL;
  const int Hq = desc->num_q_heads, Dv = desc->head_dim_v;
  if (Dv % 4) return NANOCP_ESHAPE;
  if (((uintptr_t)o_parts | (uintptr_t)out) & 15) return NANOCP_EINVAL;
  const int per_out = (Hq * (Dv / 4) + nanocp::kThreads - 1) / nanocp::kThreads;
  dim3 grid((unsigned)num_out, (unsigned)per_out);
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(nanocp::merge_kernel, grid, dim3(nanocp::kThreads), 0, st, o_parts, lse_parts, part_offsets,
                     part_index, out_rows, num_out_dev, out, out_lse, out_dtype, nanocp::out_inv_scale_of(*desc), Hq, Dv);
  return hipGetLastError() == hipSuccess ? NANOCP_OK : NANOCP_EHIP;
}

}  // extern "C"

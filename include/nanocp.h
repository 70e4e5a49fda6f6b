/*
 * nanocp.h -- C ABI of the MI355X (gfx950) DCP decode-attention hot path.
 *
 * One GPU's share of a decode step under request-level dynamic context parallelism
 * (paper: Data Plane, "Decoupled Data-Path Design", Phases 2 and 4):
 *   Phase 2  every KV-binding instance computes, for each routed query, a partial attention
 *            output over its LOCAL paged KV shard plus the log-sum-exp (LSE) of the shard's scores;
 *   Phase 4  the MoE-binding instance merges the partials of a request into exact attention.
 * The per-instance inputs are the ones Alg. 2 pools: routed Q, block table, attention lengths
 * (here: token ranges), the local paged KV; the outputs are Res and LSE.
 *
 * All pointers marked DEVICE are HIP device pointers owned by the caller (any allocator);
 * pointers marked HOST are ordinary host memory.  Device calls are asynchronous on the given
 * hipStream_t (passed as void*; NULL = the default stream) and never synchronise or allocate;
 * only nanocp_plan_upload allocates (the plan's device copy, freed by nanocp_plan_destroy).
 * Every function returns a nanocp_status; nothing throws or aborts.  Contents of device
 * buffers (block-table entries, page ids) are NOT validated: pages named by the block table
 * for a shard's token range must exist in the pools.
 *
 * Memory layouts.  x = 16 bytes / sizeof(kv element): 4 (f32), 8 (bf16), 16 (fp8).
 *   q            [num_q_rows, Hq, Dk]              q_dtype (f32 or bf16)
 *   GQA k_pool   [num_pages, Hkv, ps/4x, Dk/x, 4x, x]  a page of one kv head is ps/4x groups of 4x token slots; a
 *                                                  group is Dk/x runs of 4x 16-byte vectors, vector (c, w) holding
 *                                                  dims [c*x, c*x+x) of the group's slot w
 *   GQA v_pool   [num_pages, Hkv, ps/x, Dv, x]     vector (u, c) holds dim c of x tokens.  Token slots are taken
 *                                                  in groups of 4x; slot w = 16b + 4g + i (i < 4, g < 4) of group n
 *                                                  is element 4b + i of vector u = 4n + g.  (For f32 this is plain
 *                                                  order; for bf16/fp8 it is the order in which the matrix cores
 *                                                  produce the scores, see csrc/gqa_mfma.hip.)  ps % 4x == 0.
 *   MLA k_pool   [num_pages, ps, Dk]               one latent row per token; V = its first Dv dims; v_pool NULL
 *   k_scale, v_scale [num_pages, Hkv] float        fp8 only: value = e4m3(byte) * scale   (OCP E4M3FN)
 *   block_table  [num_bt_rows, max_blocks_per_row] int32 physical page ids; entries beyond a
 *                                                  shard's range are never read
 *   out_o        [num_shards, Hq, Dv] float        partial output, normalised over the shard's own tokens
 *   out_lse      [num_shards, Hq]     float        natural-log LSE of the shard's scaled scores
 * An empty shard (kv_begin == kv_end) yields out_o = 0, out_lse = -inf.  Token slots of a page
 * outside [kv_begin, kv_end) may hold anything (NaN included); they are masked.
 *
 * Kernels.  Matrix-core (MFMA) tile kernels exist for exactly these shapes:
 *   GQA  q bf16, kv bf16 or fp8, Hq / Hkv = 16, Dk = Dv = 128, ps = 64      ("gqa_mfma_bf16", "gqa_mfma_fp8")
 *   MLA  q bf16, kv bf16, Hq = 128 or 64, Dk = 576, Dv = 512, ps = 64,      ("mla_mfma_bf16")
 *        softmax_scale > 0 and finite.  This kernel multiplies P.V in fp16: latent values beyond fp16's range
 *        (|v| > 65504) saturate, and scores are assumed to lie within +-2^30 / log2(e).
 * Every other supported shape (any head counts, Dk <= 576, Dv <= 512, any page size the layout admits, f32 / bf16 /
 * fp8 KV; fp8 MLA is not supported at all) runs a plain fp32 kernel ("generic") that is correct but orders of
 * magnitude slower; nanocp_plan_kernel tells which one a plan uses.
 */
#ifndef NANOCP_H
#define NANOCP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  NANOCP_OK = 0,
  NANOCP_EINVAL = 1,       /* null pointer, negative size, kv_end < kv_begin, bad enum */
  NANOCP_ESHAPE = 2,       /* Hq not a multiple of Hkv, Dk not a multiple of x, GQA page size not a multiple of 4x,
                              MLA with Hkv != 1 or Dv > Dk */
  NANOCP_EBOUNDS = 3,      /* shard range beyond max_blocks*ps, q_row/bt_row out of range, workspace too small */
  NANOCP_EUNSUPPORTED = 4, /* dtype combination or shape no compiled kernel handles */
  NANOCP_ENOMEM = 5,
  NANOCP_EHIP = 6,         /* a HIP runtime call or kernel launch failed */
  NANOCP_ESTATE = 7        /* plan not uploaded, or uploaded on another device */
} nanocp_status;

typedef enum { NANOCP_F32 = 0, NANOCP_BF16 = 1, NANOCP_FP8_E4M3 = 2 } nanocp_dtype;
typedef enum { NANOCP_GQA = 0, NANOCP_MLA = 1 } nanocp_kind;

/* Attention problem shape.  Supported element types: (q,kv) = (f32,f32), (bf16,bf16), (bf16,fp8). */
typedef struct {
  int32_t kind;          /* nanocp_kind */
  int32_t q_dtype;       /* nanocp_dtype */
  int32_t kv_dtype;      /* nanocp_dtype */
  int32_t num_q_heads;   /* Hq */
  int32_t num_kv_heads;  /* Hkv (1 for MLA) */
  int32_t head_dim_qk;   /* Dk */
  int32_t head_dim_v;    /* Dv (MLA: Dv <= Dk) */
  int32_t page_size;     /* ps, tokens per page */
  float softmax_scale;   /* score = softmax_scale * <q, k> */
  float out_scale;       /* FP8 output rows only (out_dtype / final_dtype = NANOCP_FP8_E4M3): the stored code is
                            e4m3(value * (1 / out_scale)), the reciprocal rounded to float once, the product rounded to
                            nearest even and saturating at +-448 -- a static scale the caller supplies, as consumers
                            of fp8 activations do.  0 means 1.  Ignored otherwise. */
} nanocp_attn_desc;

/* One shard entry = one row of the attention batch of this instance: a whole local request, or
 * the locally held slice of a long request (the paper's per-instance KV partition).
 * Token positions are relative to page 0 of block-table row bt_row and need not be page aligned. */
typedef struct {
  int32_t q_row;     /* row of q holding the routed query */
  int32_t bt_row;    /* row of block_table */
  int32_t kv_begin;  /* first token */
  int32_t kv_end;    /* one past the last token */
} nanocp_shard;

/* One tile of the work-list: a page-aligned piece of one (shard, kv head), run by one workgroup
 * (`chunk`).  Exposed read-only for inspection and tests. */
typedef struct {
  int32_t shard;
  int32_t kv_head;
  int32_t q_row;
  int32_t bt_row;
  int32_t tok_begin;
  int32_t tok_end;
  int32_t dst;     /* >= 0: partial slot in the workspace, reduced later; -1: the (shard, head) has a single tile
                      that writes out_o / out_lse directly */
  int32_t chunk;   /* work-queue entry the tile belongs to */
} nanocp_tile;

typedef struct nanocp_plan nanocp_plan; /* opaque, library-owned */

/*
 * nanocp_plan_create -- build the split-KV tile work-list for one batch composition (HOST only).
 * The one-GPU analogue of the paper's balance objective (Dual-balanced Scheduling, WaterFill:
 * minimise the peak load): the page list of all (shard, kv head) pairs, longest shard first, is cut
 * into chunks that workgroups pull from a queue: first one big chunk of equal cost per workgroup
 * (~85 % of the work), then ever smaller ones that even out the finish times.  A very long shard is
 * thereby spread over many workgroups while short requests are packed several to a chunk.  Cuts fall
 * on page boundaries.
 *   shards            HOST, [num_shards]
 *   tile_tokens       0 = automatic (as above); > 0: every chunk holds at most this many tokens
 *   num_cus           compute units to plan for; 0 = query the current HIP device
 *   out               receives the plan; release with nanocp_plan_destroy
 * Errors: EINVAL, ESHAPE, EBOUNDS, EUNSUPPORTED, ENOMEM; EHIP only if num_cus == 0 and no device.
 */
nanocp_status nanocp_plan_create(const nanocp_attn_desc* desc, const nanocp_shard* shards, int32_t num_shards,
                                 int32_t num_q_rows, int32_t num_bt_rows, int32_t max_blocks_per_row,
                                 int32_t tile_tokens, int32_t num_cus, nanocp_plan** out);

/* Sizes the caller needs: number of tiles, number of chunks (entries of the work queue; at most
 * 1 workgroup per compute unit is launched and pulls them in order) and the bytes of DEVICE workspace
 * nanocp_decode_attn_partial requires (may be 0). Any out pointer may be NULL. */
nanocp_status nanocp_plan_query(const nanocp_plan* plan, int32_t* num_tiles, int32_t* num_chunks,
                                size_t* workspace_bytes);

/* HOST view of the tile list (valid until the plan is destroyed). */
nanocp_status nanocp_plan_tiles(const nanocp_plan* plan, const nanocp_tile** tiles, int32_t* num_tiles);

/* Name of the kernel variant the plan dispatches to ("gqa_mfma_bf16", "gqa_mfma_fp8", "mla_mfma_bf16", "generic"). */
const char* nanocp_plan_kernel(const nanocp_plan* plan);

/* Copy the work-list to the current device (allocates; asynchronous on `stream`). Call once per plan. */
nanocp_status nanocp_plan_upload(nanocp_plan* plan, void* stream);

void nanocp_plan_destroy(nanocp_plan* plan);

/*
 * nanocp_decode_attn_partial -- Phase 2: partial attention + LSE for every shard entry of the plan.
 *   q, k_pool, v_pool, k_scale, v_scale, block_table   DEVICE, layouts above (v_pool NULL for MLA,
 *                                                      scales NULL unless fp8); 16-byte aligned
 *   out_o, out_lse                                     DEVICE, written for every shard
 *   workspace                                          DEVICE scratch of at least the queried size
 *                                                      (16-byte aligned; contents need not be preserved)
 * One launch on `stream` for the GQA MFMA variants (the workgroup that delivers the last tile of a (shard, head)
 * also reduces its tile partials, and empty shards are filled by the same kernel); the MLA and generic variants
 * add a small reduction launch.  A plan must not be run concurrently on two streams: launches share the plan's
 * work-queue counters.
 * Errors: EINVAL (null), ESTATE (plan not uploaded), EBOUNDS (workspace too small), EHIP.
 */
nanocp_status nanocp_decode_attn_partial(const nanocp_plan* plan, const void* q, const void* k_pool,
                                         const void* v_pool, const float* k_scale, const float* v_scale,
                                         const int32_t* block_table, float* out_o, float* out_lse,
                                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * nanocp_merge_partials -- Phase 4: LSE-based merge.  For output r and head a, over the partials
 * i in part_index[part_offsets[r] .. part_offsets[r+1]):
 *     LSE = log sum_i exp(lse_i),   O = sum_i exp(lse_i - LSE) * o_i.
 *   o_parts    DEVICE [num_parts, Hq, Dv] float   (local partials from nanocp_decode_attn_partial and/or
 *   lse_parts  DEVICE [num_parts, Hq]     float    partials received from other instances)
 *   part_offsets DEVICE [num_out + 1] int32; part_index DEVICE [part_offsets[num_out]] int32, or NULL for identity
 *   out        DEVICE [num_out, Hq, Dv] of out_dtype: NANOCP_F32, NANOCP_BF16, or NANOCP_FP8_E4M3 (one byte per
 *              element, the code of value scaled by 1 / desc->out_scale; see nanocp_attn_desc)
 *   out_lse    DEVICE [num_out, Hq] float, or NULL
 * Partials with lse = -inf are ignored; if all are, O = 0 and LSE = -inf.  Only Hq, Dv and out_scale of desc are
 * used.
 */
nanocp_status nanocp_merge_partials(const nanocp_attn_desc* desc, const float* o_parts, const float* lse_parts,
                                    const int32_t* part_offsets, const int32_t* part_index, int32_t num_out,
                                    void* out, int32_t out_dtype, float* out_lse, void* stream);

/*
 * Final rows without a merge (the paper's concern with per-step launch and copy overhead; Phase 4 is the identity
 * for a request whose whole KV is on this instance).  nanocp_plan_set_final_rows (HOST, before nanocp_plan_upload):
 * shard_final_row[s] = r >= 0 declares that every partial of output row r (r < num_out) is a shard of this plan and
 * s is one of them (usually the only one; several shards may name the same row -- a request split over shards that
 * are all local -- and are then reduced together), -1 otherwise.  The call re-derives the partial slots: query the
 * workspace size after it.  nanocp_decode_attn_partial_final then writes the final row final_out[r] (NANOCP_F32,
 * NANOCP_BF16 or NANOCP_FP8_E4M3 as in nanocp_merge_partials, [num_out, Hq, Dv], DEVICE, 16-byte aligned) and
 * final_lse[r] ([num_out, Hq] float, may be NULL) straight from the kernel that finishes it; the out_o rows of those
 * shards are NOT written.  out_lse is: for a shard that is alone in its row it is the shard's (= the row's) LSE; for
 * shards that share a row, the row's LSE is written at the FIRST shard naming the row and the out_lse rows of the
 * others are left untouched (a plan with such shards only runs through this entry point).  All
 * other shards behave as in nanocp_decode_attn_partial.  The remaining output rows are merged with nanocp_merge_partials_rows:
 * like nanocp_merge_partials over num_out partial lists, list i producing row out_rows[i] (DEVICE int32, NULL =
 * identity) of out / out_lse.
 * Errors: as the calls they extend; ESTATE if the rows were not set (or set after upload), EBOUNDS for a row id
 * outside [-1, num_out), ESHAPE if Dv is not a multiple of 8.
 */
nanocp_status nanocp_plan_set_final_rows(nanocp_plan* plan, const int32_t* shard_final_row, int32_t num_out);
nanocp_status nanocp_decode_attn_partial_final(const nanocp_plan* plan, const void* q, const void* k_pool,
                                               const void* v_pool, const float* k_scale, const float* v_scale,
                                               const int32_t* block_table, float* out_o, float* out_lse,
                                               void* workspace, size_t workspace_bytes, void* final_out,
                                               int32_t final_dtype, float* final_lse, void* stream);
nanocp_status nanocp_merge_partials_rows(const nanocp_attn_desc* desc, const float* o_parts, const float* lse_parts,
                                         const int32_t* part_offsets, const int32_t* part_index, int32_t num_out,
                                         const int32_t* out_rows, void* out, int32_t out_dtype, float* out_lse,
                                         void* stream);

/*
 * Buckets: launches that can be recorded once and replayed for any batch composition (paper: AOT Graph Engine --
 * pre-allocated pools sized by a bucket's capacities, control metadata injected by asynchronous copies before the
 * replay, no allocation and no host decision on the replay path).
 * A bucket fixes capacities; nanocp_plan_pack serialises a plan that fits them into a HOST image of
 * nanocp_bucket_plan_bytes bytes whose layout depends on the bucket only.  The caller copies the image to a DEVICE
 * buffer of the same size (256-byte aligned; any stream-ordered copy) and runs nanocp_decode_attn_partial_image,
 * which takes the batch shape from the image on the device: the same call, with the same arguments, is valid for
 * every image of the bucket, so it can be captured in a HIP graph together with nanocp_merge_partials_dyn (the
 * row-indexed merge over at most max_out lists, the actual count read from *num_out_dev on the device).
 * num_cus workgroups are launched whatever the batch is (0 = query the current device).  final_out may be NULL.
 * One image must not be in use by two launches at a time (it holds the work-queue counters).  The kernels compare
 * the image's header with the call: an image packed for another kernel variant, or one whose shards are grouped into
 * final rows while final_out is NULL, is not run (the outputs stay untouched).
 * Errors: EBOUNDS if the plan exceeds the bucket or a buffer is too small; otherwise as the calls they mirror.
 */
typedef struct {
  int32_t max_tiles;   /* tiles of the work-list */
  int32_t max_chunks;  /* work-queue entries */
  int32_t max_segs;    /* (shard, head) results made of several tiles, and empty shards x heads */
  int32_t max_slots;   /* tile partials held in the workspace */
} nanocp_bucket;

size_t nanocp_bucket_plan_bytes(const nanocp_bucket* bucket);
size_t nanocp_bucket_workspace_bytes(const nanocp_attn_desc* desc, const nanocp_bucket* bucket);
nanocp_status nanocp_plan_pack(const nanocp_plan* plan, const nanocp_bucket* bucket, void* host_image,
                               size_t image_bytes);
nanocp_status nanocp_decode_attn_partial_image(const nanocp_attn_desc* desc, const nanocp_bucket* bucket,
                                               const void* device_image, int32_t num_cus, int32_t max_blocks_per_row,
                                               const void* q, const void* k_pool, const void* v_pool,
                                               const float* k_scale, const float* v_scale,
                                               const int32_t* block_table, float* out_o, float* out_lse,
                                               void* workspace, size_t workspace_bytes, void* final_out,
                                               int32_t final_dtype, float* final_lse, void* stream);
nanocp_status nanocp_merge_partials_dyn(const nanocp_attn_desc* desc, const float* o_parts, const float* lse_parts,
                                        const int32_t* part_offsets, const int32_t* part_index, int32_t max_out,
                                        const int32_t* num_out_dev, const int32_t* out_rows, void* out,
                                        int32_t out_dtype, float* out_lse, void* stream);

/*
 * nanocp_decode_attn_partial_image_static -- nanocp_decode_attn_partial_image for callers that cannot allocate and
 * have no workspace to hand over (launches recorded into a HIP graph, tight serving loops, harnesses that forbid
 * hipMalloc).  The tile partials go to a scratch array that is part of the library's device image -- 32 MiB
 * (33,554,432 bytes) on every GPU the library runs on, held until the process ends; its address is looked up once per
 * device, on the first call made with that device current (make that call outside a stream capture).  The call
 * allocates nothing and queries nothing: num_cus must be given (> 0).
 * Errors: as nanocp_decode_attn_partial_image; EBOUNDS if nanocp_bucket_workspace_bytes(desc, bucket) exceeds the
 * 32 MiB; EINVAL if num_cus <= 0.
 * All calls on one GPU share the one array (it keeps the previous call's partials; nothing in it needs to start at
 * zero, every slot a launch reads is written by that launch first): two such launches that overlap in time on one
 * GPU race -- order them on one stream, or with events.
 */
nanocp_status nanocp_decode_attn_partial_image_static(const nanocp_attn_desc* desc, const nanocp_bucket* bucket,
                                                      const void* device_image, int32_t num_cus,
                                                      int32_t max_blocks_per_row, const void* q, const void* k_pool,
                                                      const void* v_pool, const float* k_scale, const float* v_scale,
                                                      const int32_t* block_table, float* out_o, float* out_lse,
                                                      void* final_out, int32_t final_dtype, float* final_lse,
                                                      void* stream);

/*
 * nanocp_kv_append -- the writer that goes with the paged layouts above: stores the K / V rows of n tokens at
 * (block-table row, token position) into the pools.  A decode step appends one token per request to the local KV
 * before Phase 2 (each instance keeps only its own KV partition; paper: Data Plane); one bulk call converts a plain
 * cache into the layouts the attention kernels read.
 *   k_new     DEVICE [n, Hkv, Dk] kv elements (MLA: [n, Dk]), 16-byte aligned
 *   v_new     DEVICE [n, Hkv, Dv] kv elements (NULL for MLA: V is part of the latent row)
 *   bt_row, position   DEVICE int32 [n]; the page is block_table[bt_row][position / ps] and must exist
 * fp8: bytes are stored as given, the per-(page, head) scales stay with the caller.  Entries naming the same
 * (row, position) race.  Asynchronous on `stream`.  Errors: EINVAL, ESHAPE, EUNSUPPORTED (as nanocp_plan_create
 * for the shape), EBOUNDS (more than 2^31 blocks), EHIP.
 */
nanocp_status nanocp_kv_append(const nanocp_attn_desc* desc, const void* k_new, const void* v_new,
                               const int32_t* bt_row, const int32_t* position, int32_t n, void* k_pool, void* v_pool,
                               const int32_t* block_table, int32_t max_blocks_per_row, void* stream);

const char* nanocp_status_str(nanocp_status s);

#ifdef __cplusplus
}
#endif
#endif /* NANOCP_H */

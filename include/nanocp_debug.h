/*
 * nanocp_debug.h -- instrumentation entry points of libnanocp.so (not part of the serving interface in nanocp.h).
 */
#ifndef NANOCP_DEBUG_H
#define NANOCP_DEBUG_H

#include "nanocp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* nanocp_decode_attn_partial (see nanocp.h), and additionally records per tile {device wall clock (100 MHz ticks) at
 * its start, at its end, index of the workgroup that ran it} into tile_clock[num_tiles][3] (DEVICE, uint64) -- used
 * by the benchmark to report how much the slowest piece of the work-list straggles behind the mean. */
nanocp_status nanocp_decode_attn_partial_timed(const nanocp_plan* plan, const void* q, const void* k_pool,
                                               const void* v_pool, const float* k_scale, const float* v_scale,
                                               const int32_t* block_table, float* out_o, float* out_lse,
                                               void* workspace, size_t workspace_bytes, uint64_t* tile_clock,
                                               void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NANOCP_DEBUG_H */

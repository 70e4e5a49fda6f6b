/*
 * nanocp_sched.h -- C ABI of the host-side dual-balanced scheduler (paper: Control Plane, Alg. 1
 * "Dual-balanced Scheduling Strategy").  Pure host code: it decides, per decode iteration, each request's
 * MoE binding m_r, its KV binding P_r (the CP degree is |P_r|) and the token split over P_r; the shard
 * ranges it produces are what nanocp_plan_create consumes on each instance.
 *
 * Instances are numbered 0..S-1; node n owns instances [node_offsets[n], node_offsets[n+1]).
 * All pointers are HOST memory owned by the caller.  Every argmin and sort breaks ties towards the
 * lower index (the paper does not say).  Errors: NANOCP_EINVAL (null / negative / unsorted offsets /
 * degree outside [1, NANOCP_SCHED_MAX_CP] / empty participant set), NANOCP_EBOUNDS (instance id out of range).
 */
#ifndef NANOCP_SCHED_H
#define NANOCP_SCHED_H

#include "nanocp.h"

#ifdef __cplusplus
extern "C" {
#endif

#define NANOCP_SCHED_MAX_CP 8 /* a KV binding stays inside one node (Alg. 1, choice of k_r: k_r <= |S_n*|) */

typedef struct {
  int32_t num_nodes;
  const int32_t* node_offsets;   /* [num_nodes + 1], increasing, node_offsets[0] = 0 */
  int64_t kv_capacity;           /* K_max, tokens per instance */
  int32_t num_buckets;           /* Bucket(l): degree of the first bucket with l <= bucket_max_len[i], else the last */
  const int64_t* bucket_max_len; /* [num_buckets], increasing */
  const int32_t* bucket_degree;  /* [num_buckets] */
} nanocp_sched_config;

typedef struct {
  int32_t scheduled;   /* 1 = committed, 0 = does not fit this iteration (stays in the waiting queue) */
  int32_t node;        /* n* */
  int32_t moe_instance;                           /* m_r */
  int32_t num_participants;                       /* k_r = |P_r| */
  int32_t participants[NANOCP_SCHED_MAX_CP];      /* P_r = [m_r, then the k_r - 1 instances of the node with the smallest KV load] */
  int64_t split[NANOCP_SCHED_MAX_CP];             /* Split_r: tokens per participant, consecutive ranges in this order */
} nanocp_sched_decision;

/* WaterFill(P_r, l_r, K): split `length` tokens over n participants with current loads so that the peak
 * load + split is minimal and sum(split) = length: loads are raised to a common level, the remainder goes
 * one token each to the lowest-indexed participants at that level. */
nanocp_status nanocp_sched_water_fill(int32_t n, const int64_t* loads, int64_t length, int64_t* split);

/* Alg. 1, first part: rebalance the MoE bindings of the active requests.  Request r's participants are
 * part_instances[part_offsets[r] .. part_offsets[r+1]).  Requests are taken by ascending participant count;
 * each is bound to its participant with the fewest bound requests so far.
 * Writes moe_instance[num_active] and moe_load[S] (B_s, starting from zero). */
nanocp_status nanocp_sched_rebalance(const nanocp_sched_config* cfg, int32_t num_active, const int32_t* part_offsets,
                                     const int32_t* part_instances, int32_t* moe_instance, int32_t* moe_load);

/* Alg. 1, second part (placing the new requests): place them in order.  kv_load[S] (K_s) and moe_load[S] (B_s) are read and
 * updated by every committed placement.  Writes decisions[num_new]. */
nanocp_status nanocp_sched_place(const nanocp_sched_config* cfg, int64_t* kv_load, int32_t* moe_load, int32_t num_new,
                                 const int64_t* lengths, nanocp_sched_decision* decisions);

#ifdef __cplusplus
}
#endif
#endif /* NANOCP_SCHED_H */

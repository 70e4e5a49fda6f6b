// Host-side dual-balanced scheduler (paper: Control Plane, Alg. 1).  No GPU code.
#include <algorithm>
#include <numeric>
#include <vector>

#include "nanocp_sched.h"

namespace {

bool config_ok(const nanocp_sched_config* c) {
  if (!c || c->num_nodes <= 0 || !c->node_offsets || c->kv_capacity < 0) return false;
  if (c->node_offsets[0] != 0) return false;
  for (int n = 0; n < c->num_nodes; ++n)
    if (c->node_offsets[n + 1] <= c->node_offsets[n]) return false;
  if (c->num_buckets <= 0 || !c->bucket_max_len || !c->bucket_degree) return false;
  for (int i = 0; i < c->num_buckets; ++i) {
    if (c->bucket_degree[i] < 1 || c->bucket_degree[i] > NANOCP_SCHED_MAX_CP) return false;
    if (i && c->bucket_max_len[i] <= c->bucket_max_len[i - 1]) return false;
  }
  return true;
}

int bucket(const nanocp_sched_config* c, int64_t length) {
  for (int i = 0; i < c->num_buckets; ++i)
    if (length <= c->bucket_max_len[i]) return c->bucket_degree[i];
  return c->bucket_degree[c->num_buckets - 1];
}

// level fill: O(n log n) via the sorted loads instead of a search over levels
void water_fill(int n, const int64_t* loads, int64_t length, int64_t* split) {
  std::fill(split, split + n, (int64_t)0);
  if (length == 0 || n == 0) return;
  std::vector<int> idx(n);
  std::iota(idx.begin(), idx.end(), 0);
  std::sort(idx.begin(), idx.end(), [&](int a, int b) { return loads[a] < loads[b]; });
  // raise the j lowest loads to a common level while tokens last
  int64_t level = loads[idx[0]], left = length;
  int j = 1;  // participants idx[0..j) are at `level`
  while (j < n) {
    const int64_t step = loads[idx[j]] - level;
    if (step * j > left) break;
    left -= step * j;
    level = loads[idx[j]];
    ++j;
  }
  level += left / j;
  left %= j;
  for (int i = 0; i < n; ++i) split[i] = std::max<int64_t>(0, level - loads[i]);
  for (int i = 0; i < n && left > 0; ++i)  // remainder: lowest indices among those at the level
    if (loads[i] <= level) {
      ++split[i];
      --left;
    }
}

}  // namespace

extern "C" {

nanocp_status nanocp_sched_water_fill(int32_t n, const int64_t* loads, int64_t length, int64_t* split) {
  if (n <= 0 || !loads || !split || length < 0) return NANOCP_EINVAL;
  water_fill(n, loads, length, split);
  return NANOCP_OK;
}

nanocp_status nanocp_sched_rebalance(const nanocp_sched_config* cfg, int32_t num_active, const int32_t* part_offsets,
                                     const int32_t* part_instances, int32_t* moe_instance, int32_t* moe_load) {
  if (!config_ok(cfg) || num_active < 0 || !moe_load) return NANOCP_EINVAL;
  const int S = cfg->node_offsets[cfg->num_nodes];
  std::fill(moe_load, moe_load + S, 0);
  if (num_active == 0) return NANOCP_OK;
  if (!part_offsets || !part_instances || !moe_instance) return NANOCP_EINVAL;
  std::vector<int> order(num_active);
  std::iota(order.begin(), order.end(), 0);
  for (int r = 0; r < num_active; ++r) {
    if (part_offsets[r + 1] <= part_offsets[r]) return NANOCP_EINVAL;
    for (int k = part_offsets[r]; k < part_offsets[r + 1]; ++k)
      if (part_instances[k] < 0 || part_instances[k] >= S) return NANOCP_EBOUNDS;
  }
  // fewer participants = fewer feasible choices: those requests are bound first
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
    return part_offsets[a + 1] - part_offsets[a] < part_offsets[b + 1] - part_offsets[b];
  });
  for (int r : order) {
    int best = -1;
    for (int k = part_offsets[r]; k < part_offsets[r + 1]; ++k) {
      const int s = part_instances[k];
      if (best < 0 || moe_load[s] < moe_load[best] || (moe_load[s] == moe_load[best] && s < best)) best = s;
    }
    moe_instance[r] = best;
    ++moe_load[best];
  }
  return NANOCP_OK;
}

nanocp_status nanocp_sched_place(const nanocp_sched_config* cfg, int64_t* kv_load, int32_t* moe_load, int32_t num_new,
                                 const int64_t* lengths, nanocp_sched_decision* decisions) {
  if (!config_ok(cfg) || !kv_load || !moe_load || num_new < 0) return NANOCP_EINVAL;
  if (num_new == 0) return NANOCP_OK;
  if (!lengths || !decisions) return NANOCP_EINVAL;
  for (int r = 0; r < num_new; ++r)
    if (lengths[r] < 0) return NANOCP_EINVAL;
  std::vector<int64_t> node_load(cfg->num_nodes, 0);  // B^(n)
  for (int n = 0; n < cfg->num_nodes; ++n)
    for (int s = cfg->node_offsets[n]; s < cfg->node_offsets[n + 1]; ++s) node_load[n] += moe_load[s];
  std::vector<int> others;
  for (int r = 0; r < num_new; ++r) {
    nanocp_sched_decision& d = decisions[r];
    d = nanocp_sched_decision{};
    // node selection and CP degree
    int n_star = 0;
    for (int n = 1; n < cfg->num_nodes; ++n)
      if (node_load[n] < node_load[n_star]) n_star = n;
    const int s0 = cfg->node_offsets[n_star], s1 = cfg->node_offsets[n_star + 1];
    const int k = std::min(bucket(cfg, lengths[r]), s1 - s0);
    // intra-node placement
    int m = s0;
    for (int s = s0 + 1; s < s1; ++s)
      if (moe_load[s] < moe_load[m]) m = s;
    others.clear();
    for (int s = s0; s < s1; ++s)
      if (s != m) others.push_back(s);
    std::stable_sort(others.begin(), others.end(), [&](int a, int b) { return kv_load[a] < kv_load[b]; });
    d.node = n_star;
    d.moe_instance = m;
    d.num_participants = k;
    d.participants[0] = m;
    for (int i = 1; i < k; ++i) d.participants[i] = others[i - 1];
    int64_t loads[NANOCP_SCHED_MAX_CP];
    for (int i = 0; i < k; ++i) loads[i] = kv_load[d.participants[i]];
    water_fill(k, loads, lengths[r], d.split);
    bool fits = true;
    for (int i = 0; i < k; ++i) fits = fits && loads[i] + d.split[i] <= cfg->kv_capacity;
    d.scheduled = fits ? 1 : 0;
    if (fits) {
      for (int i = 0; i < k; ++i) kv_load[d.participants[i]] += d.split[i];
      ++moe_load[m];
      ++node_load[n_star];
    }
  }
  return NANOCP_OK;
}

}  // extern "C"

"""Plain-Python statement of the dual-balanced scheduling strategy.  TEST INFRASTRUCTURE ONLY.

Follows the paper's Alg. 1 ("Dual-balanced Scheduling Strategy") step by step, in its notation:
  N      nodes; S_n the CP instances of node n
  K_s    KV-cache load (tokens) of instance s;  K_max the per-instance capacity
  B_s    number of requests whose MoE communication is bound to instance s;  B^(n) = sum over S_n
  l_r    sequence length of request r;  P_r its participant set;  m_r its MoE binding;  Split_r its token split
Step A rebalances the MoE bindings of the active requests, steps B and C place each new request:
node with the fewest bound requests, CP degree from the length bucket, MoE binding = least-bound instance of
the node, remaining participants = smallest KV load, token split by WaterFill, commit if it fits.

Readings where the paper is silent: every argmin / sort breaks ties towards the lower index (instance id,
node id, request order); P_r is ordered [m_r, C_r in selection order] and the split is handed out as
consecutive token ranges in that order; WaterFill returns the level solution ("distributes tokens to
lower-loaded instances first"): raise the lowest loads to a common level, the remainder one token each to
the lowest-indexed participants at that level -- one of the many splits that attain the minimal peak.

Pins (tests/test_scheduler.py): WaterFill against exhaustive search of its stated objective and against
token-by-token greedy filling on tiny inputs, a hand-computed case, conservation and capacity invariants,
hand-traced placements.
"""


def bucket_degree(bucket_max_len, bucket_deg, length):
    """Bucket(l): degree of the first bucket whose upper length bound is >= l (the last one otherwise)."""
    for bound, deg in zip(bucket_max_len, bucket_deg):
        if length <= bound:
            return deg
    return bucket_deg[-1]


def water_fill(loads, length):
    """Split `length` tokens over participants with current loads so that sum(split) == length and
    max(load + split) is minimal; level solution, remainder to the lowest indices at the level."""
    n = len(loads)
    split = [0] * n
    if length == 0:
        return split
    # largest level L with sum(max(0, L - load)) <= length   (binary search on an integer level)
    lo, hi = min(loads), min(loads) + length          # at hi the least-loaded participant alone absorbs everything
    while lo < hi:
        mid = (lo + hi + 1) // 2
        need = sum(max(0, mid - k) for k in loads)
        if need <= length:
            lo = mid
        else:
            hi = mid - 1
    level = lo
    for i, k in enumerate(loads):
        split[i] = max(0, level - k)
    rem = length - sum(split)
    for i, k in enumerate(loads):                      # remainder: one more token to participants at the level
        if rem == 0:
            break
        if k <= level:
            split[i] += 1
            rem -= 1
    assert rem == 0
    return split


def rebalance(num_instances, active_participants):
    """Step A.  active_participants[r] = P_r (list of instance ids).  Returns (m[r], B[s])."""
    B = [0] * num_instances
    m = [None] * len(active_participants)
    order = sorted(range(len(active_participants)), key=lambda r: (len(active_participants[r]), r))
    for r in order:
        P = active_participants[r]
        best = min(P, key=lambda s: (B[s], s))
        m[r] = best
        B[best] += 1
    return m, B


def place(nodes, K, B, K_max, bucket_max_len, bucket_deg, lengths):
    """Steps B and C for the new requests, in order.  nodes[n] = list of instance ids; K, B are updated in
    place.  Returns one dict per request: scheduled, node, m, P, split."""
    out = []
    for length in lengths:
        n_star = min(range(len(nodes)), key=lambda n: (sum(B[s] for s in nodes[n]), n))
        S = nodes[n_star]
        k = min(bucket_degree(bucket_max_len, bucket_deg, length), len(S))
        m = min(S, key=lambda s: (B[s], s))
        others = sorted((s for s in S if s != m), key=lambda s: (K[s], s))
        P = [m] + others[:k - 1]
        split = water_fill([K[s] for s in P], length)
        ok = all(K[s] + t <= K_max for s, t in zip(P, split))
        if ok:
            for s, t in zip(P, split):
                K[s] += t
            B[m] += 1
        out.append({"scheduled": ok, "node": n_star, "m": m, "P": P, "split": split})
    return out

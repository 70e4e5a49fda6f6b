"""Float64 checker for one GPU's share of a DCP decode step.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition the GPU library is compared against.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import it; the product
path never does, and this module shares no code with it.

What it computes (paper: Data Plane, "Decoupled Data-Path Design"):
  * Phase 2, paged attention: each KV-binding instance computes, for every routed query,
    a partial attention output over its LOCAL KV shard together with the log-sum-exp of
    the shard's scores.
  * Phase 4, LSE-based merging: the MoE-binding instance combines the partials of a
    request into its final attention output.  The combination is exact: merging the
    partials of any split of a request's tokens equals attention over all of them.
Readings taken where the paper is silent (also listed in the design notes): the partial is
normalised by the shard's own softmax denominator and travels with a natural-log LSE, one
value per query head; decode has one query token per request and no mask; an empty shard
gives O = 0 and LSE = -inf and is the identity of the merge; fp8 is OCP E4M3FN with one
float32 scale per (page, kv head), dequantised as table[byte] * scale.

All arithmetic is float64 over the dequantised inputs (bf16 and fp8 widen exactly).

Pins (tests/test_oracle_pins.py): single key, equal scores, split invariance to 1e-12,
explicit-sum brute force and a hand-computed two-key case, score-shift invariance, page
permutation invariance, merge algebra, scipy logsumexp/softmax, the E4M3 table against its
format definition and torch's decoder, the page layout against a loop-written packer.
"""
import numpy as np

# --------------------------------------------------------------------------- element decoding


def decode_bf16(bits):
    """bfloat16 bit patterns (uint16) -> float64, exact."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def _e4m3fn_value(code):
    """Value of one OCP FP8 E4M3FN code: 1 sign, 4 exponent (bias 7), 3 mantissa bits;
    no infinities; S.1111.111 is NaN; exponent field 0 is subnormal (m/8 * 2^-6)."""
    sign = -1.0 if (code >> 7) & 1 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return sign * (m / 8.0) * 2.0 ** (-6)
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


E4M3FN_TABLE = np.array([_e4m3fn_value(c) for c in range(256)], dtype=np.float64)


def decode_elems(raw, dtype):
    """Stored elements -> float64 (fp8 still unscaled)."""
    if dtype == "f32":
        return np.asarray(raw, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return decode_bf16(raw)
    if dtype == "fp8":
        return E4M3FN_TABLE[np.asarray(raw, dtype=np.uint8)]
    raise ValueError(dtype)


# --------------------------------------------------------------------------- paged gather


def gather_kv(desc, k_pool, v_pool, k_scale, v_scale, bt_row, kv_begin, kv_end):
    """K[L,Hkv,Dk], V[L,Hkv,Dv] in float64 for tokens [kv_begin,kv_end) of one block-table row.

    Token t lives in physical page bt_row[t // ps], slot t % ps.
      GQA:  K[t,h,d]  = k_pool[page, h, slot // 4x, d // x, slot % 4x, d % x]
            V[t,h,dv] = v_pool[page, h, u, dv, e]                       (x = elements per 16 bytes)
                 with w = slot % 4x,  u = 4*(slot // 4x) + (w % 16) // 4,  e = 4*(w // 16) + w % 4
      MLA:  K[t,0,:]  = k_pool[page, slot, :],   V[t,0,:] = K[t,0,:Dv]
    """
    ps = desc.page_size
    L = int(kv_end) - int(kv_begin)
    tok = np.arange(int(kv_begin), int(kv_end))
    page = np.asarray(bt_row)[tok // ps].astype(np.int64)
    slot = tok % ps
    if desc.kind == "mla":
        K = decode_elems(k_pool[page, slot, :], desc.kv_dtype).reshape(L, 1, desc.head_dim_qk)
        V = K[:, :, :desc.head_dim_v]
        return K, V
    x = k_pool.shape[-1]
    K = decode_elems(k_pool[page, :, slot // (4 * x), :, slot % (4 * x), :], desc.kv_dtype)   # [L,Hkv,Dk/x,x]
    K = K.reshape(L, desc.num_kv_heads, desc.head_dim_qk)
    w = slot % (4 * x)
    u = 4 * (slot // (4 * x)) + (w % 16) // 4
    e = 4 * (w // 16) + w % 4
    V = decode_elems(v_pool[page, :, u, :, e], desc.kv_dtype)              # [L,Hkv,Dv]
    V = V.reshape(L, desc.num_kv_heads, desc.head_dim_v)
    if desc.kv_dtype == "fp8":
        K = K * k_scale[page].astype(np.float64)[:, :, None]
        V = V * v_scale[page].astype(np.float64)[:, :, None]
    return K, V


def decode_q(desc, q_row):
    return decode_elems(q_row, desc.q_dtype)


# --------------------------------------------------------------------------- Phase 2: partial attention


def attn_partial_dense(q, K, V, scale):
    """Attention of q[Hq,Dk] over tokens K[L,Hkv,Dk], V[L,Hkv,Dv]; query head a uses kv head a // (Hq/Hkv).

    Returns O[Hq,Dv] (normalised over these L tokens) and LSE[Hq] = log sum_j exp(scale * <q,k_j>).
    """
    Hq = q.shape[0]
    L, Hkv, _ = K.shape
    Dv = V.shape[2]
    G = Hq // Hkv
    O = np.zeros((Hq, Dv), np.float64)
    LSE = np.full((Hq,), -np.inf, np.float64)
    if L == 0:
        return O, LSE
    scale = np.float64(np.float32(scale))
    for h in range(Hkv):
        s = scale * (q[h * G:(h + 1) * G] @ K[:, h, :].T)          # [G,L]
        m = s.max(axis=1, keepdims=True)
        p = np.exp(s - m)
        l = p.sum(axis=1, keepdims=True)
        O[h * G:(h + 1) * G] = (p @ V[:, h, :]) / l
        LSE[h * G:(h + 1) * G] = (m + np.log(l))[:, 0]
    return O, LSE


def attn_partial_paged(desc, q, k_pool, v_pool, k_scale, v_scale, block_table, shard):
    """One shard entry (q_row, bt_row, kv_begin, kv_end) -> (O[Hq,Dv], LSE[Hq])."""
    q_row, bt_row, b, e = (int(v) for v in shard)
    K, V = gather_kv(desc, k_pool, v_pool, k_scale, v_scale, block_table[bt_row], b, e)
    return attn_partial_dense(decode_q(desc, q[q_row]), K, V, desc.softmax_scale)


# --------------------------------------------------------------------------- Phase 4: LSE merge


def merge(o_parts, lse_parts):
    """Combine d partials: LSE = log sum_i exp(LSE_i), O = sum_i exp(LSE_i - LSE) O_i.

    o_parts[d,Hq,Dv], lse_parts[d,Hq].  Empty partials (LSE = -inf) contribute nothing; if all are
    empty the result is O = 0, LSE = -inf.
    """
    o_parts = np.asarray(o_parts, np.float64)
    lse_parts = np.asarray(lse_parts, np.float64)
    d, Hq, Dv = o_parts.shape
    O = np.zeros((Hq, Dv), np.float64)
    LSE = np.full((Hq,), -np.inf, np.float64)
    for a in range(Hq):
        top = lse_parts[:, a].max() if d else -np.inf
        if top == -np.inf:
            continue
        w = np.exp(lse_parts[:, a] - top)
        tot = w.sum()
        LSE[a] = top + np.log(tot)
        O[a] = (w[:, None] * o_parts[:, a, :]).sum(axis=0) / tot
    return O, LSE


# --------------------------------------------------------------------------- whole step on a batch


def local_partials(batch):
    """(O[S,Hq,Dv], LSE[S,Hq]) for every shard entry this GPU holds."""
    d = batch.desc
    S = batch.shards.shape[0]
    O = np.zeros((S, d.num_q_heads, d.head_dim_v), np.float64)
    LSE = np.zeros((S, d.num_q_heads), np.float64)
    for s in range(S):
        O[s], LSE[s] = attn_partial_paged(d, batch.q, batch.k_pool, batch.v_pool, batch.k_scale,
                                          batch.v_scale, batch.block_table, batch.shards[s])
    return O, LSE


def remote_partials(batch):
    """Partials the other KV-binding instances would return (needs the batch's remote KV)."""
    d = batch.desc
    n = len(batch.remotes)
    O = np.zeros((n, d.num_q_heads, d.head_dim_v), np.float64)
    LSE = np.zeros((n, d.num_q_heads), np.float64)
    for i, r in enumerate(batch.remotes):
        O[i], LSE[i] = attn_partial_paged(d, batch.q, r.k_pool, r.v_pool, r.k_scale, r.v_scale,
                                          r.block_table, (r.q_row, 0, r.kv_begin, r.kv_end))
    return O, LSE


def merge_requests(o_parts, lse_parts, part_offsets, part_index):
    """Final outputs per request from the pooled partial list (CSR over requests)."""
    R = len(part_offsets) - 1
    Hq, Dv = o_parts.shape[1], o_parts.shape[2]
    O = np.zeros((R, Hq, Dv), np.float64)
    LSE = np.zeros((R, Hq), np.float64)
    for r in range(R):
        idx = part_index[part_offsets[r]:part_offsets[r + 1]]
        O[r], LSE[r] = merge(o_parts[idx], lse_parts[idx])
    return O, LSE


def request_full_attention(batch, r):
    """Unsharded attention of request r over ALL its tokens (local + remote shards, in order)."""
    d = batch.desc
    S = batch.shards.shape[0]
    Ks, Vs = [], []
    for p in batch.part_index[batch.part_offsets[r]:batch.part_offsets[r + 1]]:
        if p < S:
            _, bt_row, b, e = (int(v) for v in batch.shards[p])
            K, V = gather_kv(d, batch.k_pool, batch.v_pool, batch.k_scale, batch.v_scale,
                             batch.block_table[bt_row], b, e)
        else:
            rs = batch.remotes[p - S]
            K, V = gather_kv(d, rs.k_pool, rs.v_pool, rs.k_scale, rs.v_scale, rs.block_table[0],
                             rs.kv_begin, rs.kv_end)
        Ks.append(K)
        Vs.append(V)
    q_row = r
    return attn_partial_dense(decode_q(d, batch.q[q_row]), np.concatenate(Ks), np.concatenate(Vs),
                              d.softmax_scale)

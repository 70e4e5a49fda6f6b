"""Pins for the float64 checker: what the definitions and the mathematics fix, not its own code.

Each test names the passage or fact it rests on.  Paper: Data Plane, Phase 2 (partial attention
output + LSE over the local KV partition) and Phase 4 (LSE-based merging gives the final
attention output, i.e. the merge is exact).
"""
import itertools
import math
import types

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workloads as W


def _desc(kind="gqa", kv="f32", Hq=4, Hkv=2, Dk=8, Dv=8, ps=4, scale=0.5, q="f32"):
    return W.AttnDesc(kind, q, kv, Hq, Hkv, Dk, Dv, ps, scale)


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# ---- 1. single key: softmax over one token is 1, so O = V_0 and LSE = the score itself
def test_single_key_returns_its_value():
    rng = np.random.default_rng(1)
    q, K, V = _rand(rng, 6, 5), _rand(rng, 1, 3, 5), _rand(rng, 1, 3, 7)
    O, LSE = oracle.attn_partial_dense(q, K, V, 0.3)
    s = np.float64(np.float32(0.3))
    for a in range(6):
        assert np.array_equal(O[a], V[0, a // 2])
        assert LSE[a] == pytest.approx(s * float(q[a] @ K[0, a // 2]), rel=1e-15, abs=1e-15)


# ---- 2. equal scores: uniform softmax, O = mean of V, LSE = s + log L
def test_equal_scores_return_mean_of_v():
    rng = np.random.default_rng(2)
    L = 37
    V = _rand(rng, L, 2, 6)
    K = np.repeat(_rand(rng, 1, 2, 5), L, axis=0)          # identical keys -> identical scores
    q = _rand(rng, 4, 5)
    O, LSE = oracle.attn_partial_dense(q, K, V, 1.0)
    for a in range(4):
        np.testing.assert_allclose(O[a], V[:, a // 2].mean(axis=0), rtol=1e-13, atol=1e-14)
        assert LSE[a] == pytest.approx(float(q[a] @ K[0, a // 2]) + math.log(L), rel=1e-14)
    O0, LSE0 = oracle.attn_partial_dense(np.zeros((4, 5)), _rand(rng, L, 2, 5), V, 1.0)
    np.testing.assert_allclose(O0[0], V[:, 0].mean(axis=0), rtol=1e-13, atol=1e-14)
    assert LSE0[3] == pytest.approx(math.log(L), rel=1e-14)


# ---- 4. brute force by an explicitly written sum (no max subtraction, python loops), tiny sizes
def _brute(q, K, V, scale, G):
    Hq = len(q)
    out, lse = [], []
    for a in range(Hq):
        h = a // G
        e = []
        for j in range(len(K)):
            s = 0.0
            for d in range(len(q[a])):
                s += q[a][d] * K[j][h][d]
            e.append(math.exp(scale * s))
        den = sum(e)
        out.append([sum(e[j] * V[j][h][c] for j in range(len(K))) / den for c in range(len(V[0][h]))])
        lse.append(math.log(den))
    return np.array(out), np.array(lse)


@pytest.mark.parametrize("L,Dk,Dv,Hq,Hkv", [(1, 1, 1, 1, 1), (2, 2, 1, 2, 1), (3, 2, 2, 4, 2), (4, 1, 2, 3, 3), (4, 2, 2, 6, 2)])
def test_brute_force_tiny(L, Dk, Dv, Hq, Hkv):
    rng = np.random.default_rng(100 + L + Dk)
    q, K, V = _rand(rng, Hq, Dk), _rand(rng, L, Hkv, Dk), _rand(rng, L, Hkv, Dv)
    scale = 0.75                                               # exactly representable in float32
    O, LSE = oracle.attn_partial_dense(q, K, V, scale)
    Ob, LSEb = _brute(q.tolist(), K.tolist(), V.tolist(), scale, Hq // Hkv)
    np.testing.assert_allclose(O, Ob, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(LSE, LSEb, rtol=1e-13, atol=1e-15)


def test_two_keys_hand_case():
    # scores 0 and log 3  ->  weights 1/4 and 3/4, LSE = log 4
    q = np.array([[1.0]])
    K = np.array([[[0.0]], [[math.log(3.0)]]])
    V = np.array([[[8.0, -4.0]], [[0.0, 4.0]]])
    O, LSE = oracle.attn_partial_dense(q, K, V, 1.0)
    np.testing.assert_allclose(O, [[2.0, 2.0]], rtol=1e-15)
    assert LSE[0] == pytest.approx(math.log(4.0), rel=1e-15)


def test_gqa_head_mapping_not_transposed():
    # kv head 1 has a huge key match only for query heads 2,3 (G=2): pins a // G (not a % Hkv)
    q = np.zeros((4, 2)); q[:, 0] = 1.0
    K = np.zeros((2, 2, 2)); K[1, 1, 0] = 50.0
    V = np.zeros((2, 2, 1)); V[0, :, 0] = 1.0; V[1, :, 0] = 2.0
    O, _ = oracle.attn_partial_dense(q, K, V, 1.0)
    np.testing.assert_allclose(O[:, 0], [1.5, 1.5, 2.0, 2.0], atol=1e-12)


# ---- 5. shift invariance: a constant added to every score leaves O and shifts LSE
def test_score_shift_invariance():
    rng = np.random.default_rng(5)
    q, K, V = _rand(rng, 4, 6), _rand(rng, 29, 2, 6), _rand(rng, 29, 2, 3)
    O, LSE = oracle.attn_partial_dense(q, K, V, 1.0)
    c = 3.25
    q2 = np.concatenate([q, np.ones((4, 1))], axis=1)
    K2 = np.concatenate([K, np.full((29, 2, 1), c)], axis=2)
    O2, LSE2 = oracle.attn_partial_dense(q2, K2, V, 1.0)
    np.testing.assert_allclose(O2, O, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(LSE2, LSE + c, rtol=1e-13)


# ---- 8. textbook routines: scipy logsumexp / softmax
def test_against_scipy():
    rng = np.random.default_rng(8)
    q, K, V = _rand(rng, 4, 16), _rand(rng, 100, 1, 16), _rand(rng, 100, 1, 8)
    scale = 0.25
    O, LSE = oracle.attn_partial_dense(q, K, V, scale)
    s = scale * np.einsum("ad,jd->aj", q, K[:, 0])
    np.testing.assert_allclose(LSE, scipy.special.logsumexp(s, axis=1), rtol=1e-14)
    np.testing.assert_allclose(O, scipy.special.softmax(s, axis=1) @ V[:, 0], rtol=1e-12, atol=1e-15)


# ---- 3. split invariance (Phase 4 exactness): merge of any split == unsharded attention, 1e-12
@pytest.mark.parametrize("seed", range(6))
def test_split_invariance(seed):
    rng = np.random.default_rng(30 + seed)
    L = int(rng.integers(1, 200))
    q, K, V = _rand(rng, 8, 12), _rand(rng, L, 2, 12), _rand(rng, L, 2, 5)
    d = int(rng.integers(1, 9))
    cuts = np.sort(rng.integers(0, L + 1, size=d - 1))       # may repeat -> empty shards, 1-token shards
    edges = [0, *cuts.tolist(), L]
    parts = [oracle.attn_partial_dense(q, K[b:e], V[b:e], 0.4) for b, e in zip(edges[:-1], edges[1:])]
    O, LSE = oracle.merge(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]))
    Of, LSEf = oracle.attn_partial_dense(q, K, V, 0.4)
    assert np.max(np.abs(O - Of)) < 1e-12
    assert np.max(np.abs(LSE - LSEf)) < 1e-12


# ---- 7. merge algebra: commutative, associative, empty partial is the identity, all-empty is empty
def test_merge_algebra():
    rng = np.random.default_rng(7)
    o = _rand(rng, 5, 3, 4)
    lse = _rand(rng, 5, 3) * 3
    O, LSE = oracle.merge(o, lse)
    perm = rng.permutation(5)
    O2, LSE2 = oracle.merge(o[perm], lse[perm])
    np.testing.assert_allclose(O2, O, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(LSE2, LSE, rtol=1e-13)
    Oa, La = oracle.merge(o[:2], lse[:2])
    Ob, Lb = oracle.merge(o[2:], lse[2:])
    O3, LSE3 = oracle.merge(np.stack([Oa, Ob]), np.stack([La, Lb]))
    np.testing.assert_allclose(O3, O, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(LSE3, LSE, rtol=1e-13)
    oe = np.concatenate([o, np.full((1, 3, 4), 123.0)])
    le = np.concatenate([lse, np.full((1, 3), -np.inf)])
    O4, LSE4 = oracle.merge(oe, le)
    np.testing.assert_allclose(O4, O, rtol=1e-15)
    np.testing.assert_allclose(LSE4, LSE, rtol=1e-15)
    O5, LSE5 = oracle.merge(np.ones((2, 3, 4)), np.full((2, 3), -np.inf))
    assert np.all(O5 == 0) and np.all(LSE5 == -np.inf) and not np.isnan(O5).any()
    # closed form: two partials with LSE 0 and log 3 weigh 1/4 and 3/4
    O6, LSE6 = oracle.merge(np.array([[[4.0]], [[8.0]]]), np.array([[0.0], [math.log(3.0)]]))
    assert O6[0, 0] == pytest.approx(7.0, rel=1e-15) and LSE6[0] == pytest.approx(math.log(4.0), rel=1e-15)


def test_empty_shard():
    O, LSE = oracle.attn_partial_dense(np.ones((2, 3)), np.zeros((0, 1, 3)), np.zeros((0, 1, 2)), 1.0)
    assert np.all(O == 0) and np.all(LSE == -np.inf)


# ---- 9. fp8 table against the format definition (OCP E4M3FN) and torch's decoder
def test_e4m3fn_table():
    t = oracle.E4M3FN_TABLE
    assert np.isnan(t).sum() == 2 and np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)                             # monotone within the sign
    assert pos[0] == 0.0 and pos[1] == 2.0 ** -9 and pos[0x08] == 2.0 ** -6 and pos[0x7E] == 448.0
    assert t[0x38] == 1.0 and t[0x3C] == 1.5 and t[0x40] == 2.0
    np.testing.assert_array_equal(t[0x80:0xFF], -pos)
    assert not np.isinf(t).any()
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(np.nan_to_num(t, nan=-7.0), np.nan_to_num(ref, nan=-7.0))


def test_bf16_decode_matches_torch():
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.decode_bf16(bits)
    m = ~np.isnan(ref)
    np.testing.assert_array_equal(got[m], ref[m])


def test_generator_encoders_round_trip():
    # the generator's encoders are separate code; decoding what they wrote must be the nearest value
    rng = np.random.default_rng(9)
    x = (rng.standard_normal(5000) * 30).astype(np.float32)
    v = oracle.E4M3FN_TABLE[W.numfmt.f32_to_e4m3fn(x)]
    finite = oracle.E4M3FN_TABLE[~np.isnan(oracle.E4M3FN_TABLE)]
    best = np.abs(finite[None, :] - np.clip(x, -448, 448).astype(np.float64)[:, None]).min(axis=1)
    np.testing.assert_array_equal(np.abs(v - np.clip(x, -448, 448)), best)
    b = oracle.decode_bf16(W.numfmt.f32_to_bf16_bits(x))
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(b, ref)


# ---- 10. page layout: a packer written with explicit loops from the layout statement
def _pack_loops(desc, x, K, V, bt_row, pages, begin):
    """K[L,Hkv,Dk], V[L,Hkv,Dv] (float) -> pools in the documented layouts with x elements per vector
    (the layout of 4-, 2- and 1-byte elements, here always holding floats), token i stored at begin+i."""
    ps = desc.page_size
    if desc.kind == "mla":
        kp = np.zeros((pages, ps, desc.head_dim_qk), np.float32)
        for i in range(K.shape[0]):
            t = begin + i
            kp[bt_row[t // ps], t % ps, :] = K[i, 0]
        return kp, None
    kp = np.zeros((pages, desc.num_kv_heads, ps // (4 * x), desc.head_dim_qk // x, 4 * x, x), np.float32)
    vp = np.zeros((pages, desc.num_kv_heads, ps // x, desc.head_dim_v, x), np.float32)
    for i in range(K.shape[0]):
        t = begin + i
        p, slot = bt_row[t // ps], t % ps
        for h in range(desc.num_kv_heads):
            for d in range(desc.head_dim_qk):
                kp[p, h, slot // (4 * x), d // x, slot % (4 * x), d % x] = K[i, h, d]
            # V: groups of 4x slots; slot 16b + 4g + i of a group is element 4b + i of the group's vector g
            grp, w = slot // (4 * x), slot % (4 * x)
            b_, g_, i_ = w // 16, (w % 16) // 4, w % 4
            for c in range(desc.head_dim_v):
                vp[p, h, 4 * grp + g_, c, 4 * b_ + i_] = V[i, h, c]
    return kp, vp


@pytest.mark.parametrize("kind,x,ps", [("gqa", 4, 16), ("gqa", 8, 32), ("gqa", 16, 64), ("gqa", 8, 64), ("mla", 4, 8)])
def test_gather_matches_documented_layout(kind, x, ps):
    rng = np.random.default_rng(10)
    if kind == "gqa":
        desc = _desc("gqa", "f32", 4, 2, 16, 12, ps)
        K, V = _rand(rng, 21, 2, 16).astype(np.float32), _rand(rng, 21, 2, 12).astype(np.float32)
    else:
        desc = _desc("mla", "f32", 4, 1, 12, 8, 8)
        K = _rand(rng, 21, 1, 12).astype(np.float32)
        V = K[:, :, :8]
    bt_row = np.array([5, 2, 7, 0], np.int32)
    kp, vp = _pack_loops(desc, x, K, V, bt_row, 8, begin=3)
    Kg, Vg = oracle.gather_kv(desc, kp, vp, None, None, bt_row, 3, 24)
    np.testing.assert_array_equal(Kg, K.astype(np.float64))
    np.testing.assert_array_equal(Vg, V.astype(np.float64))


# ---- 6. paging invariance: permuting physical pages (and the block table) changes nothing, bit for bit
def test_page_permutation_invariance():
    b = W.reduced(1)
    O, LSE = oracle.local_partials(b)
    rng = np.random.default_rng(6)
    perm = rng.permutation(b.k_pool.shape[0])                  # new_pool[perm[p]] = old_pool[p]
    kp, vp = np.empty_like(b.k_pool), np.empty_like(b.v_pool)
    kp[perm], vp[perm] = b.k_pool, b.v_pool
    bt = np.where(b.block_table >= 0, perm[np.maximum(b.block_table, 0)], -1).astype(np.int32)
    b2 = types.SimpleNamespace(**{**b.__dict__, "k_pool": kp, "v_pool": vp, "block_table": bt})
    O2, LSE2 = oracle.local_partials(b2)
    assert np.array_equal(O, O2) and np.array_equal(LSE, LSE2)


# ---- the whole step on every reduced config: merged partials == unsharded attention (1e-12),
#      CP=1 partial is already the final output, nothing is NaN although unused slots are NaN-filled
@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5, 6, 7])
def test_step_exactness_on_reduced_configs(cid):
    b = W.reduced(cid)
    O, LSE = oracle.local_partials(b)
    Or, LSEr = oracle.remote_partials(b)
    assert not np.isnan(O).any() and not np.isnan(LSE).any() and not np.isnan(Or).any()
    parts_o, parts_lse = np.concatenate([O, Or]), np.concatenate([LSE, LSEr])
    Om, LSEm = oracle.merge_requests(parts_o, parts_lse, b.part_offsets, b.part_index)
    multi = [r for r in range(b.num_requests) if b.cp_degree[r] > 1]
    assert multi or cid == 2
    for r in multi + [0]:
        Of, LSEf = oracle.request_full_attention(b, r)
        assert np.max(np.abs(Om[r] - Of)) < 1e-12
        assert np.max(np.abs(LSEm[r] - LSEf)) < 1e-12
    for r in range(b.num_requests):
        if b.cp_degree[r] == 1:
            s = b.part_index[b.part_offsets[r]]
            assert np.array_equal(Om[r], O[s])


def test_fp8_scale_is_applied_per_page_and_head():
    # doubling one page's K scale must change only scores of tokens in that page (checked through LSE of a
    # single-page shard), doubling V scale doubles that shard's output exactly
    b = W.reduced(5)
    s = 1
    _, bt_row, b0, e0 = (int(v) for v in b.shards[s])
    page = int(b.block_table[bt_row, 0])
    shard = np.array([b.shards[s][0], bt_row, 0, min(e0, b.desc.page_size)])
    O1, L1 = oracle.attn_partial_paged(b.desc, b.q, b.k_pool, b.v_pool, b.k_scale, b.v_scale, b.block_table, shard)
    vs = b.v_scale.copy(); vs[page] *= 2
    O2, L2 = oracle.attn_partial_paged(b.desc, b.q, b.k_pool, b.v_pool, b.k_scale, vs, b.block_table, shard)
    np.testing.assert_allclose(O2, 2 * O1, rtol=1e-15)
    np.testing.assert_array_equal(L1, L2)
    ks = b.k_scale.copy(); ks[page, 0] *= 2
    O3, L3 = oracle.attn_partial_paged(b.desc, b.q, b.k_pool, b.v_pool, ks, b.v_scale, b.block_table, shard)
    G = b.desc.num_q_heads // b.desc.num_kv_heads
    assert np.array_equal(L3[G:], L1[G:]) and not np.allclose(L3[:G], L1[:G])

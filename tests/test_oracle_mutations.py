"""The pins must be able to fail: each plausible mistake planted in the checker (on the CPU, by patching it)
has to be caught by at least one pin from test_oracle_pins.py."""
import numpy as np
import pytest

import oracle
import oracle.attention as oa
import test_oracle_pins as pins


def _mut_no_scale(q, K, V, scale):
    return ORIG["attn"](q, K, V, 1.0)


def _mut_head_mod(q, K, V, scale):
    Hq, Hkv = q.shape[0], K.shape[1]
    G = Hq // Hkv
    perm = [(a % Hkv) * G + a // Hkv for a in range(Hq)]          # query head a uses kv head a % Hkv
    O, L = ORIG["attn"](q[perm], K, V, scale)
    inv = np.argsort(perm)
    return O[inv], L[inv]


def _mut_lse_without_max(q, K, V, scale):
    O, L = ORIG["attn"](q, K, V, scale)
    if K.shape[0]:
        G = q.shape[0] // K.shape[1]
        s = np.float64(np.float32(scale)) * np.stack([q[a] @ K[:, a // G].T for a in range(q.shape[0])])
        L = L - s.max(axis=1)
    return O, L


def _mut_unnormalised(q, K, V, scale):
    O, L = ORIG["attn"](q, K, V, scale)
    return O * np.exp(L)[:, None], L


def _mut_v_transposed_weights(q, K, V, scale):
    O, L = ORIG["attn"](q, K[::-1], V, scale)                      # probabilities paired with the wrong tokens
    return O, L


def _mut_merge_equal_weights(o, l):
    o, l = np.asarray(o, np.float64), np.asarray(l, np.float64)
    O, L = ORIG["merge"](o, l)
    live = np.isfinite(l)
    w = live / np.maximum(live.sum(axis=0, keepdims=True), 1)
    return (w[:, :, None] * np.where(live[:, :, None], o, 0)).sum(axis=0), L


def _mut_merge_lse_max(o, l):
    O, _ = ORIG["merge"](o, l)
    return O, np.asarray(l, np.float64).max(axis=0)


def _mut_gather_plain_v(desc, k_pool, v_pool, k_scale, v_scale, bt_row, b, e):
    K, V = ORIG["gather"](desc, k_pool, v_pool, k_scale, v_scale, bt_row, b, e)
    if desc.kind == "gqa":
        x, ps = k_pool.shape[-1], desc.page_size
        tok = np.arange(int(b), int(e))
        page, slot = np.asarray(bt_row)[tok // ps].astype(np.int64), tok % ps
        V = oa.decode_elems(v_pool[page, :, slot // x, :, slot % x], desc.kv_dtype).reshape(V.shape)   # plain token order
    return K, V


def _mut_gather_no_block_table(desc, k_pool, v_pool, k_scale, v_scale, bt_row, b, e):
    return ORIG["gather"](desc, k_pool, v_pool, k_scale, v_scale, np.arange(len(bt_row)), b, e)


ORIG = {}

PIN_SETS = {
    "attn": [lambda: pins.test_single_key_returns_its_value(), lambda: pins.test_equal_scores_return_mean_of_v(),
             lambda: pins.test_brute_force_tiny(3, 2, 2, 4, 2), lambda: pins.test_two_keys_hand_case(),
             lambda: pins.test_gqa_head_mapping_not_transposed(), lambda: pins.test_against_scipy(),
             lambda: pins.test_split_invariance(0)],
    "merge": [lambda: pins.test_merge_algebra(), lambda: pins.test_split_invariance(1)],
    "gather": [lambda: pins.test_gather_matches_documented_layout("gqa", 8, 32),
               lambda: pins.test_gather_matches_documented_layout("gqa", 16, 64)],
}

MUTANTS = [("attn", _mut_no_scale), ("attn", _mut_head_mod), ("attn", _mut_lse_without_max),
           ("attn", _mut_unnormalised), ("attn", _mut_v_transposed_weights),
           ("merge", _mut_merge_equal_weights), ("merge", _mut_merge_lse_max),
           ("gather", _mut_gather_plain_v), ("gather", _mut_gather_no_block_table)]
NAMES = {"attn": "attn_partial_dense", "merge": "merge", "gather": "gather_kv"}


@pytest.mark.parametrize("which,mutant", MUTANTS, ids=[m.__name__ for _, m in MUTANTS])
def test_pins_catch_planted_mistake(which, mutant, monkeypatch):
    name = NAMES[which]
    ORIG[which] = getattr(oa, name)
    for pin in PIN_SETS[which]:                  # sanity: the pins pass on the real checker
        pin()
    monkeypatch.setattr(oa, name, mutant)
    monkeypatch.setattr(oracle, name, mutant)
    caught = 0
    for pin in PIN_SETS[which]:
        try:
            pin()
        except AssertionError:
            caught += 1
    assert caught >= 1, f"no pin noticed {mutant.__name__}"

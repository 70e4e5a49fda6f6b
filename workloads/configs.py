"""The five benchmark configurations (the paper's micro-benchmark batch as a sixth, a 64-head MLA shape as a seventh) as seeded
generators, plus reduced variants for tests.

Every full-size function takes optional overrides (request count, length range) so the
parity tests can run the same recipe at sizes the float64 checker finishes in seconds.
Seeds: numpy default_rng(20260521 + config id); config 3 scans seeds upward from that
default until the draw has at least two requests longer than the CP threshold, one of
them with CP degree >= 3, and never edits drawn lengths.
"""
import math

import numpy as np

from .batches import AttnDesc, build_batch, even_split

BASE_SEED = 20260521
CP_THRESHOLD = 32768
CP_CAP = 8


def _gqa_desc(kv_dtype="bf16"):
    return AttnDesc("gqa", "bf16", kv_dtype, 64, 4, 128, 128, 64, 1.0 / math.sqrt(128.0))


def config1(seed=None, with_remote_kv=True):
    """Tiny fp32 GQA decode: lengths {17,64,130,255}; the 255-token request is split
    [0,128),[128,255) with both halves local and merged."""
    seed = BASE_SEED + 1 if seed is None else seed
    rng = np.random.default_rng(seed)
    desc = AttnDesc("gqa", "f32", "f32", 8, 2, 64, 64, 16, 1.0 / 8.0)
    lengths = [17, 64, 130, 255]
    ranges = [[(0, 17)], [(0, 64)], [(0, 130)], [(0, 128), (128, 255)]]
    local = [[0], [0], [0], [0, 1]]
    return build_batch("c1_tiny_f32_gqa", seed, desc, lengths, ranges, local, rng, with_remote_kv)


def config2(seed=None, num_requests=64, lo=1024, hi=8192, with_remote_kv=True):
    """bf16 GQA decode, all requests local (CP=1), lengths uniform in [lo,hi]."""
    seed = BASE_SEED + 2 if seed is None else seed
    rng = np.random.default_rng(seed)
    lengths = rng.integers(lo, hi + 1, size=num_requests)
    ranges = [[(0, int(L))] for L in lengths]
    local = [[0] for _ in lengths]
    return build_batch("c2_bf16_gqa_local", seed, _gqa_desc(), lengths, ranges, local, rng, with_remote_kv)


def _lognormal_lengths(rng, n, median, sigma, lo, hi):
    return np.clip(np.rint(np.exp(rng.normal(math.log(median), sigma, n))), lo, hi).astype(np.int64)


def _cp_degree(length, threshold):
    return 1 if length <= threshold else min(CP_CAP, -(-int(length) // threshold))


def config3_seed(num_requests=128, median=2048, sigma=1.2, lo=16, hi=131072, threshold=CP_THRESHOLD):
    """First seed >= the default whose length draw has >=2 long requests, one with degree >= 3."""
    seed = BASE_SEED + 3
    while True:
        L = _lognormal_lengths(np.random.default_rng(seed), num_requests, median, sigma, lo, hi)
        deg = [_cp_degree(x, threshold) for x in L]
        if sum(d > 1 for d in deg) >= 2 and max(deg) >= 3:
            return seed
        seed += 1


def config3(seed=None, num_requests=128, median=2048, sigma=1.2, lo=16, hi=131072,
            threshold=CP_THRESHOLD, with_remote_kv=True, hold_all=False):
    """Mixed long-tail DCP batch: lognormal lengths; a request longer than `threshold` has
    CP degree d=min(8,ceil(len/threshold)); this GPU holds shard (request index mod d) of it."""
    if seed is None:
        seed = config3_seed(num_requests, median, sigma, lo, hi, threshold)
    rng = np.random.default_rng(seed)
    lengths = _lognormal_lengths(rng, num_requests, median, sigma, lo, hi)
    ranges, local = [], []
    for r, L in enumerate(lengths):
        d = _cp_degree(L, threshold)
        ranges.append(even_split(L, d))
        local.append(list(range(d)) if hold_all else [r % d])
    return build_batch("c3_mixed_dcp", seed, _gqa_desc(), lengths, ranges, local, rng, with_remote_kv)


def config4(seed=None, num_requests=64, lo=4096, hi=32768, with_remote_kv=True, num_heads=128, name="c4_mla_bf16"):
    """MLA-absorbed decode: 128 heads over one 576-dim latent row per token (V = first 512 dims);
    every second request is split at CP=2 with both halves local and merged."""
    seed = BASE_SEED + 4 if seed is None else seed
    rng = np.random.default_rng(seed)
    desc = AttnDesc("mla", "bf16", "bf16", num_heads, 1, 576, 512, 64, 1.0 / math.sqrt(192.0))
    lengths = rng.integers(lo, hi + 1, size=num_requests)
    ranges, local = [], []
    for r, L in enumerate(lengths):
        if r % 2 == 1:
            ranges.append(even_split(L, 2))
            local.append([0, 1])
        else:
            ranges.append([(0, int(L))])
            local.append([0])
    return build_batch(name, seed, desc, lengths, ranges, local, rng, with_remote_kv)


def config5(seed=None, long_len=1048576, cp=8, held=3, num_short=256, lo=512, hi=4096, with_remote_kv=True,
            hold_all=False):
    """fp8 KV: shard `held` of `cp` of one very long request co-batched with short local requests.
    Request 0 is the long one."""
    seed = BASE_SEED + 5 if seed is None else seed
    rng = np.random.default_rng(seed)
    short = rng.integers(lo, hi + 1, size=num_short)
    lengths = np.concatenate([[long_len], short])
    ranges = [even_split(long_len, cp)] + [[(0, int(L))] for L in short]
    local = [list(range(cp)) if hold_all else [held]] + [[0] for _ in short]
    return build_batch("c5_fp8_long_shard", seed, _gqa_desc("fp8"), lengths, ranges, local, rng, with_remote_kv)


def config6(seed=None, num_long=3, long_len=524288, cp=8, held=5, num_short=64, short_len=2048,
            with_remote_kv=True, hold_all=False):
    """The paper's micro-benchmark batch (Evaluation, latency breakdown): `num_short` short requests of
    `short_len` tokens local to this GPU plus, for each of `num_long` (1, 3, 5 or 7) long requests of the
    node, this GPU's 1/cp slice.  All instances of the node carry the same short load, so the water-filling
    split of a long request is the even one.  Requests 0..num_long-1 are the long ones.  bf16 GQA shapes."""
    seed = BASE_SEED + 6 if seed is None else seed
    rng = np.random.default_rng(seed)
    lengths = np.array([long_len] * num_long + [short_len] * num_short, dtype=np.int64)
    ranges = [even_split(long_len, cp) for _ in range(num_long)] + [[(0, short_len)] for _ in range(num_short)]
    local = [list(range(cp)) if hold_all else [held] for _ in range(num_long)] + [[0] for _ in range(num_short)]
    return build_batch(f"c6_micro_{num_long}x{long_len}", seed, _gqa_desc(), lengths, ranges, local, rng,
                       with_remote_kv)


def config7(seed=None, num_requests=64, lo=4096, hi=32768, with_remote_kv=True):
    """Config 4's recipe with 64 query heads: the MLA shape of the paper's second model (its head count differs
    from the first; the latent dims are taken to be the same 576/512, which the paper does not state)."""
    return config4(BASE_SEED + 7 if seed is None else seed, num_requests, lo, hi, with_remote_kv, num_heads=64,
                   name="c7_mla64_bf16")


FULL = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: config6, 7: config7}


def reduced(config_id, with_remote_kv=True, hold_all=False):
    """Same recipes at sizes the float64 checker handles in seconds, still spanning several
    tiles, ragged tails and (for 3 and 5) a shard much longer than the rest.  hold_all (3 and 5):
    every shard of a split request is local, so one GPU can also run the request unsharded."""
    if config_id == 1:
        return config1(with_remote_kv=with_remote_kv)
    if config_id == 2:
        return config2(num_requests=12, lo=100, hi=3000, with_remote_kv=with_remote_kv)
    if config_id == 3:
        return config3(num_requests=24, median=300, sigma=1.2, lo=16, hi=12000, threshold=3000,
                       with_remote_kv=with_remote_kv, hold_all=hold_all)
    if config_id == 4:
        return config4(num_requests=6, lo=200, hi=1500, with_remote_kv=with_remote_kv)
    if config_id == 5:
        return config5(long_len=40000, cp=8, held=3, num_short=20, lo=50, hi=700,
                       with_remote_kv=with_remote_kv, hold_all=hold_all)
    if config_id == 6:
        return config6(num_long=3, long_len=20000, cp=8, held=5, num_short=10, short_len=333,
                       with_remote_kv=with_remote_kv, hold_all=hold_all)
    if config_id == 7:
        return config7(num_requests=6, lo=200, hi=1500, with_remote_kv=with_remote_kv)
    raise ValueError(config_id)

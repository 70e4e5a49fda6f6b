"""Host-side checks: the library loads and exports the declared C ABI; the planner's work-list is a
valid, balanced partition (coverage, page-aligned cuts, slots, chunk cost); argument errors map to codes.
No GPU is touched: plans are built with an explicit compute-unit count."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_21100_amd as nanocp
import workloads as W
from workloads.device import desc_from

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_every_declared_symbol():
    lib = ctypes.CDLL(nanocp.LIB_PATH)
    for header, exports in (("nanocp.h", nanocp.EXPORTS), ("nanocp_debug.h", nanocp.DEBUG_EXPORTS),
                            ("nanocp_sched.h", nanocp.SCHED_EXPORTS)):
        hdr = open(os.path.join(ROOT, "include", header)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)                 # declarations only, not the prose
        declared = sorted(set(re.findall(r"\b(nanocp_[a-z0-9_]+)\s*\(", hdr)))
        assert set(declared) == set(exports), header
        for name in declared:
            assert hasattr(lib, name), name
    assert ctypes.sizeof(nanocp.AttnDesc) == 40 and ctypes.sizeof(nanocp.Shard) == 16
    assert ctypes.sizeof(nanocp.Tile) == 32


def _plan(batch, tile_tokens=0, num_cus=256):
    return nanocp.Plan(desc_from(batch.desc), batch.shards, batch.q.shape[0],
                       batch.block_table.shape[0], batch.block_table.shape[1], tile_tokens, num_cus)


def _check_partition(batch, plan, tile_tokens):
    d = batch.desc
    ps = d.page_size
    tiles = plan.tiles()
    assert len(tiles) == plan.num_tiles
    # chunks are numbered consecutively in list order
    assert np.all(np.diff(tiles["chunk"]) >= 0) and (len(tiles) == 0 or tiles["chunk"][-1] == plan.num_chunks - 1)
    per = {}
    for t in tiles:
        per.setdefault((int(t["shard"]), int(t["kv_head"])), []).append(t)
    slots = []
    for s, (q_row, bt_row, b, e) in enumerate(batch.shards):
        for h in range(d.num_kv_heads):
            ts = per.get((s, h), [])
            if e == b:
                assert not ts
                continue
            assert ts[0]["tok_begin"] == b and ts[-1]["tok_end"] == e
            for a, c in zip(ts[:-1], ts[1:]):
                assert a["tok_end"] == c["tok_begin"] and a["tok_end"] % ps == 0     # page-aligned cuts
            for t in ts:
                assert t["tok_end"] > t["tok_begin"] and t["q_row"] == q_row and t["bt_row"] == bt_row
                assert (t["dst"] == -1) == (len(ts) == 1)
            if len(ts) > 1:
                ds = [int(t["dst"]) for t in ts]
                assert ds == list(range(ds[0], ds[0] + len(ts)))
                slots += ds
    assert sorted(slots) == list(range(len(slots)))
    G = d.num_q_heads // d.num_kv_heads
    if slots:
        assert plan.workspace_bytes >= len(slots) * G * (d.head_dim_v + 1) * 4
    else:
        assert plan.workspace_bytes == 0
    # cost per chunk (pages + 1 per tile) never exceeds the cap implied by the request
    cost = np.zeros(plan.num_chunks, np.int64)
    for t in tiles:
        cost[t["chunk"]] += (t["tok_end"] - 1) // ps - t["tok_begin"] // ps + 1 + 1
    return cost


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5, 6, 7])
@pytest.mark.parametrize("tile_tokens", [0, 64, 256, 1024])
def test_plan_partitions_reduced_configs(cid, tile_tokens):
    b = W.reduced(cid, with_remote_kv=False)
    if tile_tokens and tile_tokens < b.desc.page_size:
        tile_tokens = b.desc.page_size
    plan = _plan(b, tile_tokens)
    cost = _check_partition(b, plan, tile_tokens)
    if tile_tokens:
        assert cost.max() <= tile_tokens // b.desc.page_size + 1
    plan.close()


def _chunk_cost(plan, ps=64, overhead=2):
    tiles = plan.tiles()
    cost = np.zeros(plan.num_chunks, np.int64)
    for t in tiles:
        cost[t["chunk"]] += (t["tok_end"] - 1) // ps - t["tok_begin"] // ps + 1 + overhead
    return tiles, cost


def _check_queue_shape(cost, workgroups=256):
    """Head of the queue: one near-equal big chunk per workgroup (most of the work); tail: smaller chunks
    whose size decays (guided self-scheduling), none larger than half a head chunk."""
    head, tail = cost[:workgroups], cost[workgroups:]
    # (cuts snap to a (shard, head) boundary that is within 12 % of a chunk, so head chunks are equal to that margin)
    nominal = np.median(head)
    assert head.max() <= nominal * 1.13 + 3 and head[:-1].min() >= nominal * 0.87 - 3
    assert 0.60 <= head.sum() / cost.sum() <= 0.95
    assert len(tail) > 0 and tail.max() <= head.max() / 2 + 2
    k = max(len(tail) // 4, 1)
    assert tail[:k].mean() + 1 >= tail[-k:].mean()                      # sizes decay along the tail


def test_auto_plan_balances_a_long_shard():
    # one very long shard among short ones: its pages must be spread over many workgroups (the
    # balance objective), with the long shard first in the queue
    desc = W.AttnDesc("gqa", "bf16", "bf16", 64, 4, 128, 128, 64, 0.1)
    lens = [700] * 50 + [131072] + [700] * 50
    shards = np.array([[i, i, 0, L] for i, L in enumerate(lens)], np.int32)
    plan = nanocp.Plan(desc_from(desc), shards, len(lens), len(lens), 2048, 0, 256)
    tiles, cost = _chunk_cost(plan)
    assert tiles["shard"][0] == 50                               # longest first
    long_chunks = np.unique(tiles["chunk"][tiles["shard"] == 50])
    assert len(long_chunks) >= 150                               # 2/3 of the bytes -> most workgroups
    _check_queue_shape(cost)
    assert plan.kernel == "gqa_mfma_bf16"


def test_kernel_selection():
    def k(**kw):
        base = dict(kind="gqa", q_dtype="bf16", kv_dtype="bf16", num_q_heads=64, num_kv_heads=4,
                    head_dim_qk=128, head_dim_v=128, page_size=64, softmax_scale=0.1)
        base.update(kw)
        p = nanocp.Plan(nanocp.make_desc(**base), np.array([[0, 0, 0, 10]], np.int32), 1, 1, 4, 0, 8)
        name = p.kernel
        p.close()
        return name
    assert k() == "gqa_mfma_bf16"
    assert k(kv_dtype="fp8") == "gqa_mfma_fp8"
    assert k(num_q_heads=32) == "generic"
    assert k(q_dtype="f32", kv_dtype="f32", page_size=16) == "generic"
    assert k(kind="mla", num_q_heads=128, num_kv_heads=1, head_dim_qk=576, head_dim_v=512) in ("generic", "mla_mfma_bf16")


def test_argument_errors():
    d = nanocp.make_desc("gqa", "bf16", "bf16", 64, 4, 128, 128, 64, 0.1)
    sh = np.array([[0, 0, 0, 10]], np.int32)

    def status(desc=d, shards=sh, q_rows=1, bt_rows=1, max_blocks=4, tile=0, cus=8):
        with pytest.raises(nanocp.NanocpError) as e:
            nanocp.Plan(desc, shards, q_rows, bt_rows, max_blocks, tile, cus)
        return e.value.status
    assert status(shards=np.array([[0, 0, 5, 4]], np.int32)) == nanocp.EINVAL          # kv_end < kv_begin
    assert status(shards=np.array([[0, 0, -1, 4]], np.int32)) == nanocp.EINVAL
    assert status(shards=np.array([[1, 0, 0, 4]], np.int32)) == nanocp.EBOUNDS         # q_row out of range
    assert status(shards=np.array([[0, 2, 0, 4]], np.int32)) == nanocp.EBOUNDS         # bt_row out of range
    assert status(shards=np.array([[0, 0, 0, 257]], np.int32)) == nanocp.EBOUNDS       # beyond max_blocks*ps
    assert status(desc=nanocp.make_desc("gqa", "bf16", "bf16", 64, 5, 128, 128, 64, 0.1)) == nanocp.ESHAPE
    assert status(desc=nanocp.make_desc("gqa", "bf16", "bf16", 64, 4, 100, 128, 64, 0.1)) == nanocp.ESHAPE
    assert status(desc=nanocp.make_desc("mla", "bf16", "bf16", 64, 4, 576, 512, 64, 0.1)) == nanocp.ESHAPE
    assert status(desc=nanocp.make_desc("gqa", "f32", "bf16", 64, 4, 128, 128, 64, 0.1)) == nanocp.EUNSUPPORTED
    assert status(desc=nanocp.make_desc("gqa", "bf16", "bf16", 64, 4, 1024, 128, 64, 0.1)) == nanocp.EUNSUPPORTED
    assert status(desc=nanocp.make_desc(7, "bf16", "bf16", 64, 4, 128, 128, 64, 0.1)) == nanocp.EINVAL
    assert status(tile=-1) == nanocp.EINVAL
    ok = nanocp.Plan(d, np.zeros((0, 4), np.int32), 0, 0, 0, 0, 8)                     # empty batch is legal
    assert ok.num_tiles == 0 and ok.num_chunks == 0 and ok.workspace_bytes == 0
    e = nanocp.Plan(d, np.array([[0, 0, 7, 7]], np.int32), 1, 1, 4, 0, 8)              # empty shard is legal
    assert e.num_tiles == 0


def test_full_size_plans_are_balanced():
    for cid in (2, 3, 5):
        if cid == 2:                                               # lengths only: no need to draw the pools
            rng = np.random.default_rng(W.configs.BASE_SEED + 2)
            lens = rng.integers(1024, 8193, size=64)
            shards = np.array([[i, i, 0, L] for i, L in enumerate(lens)], np.int32)
            desc = W.AttnDesc("gqa", "bf16", "bf16", 64, 4, 128, 128, 64, 0.1)
            plan = nanocp.Plan(desc_from(desc), shards, 64, 64, 128, 0, 256)
        else:
            plan = _plan(W.FULL[cid](with_remote_kv=False))
        tiles, cost = _chunk_cost(plan)
        _check_queue_shape(cost)
        # scratch traffic stays small: partial rows (8 KB each way) against the KV bytes
        n_partial = int((tiles["dst"] >= 0).sum())
        kv_pages = int(((tiles["tok_end"] - 1) // 64 - tiles["tok_begin"] // 64 + 1).sum())
        assert 2 * n_partial * 16 * 129 * 4 <= 0.05 * kv_pages * 16384, (cid, n_partial, kv_pages)
        plan.close()


def test_final_rows_regroup_slots_on_the_host():
    """Shards naming one output row become one reduction segment: their tiles share consecutive slots (dst),
    single-tile rows write directly, and the workspace is re-sized."""
    b = W.reduced(4, with_remote_kv=False)                       # every second request split in two local shards
    plan = _plan(b, tile_tokens=256)
    fin, r_offs, r_idx, r_rows = nanocp.split_final_rows(b.part_offsets, b.part_index, b.num_shards)
    assert (fin >= 0).all() and len(r_rows) == 0
    before = plan.tiles()
    plan.set_final_rows(fin, b.num_requests)
    after = plan.tiles()
    assert np.array_equal(before[["shard", "kv_head", "tok_begin", "tok_end", "chunk"]],
                          after[["shard", "kv_head", "tok_begin", "tok_end", "chunk"]])   # the work-list itself is unchanged
    row_of = fin[after["shard"]]
    for r in range(b.num_requests):
        dst = np.sort(after["dst"][row_of == r])
        if len(dst) == 1:
            assert dst[0] == -1
        else:
            assert dst[0] >= 0 and np.array_equal(dst, np.arange(dst[0], dst[0] + len(dst)))
    slots = after["dst"][after["dst"] >= 0]
    assert len(set(slots.tolist())) == len(slots)
    G = b.desc.num_q_heads // b.desc.num_kv_heads
    assert plan.workspace_bytes >= len(slots) * G * (b.desc.head_dim_v + 1) * 4
    plan.close()


def test_plan_image_layout_and_capacity_errors():
    """nanocp_plan_pack is host only: header counts, chunk offsets and tiles land where the bucket's layout says;
    a plan that exceeds any capacity, or a short buffer, is refused."""
    b = W.reduced(3, with_remote_kv=False)
    plan = _plan(b, tile_tokens=128)
    nt, nc = plan.num_tiles, plan.num_chunks
    bucket = nanocp.Bucket(nt + 5, nc + 3, nt + 4 * b.num_shards, nt)
    nbytes = nanocp.bucket_plan_bytes(bucket)
    assert nbytes % 256 == 0 and nbytes >= 48 * (nt + 5) + 4 * (nc + 4)
    img = np.full(nbytes, 0xAB, np.uint8)
    plan.pack(bucket, img)
    hdr = img[:16].view(np.int32)
    assert hdr[0] == nc and hdr[3] == int((plan.tiles()["dst"] >= 0).sum())
    sync_off = 256                                                # 64 header words, then the counters
    n_sync = 2 + bucket.max_segs
    assert not img[sync_off:sync_off + 4 * n_sync].any()          # counters start at zero
    co_off = sync_off + (4 * n_sync + 255) // 256 * 256
    co = img[co_off:co_off + 4 * (nc + 1)].view(np.int32)
    assert co[0] == 0 and co[-1] == nt and np.all(np.diff(co) > 0)
    tiles_off = co_off + (4 * (bucket.max_chunks + 1) + 255) // 256 * 256
    rec = img[tiles_off:tiles_off + 48 * nt].view(np.int32).reshape(nt, 12)
    t = plan.tiles()
    assert np.array_equal(rec[:, 3], t["shard"]) and np.array_equal(rec[:, 4], t["tok_begin"])
    assert np.array_equal(rec[:, 6], t["dst"])
    for bad in (nanocp.Bucket(nt - 1, nc, nt, nt), nanocp.Bucket(nt, nc - 1, nt, nt), nanocp.Bucket(nt, nc, nt, hdr[3] - 1)):
        with pytest.raises(nanocp.NanocpError) as e:
            plan.pack(bad, img)
        assert e.value.status == nanocp.EBOUNDS
    with pytest.raises(nanocp.NanocpError) as e:
        plan.pack(bucket, img[:nbytes - 256])
    assert e.value.status == nanocp.EBOUNDS
    assert nanocp.bucket_workspace_bytes(plan.desc, bucket) >= plan.workspace_bytes
    plan.close()

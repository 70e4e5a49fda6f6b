"""GPU parity: the HIP path, called through the C ABI, against the float64 checker element by element
on the same seeded inputs (reduced configs spanning several tiles and ragged tails, several tilings),
the Phase-4 merge against exact unsharded attention, the GPU's merged result against its own
unsharded run, edge cases, and sampled outputs at the full benchmark sizes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_21100_amd as nanocp
import workloads as W
from workloads.device import DeviceBatch
from parity import MERGE_VS_UNSHARDED_ABS, check_output

pytestmark = pytest.mark.gpu

EXPECTED_KERNEL = {1: "generic", 2: "gqa_mfma_bf16", 3: "gqa_mfma_bf16", 4: "mla_mfma_bf16", 5: "gqa_mfma_fp8", 6: "gqa_mfma_bf16", 7: "mla_mfma_bf16"}


def _say(msg):
    print(msg, flush=True)


def _merge_on_gpu(db, o_parts, lse_parts, out_dtype=torch.float32):
    b = db.batch
    R = b.num_requests
    d = b.desc
    out = torch.empty((R, d.num_q_heads, d.head_dim_v), dtype=out_dtype, device="cuda")
    out_lse = torch.empty((R, d.num_q_heads), dtype=torch.float32, device="cuda")
    po = torch.from_numpy(b.part_offsets).cuda()
    pi = torch.from_numpy(b.part_index).cuda()
    nanocp.nanocp_merge_partials(db.desc, o_parts, lse_parts, po, pi, R, out, out_lse)
    torch.cuda.synchronize()
    return out, out_lse


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5, 6, 7])
@pytest.mark.parametrize("tile_tokens", [0, 128, 448])
def test_partial_and_merge_match_oracle(cid, tile_tokens):
    _say(f"[case] reduced config {cid} tile_tokens {tile_tokens}")
    b = W.reduced(cid)
    ps = b.desc.page_size
    tt = 0 if tile_tokens == 0 else max(ps, tile_tokens // ps * ps)
    db = DeviceBatch(b, tile_tokens=tt)
    if cid in EXPECTED_KERNEL:
        assert db.plan.kernel == EXPECTED_KERNEL[cid]
    if tt:
        assert (db.plan.tiles()["dst"] >= 0).any()          # the tiling really splits shards
    o, lse = db.partial()
    torch.cuda.synchronize()
    ref_o, ref_lse = oracle.local_partials(b)
    check_output(b.desc, o.cpu().numpy(), lse.cpu().numpy(), ref_o, ref_lse, f"c{cid} partial")

    # Phase 4: local partials (GPU) + remote partials (checker, rounded to f32) -> exact attention
    rem_o, rem_lse = oracle.remote_partials(b)
    parts_o = torch.cat([o, torch.from_numpy(rem_o.astype(np.float32)).cuda()])
    parts_lse = torch.cat([lse, torch.from_numpy(rem_lse.astype(np.float32)).cuda()])
    out, out_lse = _merge_on_gpu(db, parts_o, parts_lse)
    ref_m, ref_mlse = oracle.merge_requests(np.concatenate([ref_o, rem_o]), np.concatenate([ref_lse, rem_lse]),
                                            b.part_offsets, b.part_index)
    check_output(b.desc, out.cpu().numpy(), out_lse.cpu().numpy(), ref_m, ref_mlse, f"c{cid} merged")
    for r in [r for r in range(b.num_requests) if b.cp_degree[r] > 1][:3]:
        full_o, full_lse = oracle.request_full_attention(b, r)
        check_output(b.desc, out[r].cpu().numpy(), out_lse[r].cpu().numpy(), full_o, full_lse, f"c{cid} req {r} vs full")
    # bf16 output epilogue: same values rounded once
    out16, _ = _merge_on_gpu(db, parts_o, parts_lse, torch.bfloat16)
    assert torch.equal(out16, out.to(torch.bfloat16))
    db.plan.close()


@pytest.mark.parametrize("cid", [1, 3, 4, 5, 6, 7])
def test_merged_equals_gpu_unsharded(cid):
    """The GPU's merge of its own d partials against the GPU's own single-shard run of the same request."""
    _say(f"[case] merged vs unsharded, reduced config {cid}")
    b = W.reduced(cid, hold_all=True) if cid in (3, 5, 6) else W.reduced(cid)
    _merged_vs_unsharded(b, 256 if b.desc.page_size <= 64 else 0)


def test_merged_equals_gpu_unsharded_full_size_long_request():
    """Config 5's 1,048,576-token fp8 request with all 8 shards on this GPU (automatic tiling, as benchmarked): the
    merge of the 8 partials against one unsharded pass over the million tokens."""
    _say("[case] merged vs unsharded, full-size config 5 request (1,048,576 tokens, CP = 8)")
    b = W.FULL[5](num_short=16, hold_all=True, with_remote_kv=False)
    assert int(b.shards[:8, 3].max()) == 1048576
    _merged_vs_unsharded(b, 0)


def _merged_vs_unsharded(b, tile_tokens):
    assert len(b.remote_meta) == 0
    db = DeviceBatch(b, tile_tokens=tile_tokens)
    o, lse = db.partial()
    out, out_lse = _merge_on_gpu(db, o, lse)
    # unsharded: one shard per request covering all its tokens, on the same pools / block table
    whole = []
    for r in range(b.num_requests):
        idx = b.part_index[b.part_offsets[r]:b.part_offsets[r + 1]]
        sh = b.shards[idx]
        assert len(set(sh[:, 1].tolist())) == 1
        whole.append([r, sh[0, 1], sh[:, 2].min(), sh[:, 3].max()])
    whole = np.asarray(whole, np.int32)
    plan = nanocp.Plan(db.desc, whole, b.q.shape[0], b.block_table.shape[0], b.block_table.shape[1]).upload()
    d = b.desc
    uo = torch.empty((len(whole), d.num_q_heads, d.head_dim_v), dtype=torch.float32, device="cuda")
    ul = torch.empty((len(whole), d.num_q_heads), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    nanocp.nanocp_decode_attn_partial(plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table,
                                      uo, ul, ws)
    torch.cuda.synchronize()
    split = [r for r in range(b.num_requests) if b.cp_degree[r] > 1]
    assert split
    err = (out[split] - uo[split]).abs().max().item()
    lerr = (out_lse[split] - ul[split]).abs().max().item()
    _say(f"    merged vs unsharded: max abs {err:.3e}, LSE {lerr:.3e}")
    assert err <= MERGE_VS_UNSHARDED_ABS and lerr <= MERGE_VS_UNSHARDED_ABS
    plan.close()
    db.plan.close()


def _edge_batch(kv_dtype, shards_spec, seed=77):
    """Hand-made shard ranges on one row per shard (GQA 64/4x128, page 64; f32 uses the small C1 shape)."""
    rng = np.random.default_rng(seed)
    if kv_dtype == "f32":
        desc = W.AttnDesc("gqa", "f32", "f32", 8, 2, 64, 64, 16, 0.125)
    elif kv_dtype in ("mla", "mla64"):
        desc = W.AttnDesc("mla", "bf16", "bf16", 128 if kv_dtype == "mla" else 64, 1, 576, 512, 64, 192 ** -0.5)
    else:
        desc = W.AttnDesc("gqa", "bf16", kv_dtype, 64, 4, 128, 128, 64, 128 ** -0.5)
    lengths = [max(e, 1) for (_, e) in shards_spec]
    ranges = [[(0, L)] for L in lengths]
    b = W.build_batch("edge", seed, desc, lengths, ranges, [[0]] * len(lengths), rng)
    for i, (bg, en) in enumerate(shards_spec):           # narrow each shard to the requested range
        b.shards[i, 2], b.shards[i, 3] = bg, en
    return b


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16", "fp8", "mla", "mla64"])
def test_edge_ranges(kv_dtype):
    """Empty shard, single token, ranges inside one page, starting / ending mid-page, exact page multiples."""
    _say(f"[case] edge ranges {kv_dtype}")
    ps = 16 if kv_dtype == "f32" else 64
    spec = [(0, 0), (0, 1), (5, 6), (3, ps - 2), (ps - 1, ps + 1), (0, ps), (0, 4 * ps), (7, 5 * ps + 9),
            (2 * ps, 2 * ps), (ps + 1, 3 * ps), (0, 33), (31, 33), (32, 64 if ps == 64 else 48), (0, 9 * ps + 1)]
    b = _edge_batch(kv_dtype, spec)
    for tt in (0, ps, 2 * ps):
        db = DeviceBatch(b, tile_tokens=tt)
        o, lse = db.partial()
        torch.cuda.synchronize()
        ref_o, ref_lse = oracle.local_partials(b)
        check_output(b.desc, o.cpu().numpy(), lse.cpu().numpy(), ref_o, ref_lse, f"edge {kv_dtype} tt={tt}")
        assert torch.all(o[0] == 0) and torch.all(torch.isneginf(lse[0]))
        db.plan.close()


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16", "fp8", "mla"])
def test_edge_ranges_as_final_rows(kv_dtype):
    """The same hand-made ranges with every shard its own output row: empty shards become zero rows with LSE = -inf
    straight from the attention launch (plan and plan-image entry points), the others equal partial + merge."""
    _say(f"[case] edge ranges as final rows {kv_dtype}")
    ps = 16 if kv_dtype == "f32" else 64
    spec = [(0, 0), (0, 1), (3, ps - 2), (ps - 1, ps + 1), (2 * ps, 2 * ps), (0, 4 * ps), (7, 5 * ps + 9), (0, 0)]
    b = _edge_batch(kv_dtype, spec)
    S, d = b.num_shards, b.desc
    base = DeviceBatch(b)
    o, lse = base.partial()
    want, want_lse = _merge_on_gpu(base, o, lse)
    db = DeviceBatch(b, final_rows=True)
    assert (db.shard_final_row >= 0).all() and len(db.rest_rows) == 0
    bucket = nanocp.Bucket(db.plan.num_tiles + 8, db.plan.num_chunks + 8, db.plan.num_tiles + S * d.num_kv_heads + 8,
                           db.plan.num_tiles + 8)
    host_img = torch.empty(nanocp.bucket_plan_bytes(bucket), dtype=torch.uint8).pin_memory()
    db.plan.pack(bucket, host_img)
    dev_img = host_img.cuda()
    ws = torch.empty(max(nanocp.bucket_workspace_bytes(db.desc, bucket), 16), dtype=torch.uint8, device="cuda")
    for dt in (torch.float32, torch.bfloat16):
        for image in (False, True):
            out = torch.full((S, d.num_q_heads, d.head_dim_v), float("nan"), dtype=dt, device="cuda")
            out_lse = torch.full((S, d.num_q_heads), float("nan"), device="cuda")
            po, pl = torch.full_like(o, float("nan")), torch.full_like(lse, float("nan"))
            if image:
                nanocp.nanocp_decode_attn_partial_image(db.desc, bucket, dev_img, 0, b.block_table.shape[1], db.q,
                                                        db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table,
                                                        po, pl, ws, final_out=out, final_lse=out_lse)
            else:
                nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale,
                                                  db.block_table, po, pl, db.workspace, final_out=out,
                                                  final_lse=out_lse)
            torch.cuda.synchronize()
            assert torch.equal(out, want.to(dt)), f"{kv_dtype} {dt} image={image}"
            assert torch.equal(out_lse, want_lse) and torch.equal(pl, lse)
            for e in (0, 4, 7):
                assert torch.all(out[e] == 0) and torch.all(torch.isneginf(out_lse[e]))
    base.plan.close()
    db.plan.close()


def test_merge_edge_cases():
    """All-empty merge, identity (one part), parts ignored when LSE = -inf even if their output is NaN."""
    _say("[case] merge edge cases")
    desc = nanocp.make_desc("gqa", "bf16", "bf16", 8, 2, 64, 64, 64, 0.1)
    rng = np.random.default_rng(3)
    o = rng.standard_normal((5, 8, 64)).astype(np.float32)
    lse = rng.standard_normal((5, 8)).astype(np.float32)
    lse[3] = -np.inf
    o[3] = np.nan
    lse[4] = -np.inf
    offs = np.array([0, 1, 4, 5, 5, 7], np.int32)            # r0: {0}; r1: {1,2,3}; r2: {4} all empty; r3: none; r4: {0,1}
    idx = np.array([0, 1, 2, 3, 4, 0, 1], np.int32)
    R = 5
    out = torch.empty((R, 8, 64), device="cuda")
    out_lse = torch.empty((R, 8), device="cuda")
    nanocp.nanocp_merge_partials(desc, torch.from_numpy(o).cuda(), torch.from_numpy(lse).cuda(),
                                 torch.from_numpy(offs).cuda(), torch.from_numpy(idx).cuda(), R, out, out_lse)
    torch.cuda.synchronize()
    o64 = np.where(np.isnan(o), 0.0, o).astype(np.float64)
    ref_o, ref_lse = oracle.merge_requests(o64, lse.astype(np.float64), offs, idx)
    got = out.cpu().numpy()
    assert not np.isnan(got).any()
    np.testing.assert_allclose(got, ref_o, atol=1e-6)
    gl = out_lse.cpu().numpy()
    assert np.array_equal(np.isneginf(gl), np.isneginf(ref_lse))
    np.testing.assert_allclose(gl[np.isfinite(ref_lse)], ref_lse[np.isfinite(ref_lse)], atol=1e-6)
    assert np.array_equal(got[0], o[0])                          # single part: identity
    # identity part_index (NULL)
    offs2 = np.array([0, 2, 3], np.int32)
    out2 = torch.empty((2, 8, 64), device="cuda")
    nanocp.nanocp_merge_partials(desc, torch.from_numpy(o[:3]).cuda(), torch.from_numpy(lse[:3]).cuda(),
                                 torch.from_numpy(offs2).cuda(), None, 2, out2, None)
    torch.cuda.synchronize()
    r2, _ = oracle.merge_requests(o64[:3], lse[:3].astype(np.float64), offs2, np.arange(3))
    np.testing.assert_allclose(out2.cpu().numpy(), r2, atol=1e-6)


def test_device_call_errors():
    _say("[case] device call errors")
    b = W.reduced(2)
    db = DeviceBatch(b, tile_tokens=128)
    assert db.plan.workspace_bytes > 0
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, None, None, db.block_table,
                                          db.out_o, db.out_lse, small)
    assert e.value.status == nanocp.EBOUNDS
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.nanocp_decode_attn_partial(db.plan, None, db.k_pool, db.v_pool, None, None, db.block_table,
                                          db.out_o, db.out_lse, db.workspace)
    assert e.value.status == nanocp.EINVAL
    fresh = nanocp.Plan(db.desc, b.shards, b.q.shape[0], b.block_table.shape[0], b.block_table.shape[1])
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.nanocp_decode_attn_partial(fresh, db.q, db.k_pool, db.v_pool, None, None, db.block_table,
                                          db.out_o, db.out_lse, db.workspace)
    assert e.value.status == nanocp.ESTATE
    fresh.close()
    db.plan.close()


def test_run_to_run_determinism():
    _say("[case] determinism")
    b = W.reduced(3)
    db = DeviceBatch(b)
    o1, l1 = (t.clone() for t in db.partial())
    o2, l2 = db.partial()
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    db.plan.close()


def _launch_variants(b, tile_tokens):
    """The three ways a plan reaches the tile kernels: the plain entry point, the final-row entry point and the
    plan-image entry point (final rows), each as (name, launch(), tensors that must not change between launches)."""
    d, S, R = b.desc, b.num_shards, b.num_requests
    out = []
    db = DeviceBatch(b, tile_tokens=tile_tokens)
    out.append(("plain", db, lambda: db.partial(), [db.out_o, db.out_lse]))
    dbf = DeviceBatch(b, tile_tokens=tile_tokens, final_rows=True)
    fin = torch.zeros((R, d.num_q_heads, d.head_dim_v), dtype=torch.bfloat16, device="cuda")
    fin_lse = torch.zeros((R, d.num_q_heads), device="cuda")

    def run_final():
        nanocp.nanocp_decode_attn_partial(dbf.plan, dbf.q, dbf.k_pool, dbf.v_pool, dbf.k_scale, dbf.v_scale,
                                          dbf.block_table, dbf.out_o, dbf.out_lse, dbf.workspace, final_out=fin,
                                          final_lse=fin_lse)
    keep = torch.from_numpy(dbf.shard_final_row < 0).cuda()       # O rows of final-row shards are not written
    out.append(("final", dbf, run_final, [fin, fin_lse, dbf.out_lse, (dbf.out_o, keep)]))
    nt = dbf.plan.num_tiles
    bucket = nanocp.Bucket(nt + 8, dbf.plan.num_chunks + 8, nt + S * d.num_kv_heads + 8, nt + 8)
    host_img = torch.empty(nanocp.bucket_plan_bytes(bucket), dtype=torch.uint8).pin_memory()
    dbf.plan.pack(bucket, host_img)
    dev_img = host_img.cuda()
    ws = torch.empty(max(nanocp.bucket_workspace_bytes(dbf.desc, bucket), 16), dtype=torch.uint8, device="cuda")
    fin2, fin_lse2 = torch.zeros_like(fin), torch.zeros_like(fin_lse)
    o2, l2 = torch.zeros_like(dbf.out_o), torch.zeros_like(dbf.out_lse)

    def run_image():
        nanocp.nanocp_decode_attn_partial_image(dbf.desc, bucket, dev_img, 0, b.block_table.shape[1], dbf.q, dbf.k_pool,
                                                dbf.v_pool, dbf.k_scale, dbf.v_scale, dbf.block_table, o2, l2, ws,
                                                final_out=fin2, final_lse=fin_lse2)
    out.append(("image", dbf, run_image, [fin2, fin_lse2, l2, (o2, keep)]))
    return out


def _snap(ts):
    return [(t[0][t[1]] if isinstance(t, tuple) else t).clone() for t in ts]


@pytest.mark.parametrize("cid, tile_tokens", [(2, 1024), (5, 1024), (3, 0), (3, 1024), (4, 0)])
def test_fused_reduction_is_stable_over_many_launches(cid, tile_tokens):
    """Full-size batch, every long (shard, head) reduced by the workgroup that delivers its last tile while the memory
    system is saturated: 100 launches through each entry point (plain, final rows, plan image), every one compared
    with the first and the run stopped at the first difference.  A partial counted as arrived before its stores
    have landed shows up here as a wrong row."""
    _say(f"[case] repeated launches, full-size config {cid}, tile_tokens {tile_tokens}")
    b = W.FULL[cid](with_remote_kv=False)
    variants = _launch_variants(b, tile_tokens)
    for name, db, launch, watched in variants:
        assert (db.plan.tiles()["dst"] >= 0).any()               # the work-list really has multi-tile pairs
        launch()
        torch.cuda.synchronize()
        first = _snap(watched)
        for it in range(100):
            launch()
            now = _snap(watched)
            same = all(torch.equal(torch.nan_to_num(x.float()), torch.nan_to_num(y.float())) for x, y in zip(now, first))
            assert same, f"c{cid} {name}: launch {it} differs from the first"
        if name == "plain":
            ro, rl = oracle.attn_partial_paged(b.desc, b.q, b.k_pool, b.v_pool, b.k_scale, b.v_scale, b.block_table,
                                               b.shards[0])
            check_output(b.desc, first[0][0].cpu().numpy(), first[1][0].cpu().numpy(), ro, rl,
                         f"c{cid} repeated launches, shard 0")
    for db in {id(v[1]): v[1] for v in variants}.values():
        db.plan.close()


@pytest.mark.parametrize("cid", [1, 2, 4, 5])
def test_pages_beyond_4_gib_into_the_pool(cid):
    """Maximum sizes: the same batch with its pages moved to the end of pools larger than 4 GiB (page ids shifted in the
    block table) must give bit-identical results - byte offsets into the pools need 64 bits."""
    _say(f"[case] pool offsets beyond 4 GiB, reduced config {cid}")
    b = W.reduced(cid)
    db = DeviceBatch(b)
    o_ref, lse_ref = (t.clone() for t in db.partial())

    def grow(t, n_big):
        if t is None:
            return None
        big = torch.empty((n_big,) + tuple(t.shape[1:]), dtype=t.dtype, device="cuda")
        big[n_big - t.shape[0]:] = t
        return big

    pages = db.k_pool.shape[0]
    page_bytes = db.k_pool[0].numel() * db.k_pool.element_size()
    n_big = (5 << 30) // page_bytes + pages
    shift = n_big - pages
    assert shift * page_bytes > 1 << 32
    k, v = grow(db.k_pool, n_big), grow(db.v_pool, n_big)
    ks, vs = grow(db.k_scale, n_big), grow(db.v_scale, n_big)
    bt = db.block_table + shift
    o, lse = torch.empty_like(o_ref), torch.empty_like(lse_ref)
    nanocp.nanocp_decode_attn_partial(db.plan, db.q, k, v, ks, vs, bt, o, lse, db.workspace)
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    db.plan.close()


def _sample_shards(b, k, rng):
    lens = b.shards[:, 3] - b.shards[:, 2]
    order = np.argsort(lens)
    pick = {int(order[-1]), int(order[0]), int(order[len(order) // 2])}
    pick |= set(int(i) for i in rng.choice(len(lens), size=min(k, len(lens)), replace=False))
    return sorted(pick)


@pytest.mark.parametrize("cid", [2, 3, 4, 5, 6, 7])
def test_full_size(cid):
    """Full benchmark sizes in the launch configuration bench.py times (automatic tiling).  GQA workloads: EVERY shard
    entry against the checker (a second or two of float64 work each).  MLA workloads (the checker needs minutes for
    all of them): sampled shard entries, always including the longest and the shortest, one by one; the rest must be
    finite and agree with a second tiling of the same batch."""
    _say(f"[case] full-size config {cid}")
    b = W.FULL[cid](with_remote_kv=False)
    db = DeviceBatch(b)
    assert db.plan.kernel == EXPECTED_KERNEL[cid]
    o, lse = db.partial()
    torch.cuda.synchronize()
    assert torch.isfinite(o).all() and torch.isfinite(lse).all()
    o_h, lse_h = o.cpu().numpy(), lse.cpu().numpy()
    if b.desc.kind == "gqa":
        ref_o, ref_lse = oracle.local_partials(b)
        assert ref_o.shape[0] == b.num_shards
        check_output(b.desc, o_h, lse_h, ref_o, ref_lse, f"c{cid} full size, all {b.num_shards} shard entries")
        _say(f"    compared {b.num_shards} shard entries")
    else:
        rng = np.random.default_rng(cid)
        for s in _sample_shards(b, 4, rng):
            _say(f"    shard {s}: tokens {int(b.shards[s, 3] - b.shards[s, 2])}")
            ro, rl = oracle.attn_partial_paged(b.desc, b.q, b.k_pool, b.v_pool, b.k_scale, b.v_scale,
                                               b.block_table, b.shards[s])
            check_output(b.desc, o_h[s], lse_h[s], ro, rl, f"c{cid} full shard {s}")
    # split invariance at full size: the result is insensitive to the tiling used
    db2 = DeviceBatch(b, tile_tokens=1024)
    o2, lse2 = db2.partial()
    torch.cuda.synchronize()
    assert (o2 - o).abs().max().item() <= 1e-5 and (lse2 - lse).abs().max().item() <= 1e-5
    db.plan.close()
    db2.plan.close()


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5, 6, 7])
@pytest.mark.parametrize("tile_tokens", [0, 128])
@pytest.mark.parametrize("single_only", [False, True])
def test_final_rows_equal_partial_plus_merge(cid, tile_tokens, single_only):
    """Shards that are a whole output row write it in final form from the tile / reduction kernel; the rest goes
    through the row-indexed merge.  The result must be bit-identical to partial + merge of the same plan shape
    (same arithmetic, one cast), in f32 and bf16, and match the checker."""
    _say(f"[case] final rows, reduced config {cid} tile_tokens {tile_tokens}")
    b = W.reduced(cid)
    ps = b.desc.page_size
    tt = 0 if tile_tokens == 0 else max(ps, tile_tokens // ps * ps)
    base = DeviceBatch(b, tile_tokens=tt)
    o, lse = base.partial()
    rem_o, rem_lse = oracle.remote_partials(b)
    rem_o_t = torch.from_numpy(rem_o.astype(np.float32)).cuda()
    rem_lse_t = torch.from_numpy(rem_lse.astype(np.float32)).cuda()
    want, want_lse = _merge_on_gpu(base, torch.cat([o, rem_o_t]), torch.cat([lse, rem_lse_t]))
    S, R, d = b.num_shards, b.num_requests, b.desc
    db = DeviceBatch(b, tile_tokens=tt, final_rows=True, single_only=single_only)
    n_local = np.array([(b.part_index[b.part_offsets[r]:b.part_offsets[r + 1]] < S).sum() for r in range(R)])
    all_local = n_local == np.diff(b.part_offsets)
    assert (db.shard_final_row >= 0).sum() == int(n_local[all_local & ((n_local == 1) | (not single_only))].sum())
    grouped = not single_only and bool((all_local & (n_local > 1)).any())
    assert grouped == (cid in (1, 4, 7) and not single_only)
    for dt in (torch.float32, torch.bfloat16):
        out = torch.full((R, d.num_q_heads, d.head_dim_v), float("nan"), dtype=dt, device="cuda")
        out_lse = torch.full((R, d.num_q_heads), float("nan"), device="cuda")
        parts_o = torch.cat([torch.full_like(o, float("nan")), rem_o_t])
        parts_lse = torch.cat([torch.full_like(lse, float("nan")), rem_lse_t])
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table,
                                          parts_o[:S], parts_lse[:S], db.workspace, final_out=out, final_lse=out_lse)
        n_rest = len(db.rest_rows)
        if n_rest:
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, torch.from_numpy(db.rest_offsets).cuda(),
                                         torch.from_numpy(db.rest_index).cuda(), n_rest, out, out_lse,
                                         out_rows=torch.from_numpy(db.rest_rows).cuda())
        torch.cuda.synchronize()
        fin = torch.from_numpy(db.shard_final_row >= 0).cuda()
        if not grouped:
            assert torch.equal(out, want.to(dt)), f"c{cid} {dt}"
            assert torch.equal(out_lse, want_lse)
            # per-shard LSE is still delivered for every shard
            assert torch.equal(parts_lse[:S], lse)
        else:
            # shards of one row reduced as one segment: same operator, different association -> fp32 rounding
            err = (out.float() - want).abs()
            if dt == torch.float32:
                assert err.max().item() <= 1e-5, err.max().item()
            else:                                   # one bf16 rounding of a value that is within 1e-5
                assert bool((err <= 2.0 ** -8 * want.abs() + 1e-5).all()), err.max().item()
            assert (out_lse - want_lse).abs().max().item() <= 1e-5
        # O rows of shards that feed a final row are left alone, the others are as before
        assert torch.isnan(parts_o[:S][fin]).all() and torch.equal(parts_o[:S][~fin], o[~fin])
    ref_o, ref_lse = oracle.local_partials(b)
    ref_m, ref_mlse = oracle.merge_requests(np.concatenate([ref_o, rem_o]), np.concatenate([ref_lse, rem_lse]),
                                            b.part_offsets, b.part_index)
    check_output(b.desc, want.cpu().numpy(), want_lse.cpu().numpy(), ref_m, ref_mlse, f"c{cid} final rows")
    base.plan.close()
    db.plan.close()


def test_final_rows_errors():
    b = W.reduced(2)
    db = DeviceBatch(b)
    d = b.desc
    out = torch.empty((b.num_requests, d.num_q_heads, d.head_dim_v), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nanocp.NanocpError) as e:        # rows were never declared
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table,
                                          db.out_o, db.out_lse, db.workspace, final_out=out)
    assert e.value.status == nanocp.ESTATE
    with pytest.raises(nanocp.NanocpError) as e:        # the uploaded plan is immutable
        db.plan.set_final_rows(np.zeros(b.num_shards, np.int32), b.num_requests)
    assert e.value.status == nanocp.ESTATE
    plan = nanocp.Plan(db.desc, b.shards, b.q.shape[0], b.block_table.shape[0], b.block_table.shape[1])
    with pytest.raises(nanocp.NanocpError) as e:
        plan.set_final_rows(np.full(b.num_shards, b.num_requests, np.int32), b.num_requests)
    assert e.value.status == nanocp.EBOUNDS
    plan.close()
    db.plan.close()


@pytest.mark.parametrize("cid", [1, 2, 4, 5, 7])
def test_peaked_scores_exercise_the_running_maximum(cid):
    """Queries scaled by 32 (exact in every input type): scores spread over hundreds of log2 units, the softmax is
    nearly one-hot and the running maximum moves again and again inside a tile - the rescaling paths, the masked
    tails and the LSE at large magnitude are what is checked here."""
    _say(f"[case] peaked scores, reduced config {cid}")
    b = W.reduced(cid)
    if b.q.dtype == np.uint16:                                   # bf16 bits: exponent + 5
        q = b.q.copy()
        nz = (q & 0x7F80) != 0
        q[nz] = q[nz] + np.uint16(5 << 7)
        b.q = q
    else:
        b.q = (b.q * np.float32(32.0)).astype(np.float32)
    for tt in (0, 128):
        ps = b.desc.page_size
        db = DeviceBatch(b, tile_tokens=0 if tt == 0 else max(ps, tt // ps * ps))
        o, lse = db.partial()
        torch.cuda.synchronize()
        ref_o, ref_lse = oracle.local_partials(b)
        assert np.abs(ref_lse).max() > 20.0                      # the case really is extreme
        if b.desc.kv_dtype == "f32":
            # scores reach |s| ~ 100 here, where one fp32 ulp of a score is 8e-6: the 1e-5 bar of the ordinary cases
            # is below what fp32 scores can resolve; 1e-4 = a dozen ulps of the largest score
            assert np.abs(o.cpu().numpy() - ref_o).max() <= 1e-4
            assert np.abs(lse.cpu().numpy() - ref_lse).max() <= 1e-4
        else:
            check_output(b.desc, o.cpu().numpy(), lse.cpu().numpy(), ref_o, ref_lse, f"c{cid} peaked tt={tt}")
        db.plan.close()

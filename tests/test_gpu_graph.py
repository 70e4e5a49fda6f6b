"""The decode step (partial + merge) captured into a HIP graph and replayed: every replay must reproduce the
eager result bit for bit, with eager work and synchronisations between replays (the path records no memset
nodes: the work-queue counters re-arm themselves inside the kernel)."""
import numpy as np
import pytest
import torch

import paper_2605_21100_amd as nanocp
import workloads as W
from workloads.device import DeviceBatch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid", [3, 5])
def test_graph_replay_matches_eager(cid):
    print(f"[case] graph replay, reduced config {cid}", flush=True)
    b = W.reduced(cid, with_remote_kv=False)
    db = DeviceBatch(b, tile_tokens=256)
    d = b.desc
    S, R = b.num_shards, b.num_requests
    rem_o, rem_lse = W.synthetic_remote_partials(b)
    parts_o = torch.zeros((S + len(b.remote_meta), d.num_q_heads, d.head_dim_v), device="cuda")
    parts_lse = torch.zeros((S + len(b.remote_meta), d.num_q_heads), device="cuda")
    if len(b.remote_meta):
        parts_o[S:] = torch.from_numpy(rem_o).cuda()
        parts_lse[S:] = torch.from_numpy(rem_lse).cuda()
    po, pi = torch.from_numpy(b.part_offsets).cuda(), torch.from_numpy(b.part_index).cuda()
    out = torch.zeros((R, d.num_q_heads, d.head_dim_v), device="cuda")
    out_lse = torch.zeros((R, d.num_q_heads), device="cuda")

    def step():
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale,
                                          db.block_table, parts_o[:S], parts_lse[:S], db.workspace)
        nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, po, pi, R, out, out_lse)

    step()
    torch.cuda.synchronize()
    ref_out, ref_lse, ref_parts = out.clone(), out_lse.clone(), parts_o.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(4):
        out.zero_(), out_lse.zero_(), parts_o[:S].zero_()        # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(out_lse, ref_lse) and torch.equal(parts_o, ref_parts), rep
        step()                                   # an eager step in between must not disturb the graph's state
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out)
    db.plan.close()


def _compositions(b, rng):
    """Different batches over the same pools / block table / q rows: (shards, CSR over [local | remote]) each."""
    S = b.num_shards
    full = (b.shards.copy(), b.part_offsets.copy(), b.part_index.copy())
    # 2: a random subset of the requests, in another order, some ranges shortened (still inside their rows)
    keep = rng.permutation(b.num_requests)[: max(2, b.num_requests // 2)]
    shards, offs, idx = [], [0], []
    for r in keep:
        for pi in b.part_index[b.part_offsets[r]:b.part_offsets[r + 1]]:
            if pi < S:
                q_row, bt_row, kb, ke = b.shards[pi]
                if ke - kb > 40:
                    ke = kb + int(rng.integers(1, ke - kb))
                idx.append(len(shards))
                shards.append([q_row, bt_row, kb, ke])
        if len(idx) == offs[-1]:
            continue
        offs.append(len(idx))
    sub = (np.asarray(shards, np.int32), np.asarray(offs, np.int32), np.asarray(idx, np.int32))
    # 3: one single short request
    one = (b.shards[S - 1:S].copy(), np.array([0, 1], np.int32), np.array([0], np.int32))
    return [full, sub, one, full]


@pytest.mark.parametrize("cid", [1, 3, 4, 5])
def test_bucket_graph_replays_different_compositions(cid):
    """One captured graph (image-driven partial + dynamic merge) serves every batch composition of the bucket:
    between replays only the plan image and the merge lists are copied in.  Each replay must equal the eager
    result of an ordinary plan for that composition, bit for bit."""
    print(f"[case] bucket graph, reduced config {cid}", flush=True)
    import oracle
    from parity import check_output
    b = W.reduced(cid, with_remote_kv=False, hold_all=True) if cid in (3, 5) else W.reduced(cid, with_remote_kv=False)
    db = DeviceBatch(b, tile_tokens=256)          # pools, q, block table; its own plan is not used below
    d = b.desc
    rng = np.random.default_rng(17 + cid)
    comps = _compositions(b, rng)
    nq, nbt, mb = b.q.shape[0], b.block_table.shape[0], b.block_table.shape[1]
    plans = []
    for shards, offs, idx in comps:
        fin, r_offs, r_idx, r_rows = nanocp.split_final_rows(offs, idx, len(shards))
        pl = nanocp.Plan(db.desc, shards, nq, nbt, mb, 256).set_final_rows(fin, len(offs) - 1)
        plans.append((pl, shards, offs, idx, r_offs, r_idx, r_rows))
    seg_counts = []
    for pl, *_ in plans:
        t = pl.tiles()
        seg_counts.append(len(t))                        # safe upper bound for segments and slots
    bucket = nanocp.Bucket(max(p[0].num_tiles for p in plans), max(p[0].num_chunks for p in plans),
                           max(max(seg_counts), d.num_kv_heads * max(len(p[1]) for p in plans)), max(seg_counts))
    S_max, R_max = max(len(p[1]) for p in plans), max(len(p[2]) - 1 for p in plans)
    img_bytes = nanocp.bucket_plan_bytes(bucket)
    host_img = torch.empty(img_bytes, dtype=torch.uint8).pin_memory()
    dev_img = torch.zeros(img_bytes, dtype=torch.uint8, device="cuda")
    ws = torch.empty(max(nanocp.bucket_workspace_bytes(db.desc, bucket), 16), dtype=torch.uint8, device="cuda")
    parts_o = torch.zeros((S_max, d.num_q_heads, d.head_dim_v), device="cuda")
    parts_lse = torch.zeros((S_max, d.num_q_heads), device="cuda")
    out = torch.zeros((R_max, d.num_q_heads, d.head_dim_v), dtype=torch.bfloat16, device="cuda")
    out_lse = torch.zeros((R_max, d.num_q_heads), device="cuda")
    m_offs = torch.zeros(R_max + 1, dtype=torch.int32, device="cuda")
    m_idx = torch.zeros(S_max, dtype=torch.int32, device="cuda")
    m_rows = torch.zeros(R_max, dtype=torch.int32, device="cuda")
    m_count = torch.zeros(1, dtype=torch.int32, device="cuda")

    def inject(k):
        pl, shards, offs, idx, r_offs, r_idx, r_rows = plans[k]
        pl.pack(bucket, host_img)
        dev_img.copy_(host_img, non_blocking=True)
        m_offs[: len(r_offs)].copy_(torch.from_numpy(r_offs))
        m_idx[: len(r_idx)].copy_(torch.from_numpy(r_idx))
        m_rows[: len(r_rows)].copy_(torch.from_numpy(r_rows))
        m_count.fill_(len(r_rows))

    def step():
        nanocp.nanocp_decode_attn_partial_image(db.desc, bucket, dev_img, 0, mb, db.q, db.k_pool, db.v_pool, db.k_scale,
                                                db.v_scale, db.block_table, parts_o, parts_lse, ws, final_out=out,
                                                final_lse=out_lse)
        nanocp.nanocp_merge_partials_dyn(db.desc, parts_o, parts_lse, m_offs, m_idx, R_max, m_count, m_rows, out, out_lse)

    def eager(k):
        pl, shards, offs, idx, r_offs, r_idx, r_rows = plans[k]
        p2 = nanocp.Plan(db.desc, shards, nq, nbt, mb, 256)
        fin, *_ = nanocp.split_final_rows(offs, idx, len(shards))
        p2.set_final_rows(fin, len(offs) - 1).upload()
        S, R = len(shards), len(offs) - 1
        po = torch.zeros((S, d.num_q_heads, d.head_dim_v), device="cuda")
        pls = torch.zeros((S, d.num_q_heads), device="cuda")
        o = torch.zeros((R, d.num_q_heads, d.head_dim_v), dtype=torch.bfloat16, device="cuda")
        ol = torch.zeros((R, d.num_q_heads), device="cuda")
        w2 = torch.empty(max(p2.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
        nanocp.nanocp_decode_attn_partial(p2, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table, po, pls,
                                          w2, final_out=o, final_lse=ol)
        if len(r_rows):
            nanocp.nanocp_merge_partials(db.desc, po, pls, torch.from_numpy(r_offs).cuda(), torch.from_numpy(r_idx).cuda(),
                                         len(r_rows), o, ol, out_rows=torch.from_numpy(r_rows).cuda())
        torch.cuda.synchronize()
        p2.close()
        return o, ol

    inject(0)
    step()                                               # eager warm-up of the image path
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for k in range(len(plans)):
        want, want_lse = eager(k)
        out.zero_(), out_lse.zero_()
        inject(k)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        R = want.shape[0]
        assert torch.equal(out[:R], want) and torch.equal(out_lse[:R], want_lse), f"composition {k}"
    # the second composition against the checker, request by request
    pl, shards, offs, idx, *_ = plans[1]
    want, want_lse = eager(1)
    for r in range(min(3, len(offs) - 1)):
        sh = shards[idx[offs[r]:offs[r + 1]]]
        o_parts, l_parts = [], []
        for s in sh:
            ro, rl = oracle.attn_partial_paged(b.desc, b.q, b.k_pool, b.v_pool, b.k_scale, b.v_scale, b.block_table, s)
            o_parts.append(ro), l_parts.append(rl)
        mo, ml = oracle.merge(np.stack(o_parts), np.stack(l_parts))
        got = want[r].float().cpu().numpy()
        assert np.abs(got - mo).max() <= 2.0 ** -8 * np.abs(mo).max() + 2e-3 * np.abs(mo).max()
        assert np.abs(want_lse[r].cpu().numpy() - ml).max() <= 1e-4
    for pl, *_ in plans:
        pl.close()
    db.plan.close()

"""The decode step (partial + merge) captured into a HIP graph and replayed: every replay must reproduce the
eager result bit for bit, with eager work and synchronisations between replays (the path records no memset
nodes: the work-queue counters re-arm themselves inside the kernel)."""
import numpy as np
import pytest
import torch

import paper_2605_21100_amd as nanocp
import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid", [3, 5])
def test_graph_replay_matches_eager(cid):
    print(f"[case] graph replay, reduced config {cid}", flush=True)
    b = W.reduced(cid, with_remote_kv=False)
    db = nanocp.DeviceBatch(b, tile_tokens=256)
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

"""GPU end-to-end: the shard ranges come from the dual-balanced scheduler (Alg. 1: node choice, bucket degree,
smallest-KV participants, WaterFill split) instead of a fixed 1/d rule; one instance's share of the resulting
batch runs through plan -> partial attention -> merge and must reproduce exact attention of every request it
touches (remote shards' partials come from the float64 checker, as in the other parity tests)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_21100_amd as nanocp
import workloads as W
from workloads.device import DeviceBatch
from parity import check_output
from workloads.batches import build_batch

pytestmark = pytest.mark.gpu

DESCS = {
    "bf16": W.AttnDesc("gqa", "bf16", "bf16", 64, 4, 128, 128, 64, 128 ** -0.5),
    "fp8": W.AttnDesc("gqa", "bf16", "fp8", 64, 4, 128, 128, 64, 128 ** -0.5),
    "mla": W.AttnDesc("mla", "bf16", "bf16", 128, 1, 576, 512, 64, 192 ** -0.5),
}


def _schedule(seed, num_requests):
    """One 8-instance node with uneven resident load; a long-tailed request stream placed one by one."""
    rng = np.random.default_rng(seed)
    sched = nanocp.Scheduler([8], kv_capacity=200_000, bucket_max_len=[700, 1500, 3000, 1 << 40],
                             bucket_degree=[1, 2, 4, 8])
    sched.kv_load[:] = rng.integers(0, 3000, size=8)        # KV already resident on each instance
    lengths = np.clip(np.round(np.exp(rng.normal(np.log(400), 1.2, size=num_requests))), 16, 12000).astype(np.int64)
    decisions = sched.place(lengths)
    assert all(d["scheduled"] for d in decisions)
    return rng, lengths, decisions


@pytest.mark.parametrize("kv", ["bf16", "fp8", "mla"])
def test_scheduler_splits_drive_the_attention_path(kv):
    print(f"[case] scheduler-made batch, {kv}", flush=True)
    rng, lengths, decisions = _schedule(20260521 + 40, 48)
    degrees = [len(d["P"]) for d in decisions]
    assert max(degrees) >= 4 and min(degrees) == 1           # the stream exercises several CP degrees
    # the instance that takes part in the most split requests
    counts = np.zeros(8, int)
    for d in decisions:
        if len(d["P"]) > 1:
            counts[d["P"]] += 1
    inst = int(np.argmax(counts))
    lens, ranges, local = [], [], []
    for L, d in zip(lengths, decisions):
        if inst not in d["P"]:
            continue
        assert sum(d["split"]) == L
        cuts = np.concatenate([[0], np.cumsum(d["split"])])   # consecutive token ranges in P_r's order
        lens.append(int(L))
        ranges.append([(int(cuts[i]), int(cuts[i + 1])) for i in range(len(d["P"]))])
        local.append([d["P"].index(inst)])
    assert sum(len(r) > 1 for r in ranges) >= 3
    uneven = [r for r in ranges if len(r) > 1 and len({e - b for b, e in r}) > 1]
    assert uneven                                             # WaterFill really produced unequal shards
    b = build_batch(f"sched_e2e_{kv}", 20260521 + 40, DESCS[kv], np.asarray(lens, np.int64), ranges, local, rng)

    for final_rows in (False, True):
        db = DeviceBatch(b, final_rows=final_rows)
        S, R, d = b.num_shards, b.num_requests, b.desc
        out = torch.full((R, d.num_q_heads, d.head_dim_v), float("nan"), device="cuda")
        out_lse = torch.full((R, d.num_q_heads), float("nan"), device="cuda")
        rem_o, rem_lse = oracle.remote_partials(b)
        parts_o = torch.cat([db.out_o, torch.from_numpy(rem_o.astype(np.float32)).cuda()])
        parts_lse = torch.cat([db.out_lse, torch.from_numpy(rem_lse.astype(np.float32)).cuda()])
        if final_rows:
            nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale,
                                              db.block_table, parts_o[:S], parts_lse[:S], db.workspace,
                                              final_out=out, final_lse=out_lse)
            if len(db.rest_rows):
                nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, torch.from_numpy(db.rest_offsets).cuda(),
                                             torch.from_numpy(db.rest_index).cuda(), len(db.rest_rows), out, out_lse,
                                             out_rows=torch.from_numpy(db.rest_rows).cuda())
        else:
            nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale,
                                              db.block_table, parts_o[:S], parts_lse[:S], db.workspace)
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, torch.from_numpy(b.part_offsets).cuda(),
                                         torch.from_numpy(b.part_index).cuda(), R, out, out_lse)
        torch.cuda.synchronize()
        if not final_rows:
            ref_o, ref_lse = oracle.local_partials(b)
            check_output(d, parts_o[:S].cpu().numpy(), parts_lse[:S].cpu().numpy(), ref_o, ref_lse, f"{kv} partials")
        for r in range(R):                                    # every request against exact unsharded attention
            full_o, full_lse = oracle.request_full_attention(b, r)
            check_output(d, out[r].cpu().numpy(), out_lse[r].cpu().numpy(), full_o, full_lse,
                         f"{kv} request {r} (d={len(ranges[r])}, final_rows={final_rows})")
        db.plan.close()

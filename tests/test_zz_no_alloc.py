"""nanocp_decode_attn_partial_image_static: the plan-image entry point for callers that cannot allocate, with the
tile partials in the library's own static scratch.  Its output must equal, bit for bit, that of
nanocp_decode_attn_partial_image with a caller-owned workspace (same kernels, same reduction order), on two calls in a
row -- the second on a smaller batch, which finds the first call's partials still in the scratch."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_21100_amd as nanocp
import workloads as W
from workloads.device import DeviceBatch

pytestmark = pytest.mark.gpu


def _image_case(b, tile_tokens):
    """Pools and plan image of batch b; every request whose partials are all local is a final row."""
    db = DeviceBatch(b, tile_tokens=tile_tokens, final_rows=True)
    d = b.desc
    S = b.num_shards
    nt = db.plan.num_tiles
    bucket = nanocp.Bucket(nt + 8, db.plan.num_chunks + 8, nt + S * d.num_kv_heads + 8, nt + 8)
    host_img = torch.empty(nanocp.bucket_plan_bytes(bucket), dtype=torch.uint8).pin_memory()
    db.plan.pack(bucket, host_img)
    return db, bucket, host_img


def _run(db, bucket, host_img, static, num_cus):
    b, d = db.batch, db.batch.desc
    S, R = b.num_shards, b.num_requests
    dev_img = host_img.cuda()                           # a fresh image per launch: the work-queue counters start at 0
    o = torch.full((S, d.num_q_heads, d.head_dim_v), float("nan"), device="cuda")
    lse = torch.full((S, d.num_q_heads), float("nan"), device="cuda")
    fin = torch.full((R, d.num_q_heads, d.head_dim_v), float("nan"), dtype=torch.bfloat16, device="cuda")
    fin_lse = torch.full((R, d.num_q_heads), float("nan"), device="cuda")
    mb = b.block_table.shape[1]
    if static:
        nanocp.nanocp_decode_attn_partial_image_static(db.desc, bucket, dev_img, num_cus, mb, db.q, db.k_pool, db.v_pool,
                                                       db.k_scale, db.v_scale, db.block_table, o, lse, final_out=fin,
                                                       final_lse=fin_lse)
    else:
        ws = torch.empty(max(nanocp.bucket_workspace_bytes(db.desc, bucket), 16), dtype=torch.uint8, device="cuda")
        nanocp.nanocp_decode_attn_partial_image(db.desc, bucket, dev_img, num_cus, mb, db.q, db.k_pool, db.v_pool,
                                                db.k_scale, db.v_scale, db.block_table, o, lse, ws, final_out=fin,
                                                final_lse=fin_lse)
    torch.cuda.synchronize()
    return o, lse, fin, fin_lse


def _same(a, b):
    return all(torch.equal(torch.nan_to_num(x.float(), nan=12345.0), torch.nan_to_num(y.float(), nan=12345.0))
               for x, y in zip(a, b))


@pytest.mark.parametrize("first, second", [((3, 128), (2, 256)), ((5, 128), (5, 448)), ((1, 32), (1, 64)),
                                           ((4, 256), (7, 448))])
def test_static_scratch_entry_point_equals_workspace_entry_point(first, second):
    print(f"[case] static-scratch entry point: reduced configs {first} then {second}", flush=True)
    num_cus = torch.cuda.get_device_properties(0).multi_processor_count
    cases = []
    for cid, tt in (first, second):
        b = W.reduced(cid, with_remote_kv=False)
        ps = b.desc.page_size
        cases.append(_image_case(b, max(ps, tt // ps * ps)))
    # the second input is the smaller one, and both really use partial slots
    need = [nanocp.bucket_workspace_bytes(db.desc, bk) for db, bk, _ in cases]
    assert 0 < need[1] < need[0] <= nanocp.STATIC_SCRATCH_BYTES, need
    want = [_run(db, bk, img, False, num_cus) for db, bk, img in cases]
    got = [_run(db, bk, img, True, num_cus) for db, bk, img in cases]       # two static calls in a row
    for i in range(2):
        assert _same(got[i], want[i]), f"call {i}"
    for db, _, _ in cases:
        db.plan.close()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    print("[case] static-scratch entry point: size and argument errors", flush=True)
    b = W.reduced(4, with_remote_kv=False)
    db, bucket, host_img = _image_case(b, 256)
    num_cus = torch.cuda.get_device_properties(0).multi_processor_count
    G = b.desc.num_q_heads // b.desc.num_kv_heads
    per_slot = G * (b.desc.head_dim_v + 1) * 4
    big = nanocp.Bucket(bucket.max_tiles, bucket.max_chunks, bucket.max_segs, nanocp.STATIC_SCRATCH_BYTES // per_slot + 8)
    assert nanocp.bucket_workspace_bytes(db.desc, big) > nanocp.STATIC_SCRATCH_BYTES
    d = b.desc
    o = torch.empty((b.num_shards, d.num_q_heads, d.head_dim_v), device="cuda")
    lse = torch.empty((b.num_shards, d.num_q_heads), device="cuda")
    img = torch.zeros(nanocp.bucket_plan_bytes(big), dtype=torch.uint8, device="cuda")
    args = (db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table, o, lse)
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.nanocp_decode_attn_partial_image_static(db.desc, big, img, num_cus, b.block_table.shape[1], *args)
    assert e.value.status == nanocp.EBOUNDS
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.nanocp_decode_attn_partial_image_static(db.desc, bucket, host_img.cuda(), 0, b.block_table.shape[1], *args)
    assert e.value.status == nanocp.EINVAL
    db.plan.close()

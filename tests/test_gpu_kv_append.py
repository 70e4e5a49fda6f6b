"""nanocp_kv_append against the layout definition of include/nanocp.h written out with numpy indexing: the tokens of
a seeded batch are read out of its pools as plain rows, appended on the GPU into empty pools, and (a) the pools must
be bit-identical wherever a token lives, (b) attention over the rebuilt pools must be bit-identical to attention
over the original ones (which hold NaN patterns in the unused slots, the rebuilt ones zeros)."""
import numpy as np
import pytest
import torch

import paper_2605_21100_amd as nanocp
import workloads as W
from workloads.device import DeviceBatch, to_device

pytestmark = pytest.mark.gpu


def _token_table(b):
    """(bt_row, position) of every token of every shard, once."""
    rows, pos = [], []
    for _, bt_row, lo, hi in b.shards:
        rows.append(np.full(hi - lo, bt_row, np.int32))
        pos.append(np.arange(lo, hi, dtype=np.int32))
    tab = np.unique(np.stack([np.concatenate(rows), np.concatenate(pos)], 1), axis=0)
    return tab[:, 0].copy(), tab[:, 1].copy()


@pytest.mark.parametrize("cid", [1, 2, 4, 5])
def test_append_builds_the_documented_layouts(cid):
    print(f"[case] kv append, reduced config {cid}", flush=True)
    b = W.reduced(cid)
    d = b.desc
    ps, Hkv, Dk, Dv = d.page_size, d.num_kv_heads, d.head_dim_qk, d.head_dim_v
    bt_row, position = _token_table(b)
    page = b.block_table[bt_row, position // ps]
    slot = position % ps
    k, v = b.k_pool, b.v_pool
    if d.kind == "mla":
        # k_pool [pages, ps, Dk]
        k_rows = k[page, slot]                                           # [n, Dk]
        v_rows = None
        want_k = np.zeros_like(k)
        want_k[page, slot] = k_rows
        want_v = None
    else:
        x = 16 // k.dtype.itemsize
        grp, w = slot // (4 * x), slot % (4 * x)
        # k_pool [pages, Hkv, ps/4x, Dk/x, 4x, x]: vector (c, w) = dims [cx, cx + x) of slot w of the group
        k_rows = k[page, :, grp, :, w, :].reshape(len(page), Hkv, Dk)     # [n, Hkv, Dk/x, x] -> dims in order
        want_k = np.zeros_like(k)
        want_k[page, :, grp, :, w, :] = k[page, :, grp, :, w, :]
        # v_pool [pages, Hkv, ps/x, Dv, x]: slot w = 16b + 4g + i is element 4b + i of vector u = 4 grp + g
        u = 4 * grp + (w % 16) // 4
        e = 4 * (w // 16) + w % 4
        v_rows = v[page, :, u, :, e]                                      # [n, Hkv, Dv]
        want_v = np.zeros_like(v)
        want_v[page, :, u, :, e] = v_rows
    db = DeviceBatch(b)
    o_ref, lse_ref = (t.clone() for t in db.partial())
    k_dev = torch.zeros_like(db.k_pool)
    v_dev = None if db.v_pool is None else torch.zeros_like(db.v_pool)
    nanocp.nanocp_kv_append(db.desc, to_device(np.ascontiguousarray(k_rows)),
                            None if v_rows is None else to_device(np.ascontiguousarray(v_rows)),
                            torch.from_numpy(bt_row).cuda(), torch.from_numpy(position).cuda(), k_dev, v_dev,
                            db.block_table)
    torch.cuda.synchronize()

    def bits(t):
        return t.view(torch.int16 if t.dtype == torch.bfloat16 else t.dtype).cpu().numpy().view(k.dtype)

    assert np.array_equal(bits(k_dev).view(np.uint8), want_k.view(np.uint8))
    if want_v is not None:
        assert np.array_equal(bits(v_dev).view(np.uint8), want_v.view(np.uint8))
    # attention over the rebuilt pools: identical, the unused slots are masked either way
    o, lse = torch.empty_like(o_ref), torch.empty_like(lse_ref)
    nanocp.nanocp_decode_attn_partial(db.plan, db.q, k_dev, v_dev, db.k_scale, db.v_scale, db.block_table, o, lse,
                                      db.workspace)
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    db.plan.close()


def test_append_errors():
    b = W.reduced(2)
    db = DeviceBatch(b)
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    rows = torch.zeros((1, 4, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nanocp.NanocpError) as e:                  # V rows missing for a GQA cache
        nanocp.nanocp_kv_append(db.desc, rows, None, one, one, db.k_pool, db.v_pool, db.block_table)
    assert e.value.status == nanocp.EINVAL
    bad = nanocp.make_desc("gqa", "bf16", "bf16", 64, 4, 128, 128, 48, 0.1)   # page size not a multiple of 32
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.nanocp_kv_append(bad, rows, rows, one, one, db.k_pool, db.v_pool, db.block_table)
    assert e.value.status == nanocp.ESHAPE
    db.plan.close()

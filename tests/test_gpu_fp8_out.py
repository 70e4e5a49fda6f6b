"""FP8 (OCP E4M3FN) output epilogue of the Phase 4 merge and of the final rows written by the attention kernels:
stored code = e4m3(value * (1 / out_scale)), round to nearest even, saturating, with a caller-supplied static scale.

Checked (i) against the format itself: the device encoder must agree bit for bit with the generators' numpy encoder
on a dense set of values (every code, every rounding boundary and its float32 neighbours, the subnormal range, the
saturating range); (ii) bit for bit against the same kernels' float32 rows pushed through that encoder (same
arithmetic, one cast); (iii) against the float64 checker's exact attention: the decoded fp8 value must lie within the
parity bar of the attention result plus half an E4M3 step at that magnitude (relative 2^-4, or 2^-10 of the scale in
the subnormal range)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_21100_amd as nanocp
import workloads as W
from workloads import numfmt
from parity import FP32_ABS, LOWP_REL
from workloads.device import DeviceBatch

pytestmark = pytest.mark.gpu


def _ordered(code):
    """Signed position of an E4M3 code on the number line (codes of one sign are monotone in their low 7 bits)."""
    c = code.astype(np.int32)
    return np.where(c & 0x80, -(c & 0x7F), c & 0x7F)


def _merge_identity(values, out_scale):
    """Push float32 values through the merge kernel as single-part rows (a copy) with fp8 output."""
    Hq, Dv = 4, 64
    n = -(-values.size // (Hq * Dv))
    buf = np.zeros(n * Hq * Dv, np.float32)
    buf[:values.size] = values
    desc = nanocp.make_desc("gqa", "bf16", "bf16", Hq, 1, 64, Dv, 64, 1.0, out_scale)
    o = torch.from_numpy(buf.reshape(n, Hq, Dv)).cuda()
    lse = torch.zeros((n, Hq), device="cuda")
    offs = torch.arange(n + 1, dtype=torch.int32, device="cuda")
    out = torch.zeros((n, Hq, Dv), dtype=torch.uint8, device="cuda")
    nanocp.nanocp_merge_partials(desc, o, lse, offs, None, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().reshape(-1)[:values.size]


def test_device_e4m3_encoder_matches_the_format():
    print("[case] fp8 output: encoder against the format definition", flush=True)
    codes = np.arange(256, dtype=np.uint8)
    table = oracle.E4M3FN_TABLE.astype(np.float64)
    finite = np.isfinite(table)
    vals = [table[finite]]
    pos = np.sort(table[finite & (table >= 0)])
    mid = (pos[:-1] + pos[1:]) / 2                        # rounding boundaries: exact in float32
    for m in (mid, -mid):
        m32 = m.astype(np.float32)
        vals += [m32, np.nextafter(m32, np.float32(np.inf)), np.nextafter(m32, np.float32(-np.inf))]
    rng = np.random.default_rng(11)
    vals += [rng.standard_normal(4096) * s for s in (1e-3, 0.02, 1.0, 30.0, 300.0)]
    vals += [np.array([448.0, 449.0, 463.9, 464.0, 465.0, 1e6, 3e38, -448.0, -464.0, -1e9, 0.0, -0.0, 2.0 ** -10,
                       2.0 ** -9, 1.5 * 2.0 ** -9, 2.5 * 2.0 ** -9, 2.0 ** -6, 1e-30, -1e-30])]
    x = np.concatenate([np.asarray(v, np.float32) for v in vals])
    for scale in (1.0, 0.0371, 4.0):
        got = _merge_identity(x, scale)
        want = numfmt.f32_to_e4m3fn(x * (np.float32(1) / np.float32(scale)))
        bad = np.nonzero(got != want)[0]
        assert bad.size == 0, (scale, x[bad[:5]], got[bad[:5]], want[bad[:5]])
    # every code decodes (the checker's table, written from the format) and re-encodes to itself
    assert np.array_equal(_merge_identity(table[finite].astype(np.float32), 1.0), codes[finite])
    # infinities saturate, NaN becomes the NaN code, out_scale = 0 means 1
    sp = _merge_identity(np.array([np.inf, -np.inf, np.nan, 1.0], np.float32), 0.0)
    assert sp.tolist() == [0x7E, 0xFE, 0x7F, 0x38] or sp.tolist() == [0x7E, 0xFE, 0xFF, 0x38]


@pytest.mark.parametrize("cid", [1, 3, 4, 5, 7])
@pytest.mark.parametrize("tile_tokens", [0, 128])
def test_fp8_final_rows_and_merge(cid, tile_tokens):
    """Every writer of final rows (tile kernels' direct path, fused last-arriver reduction, reduction kernel, merge)
    with fp8 output, against its own float32 output and against the checker."""
    print(f"[case] fp8 output rows, reduced config {cid} tile_tokens {tile_tokens}", flush=True)
    b = W.reduced(cid)
    ps = b.desc.page_size
    tt = 0 if tile_tokens == 0 else max(ps, tile_tokens // ps * ps)
    d, S, R = b.desc, b.num_shards, b.num_requests
    ref_o, ref_lse = oracle.local_partials(b)
    rem_o, rem_lse = oracle.remote_partials(b)
    ref_m, _ = oracle.merge_requests(np.concatenate([ref_o, rem_o]), np.concatenate([ref_lse, rem_lse]),
                                     b.part_offsets, b.part_index)
    out_scale = float(np.float32(np.abs(ref_m).max() / 448.0 * 1.25))     # a static scale with some headroom
    db = DeviceBatch(b, tile_tokens=tt, final_rows=True, out_scale=out_scale)
    rem_o_t = torch.from_numpy(rem_o.astype(np.float32)).cuda()
    rem_lse_t = torch.from_numpy(rem_lse.astype(np.float32)).cuda()
    res = {}
    for dt in (torch.float32, torch.uint8):
        out = torch.zeros((R, d.num_q_heads, d.head_dim_v), dtype=dt, device="cuda")
        parts_o = torch.cat([torch.zeros((S, d.num_q_heads, d.head_dim_v), device="cuda"), rem_o_t])
        parts_lse = torch.cat([torch.zeros((S, d.num_q_heads), device="cuda"), rem_lse_t])
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table,
                                          parts_o[:S], parts_lse[:S], db.workspace, final_out=out)
        if len(db.rest_rows):
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, torch.from_numpy(db.rest_offsets).cuda(),
                                         torch.from_numpy(db.rest_index).cuda(), len(db.rest_rows), out,
                                         out_rows=torch.from_numpy(db.rest_rows).cuda())
        torch.cuda.synchronize()
        res[dt] = out.cpu().numpy()
    f32, q8 = res[torch.float32], res[torch.uint8]
    inv = np.float32(1) / np.float32(out_scale)
    assert np.array_equal(q8, numfmt.f32_to_e4m3fn(f32 * inv)), "fp8 rows != encoder(f32 rows)"
    got = oracle.E4M3FN_TABLE[q8] * out_scale                              # decoded with the checker's own table
    if d.kv_dtype == "f32":
        bar = np.full_like(ref_m, FP32_ABS)
    else:
        bar = LOWP_REL * np.abs(ref_m) + LOWP_REL * np.sqrt((ref_m ** 2).mean(axis=-1, keepdims=True))
    half_step = np.maximum(2.0 ** -10, (np.abs(ref_m) + bar) / out_scale * 2.0 ** -4) * out_scale
    assert np.all(np.abs(got - ref_m) <= bar + 1.001 * half_step), float((np.abs(got - ref_m) - bar - half_step).max())
    # and most codes are exactly the checker's (a sanity check that the bound above is not what carries the test)
    want = numfmt.f32_to_e4m3fn((ref_m / out_scale).astype(np.float32))
    big = np.abs(ref_m) / out_scale >= 2.0 ** -3
    assert ((_ordered(q8) != _ordered(want)) & big).sum() <= 0.02 * big.sum()
    assert (q8 & 0x7F).max() <= 0x7E and (q8 & 0x7F).max() >= 0x70      # no NaN code; the scale uses the top binades
    db.plan.close()


@pytest.mark.parametrize("cid", [3, 5])
def test_fp8_output_full_size(cid):
    """Benchmark-size batch in the benchmark's launch configuration, rows written as fp8 by the attention kernel and the
    merge: equal to the encoder applied to the float32 rows of the same launch configuration."""
    print(f"[case] fp8 output rows, full-size config {cid}", flush=True)
    b = W.FULL[cid](with_remote_kv=False)
    d, S, R = b.desc, b.num_shards, b.num_requests
    out_scale = 0.004
    db = DeviceBatch(b, final_rows=True, out_scale=out_scale)
    rem_o, rem_lse = W.synthetic_remote_partials(b)
    res = {}
    for dt in (torch.float32, torch.uint8):
        out = torch.zeros((R, d.num_q_heads, d.head_dim_v), dtype=dt, device="cuda")
        parts_o = torch.cat([torch.zeros((S, d.num_q_heads, d.head_dim_v), device="cuda"),
                             torch.from_numpy(rem_o).cuda().reshape(-1, d.num_q_heads, d.head_dim_v)])
        parts_lse = torch.cat([torch.zeros((S, d.num_q_heads), device="cuda"),
                               torch.from_numpy(rem_lse).cuda().reshape(-1, d.num_q_heads)])
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, db.k_pool, db.v_pool, db.k_scale, db.v_scale, db.block_table,
                                          parts_o[:S], parts_lse[:S], db.workspace, final_out=out)
        if len(db.rest_rows):
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, torch.from_numpy(db.rest_offsets).cuda(),
                                         torch.from_numpy(db.rest_index).cuda(), len(db.rest_rows), out,
                                         out_rows=torch.from_numpy(db.rest_rows).cuda())
        torch.cuda.synchronize()
        res[dt] = out.cpu().numpy()
    assert np.array_equal(res[torch.uint8], numfmt.f32_to_e4m3fn(res[torch.float32] * (np.float32(1) / np.float32(out_scale))))
    db.plan.close()

"""Test / benchmark harness glue: a synthetic batch made resident in HBM, with its plan, outputs and workspace.

Not imported by `workloads/__init__` (the float64 checker must not pull in the GPU library); tests, bench.py and
the smoke entry import it explicitly.  Marshalling only -- no attention arithmetic.
"""
import numpy as np


def desc_from(d, out_scale=0.0):
    """The library's AttnDesc from the generator's description of the problem shape."""
    import paper_2605_21100_amd as nanocp
    return nanocp.make_desc(d.kind, d.q_dtype, d.kv_dtype, d.num_q_heads, d.num_kv_heads, d.head_dim_qk,
                            d.head_dim_v, d.page_size, d.softmax_scale, out_scale)


def to_device(arr, device="cuda"):
    """numpy raw buffer -> torch device tensor of the matching element type (bf16 bits, fp8 bytes)."""
    import torch
    if arr is None:
        return None
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


class DeviceBatch:
    """A synthetic batch resident in HBM plus its plan, outputs and workspace."""

    def __init__(self, batch, tile_tokens=0, num_cus=0, device="cuda", final_rows=False, single_only=False,
                 out_scale=0.0):
        import torch
        import paper_2605_21100_amd as nanocp
        self.batch = batch
        d = batch.desc
        self.desc = desc_from(d, out_scale)
        self.q = to_device(batch.q, device=device)
        self.k_pool = to_device(batch.k_pool, device=device)
        self.v_pool = to_device(batch.v_pool, device=device)
        self.k_scale = to_device(batch.k_scale, device=device)
        self.v_scale = to_device(batch.v_scale, device=device)
        self.block_table = to_device(batch.block_table, device=device)
        S = batch.shards.shape[0]
        self.plan = nanocp.Plan(self.desc, batch.shards, batch.q.shape[0], batch.block_table.shape[0],
                                batch.block_table.shape[1], tile_tokens, num_cus)
        if final_rows:      # requests whose partials are all local skip the merge
            fin, self.rest_offsets, self.rest_index, self.rest_rows = nanocp.split_final_rows(
                batch.part_offsets, batch.part_index, S, single_only)
            self.plan.set_final_rows(fin, batch.num_requests)
            self.shard_final_row = fin
        self.plan.upload()
        self.out_o = torch.empty((S, d.num_q_heads, d.head_dim_v), dtype=torch.float32, device=device)
        self.out_lse = torch.empty((S, d.num_q_heads), dtype=torch.float32, device=device)
        self.workspace = torch.empty(max(self.plan.workspace_bytes, 16), dtype=torch.uint8, device=device)

    def partial(self, tile_clock=None):
        import paper_2605_21100_amd as nanocp
        nanocp.nanocp_decode_attn_partial(self.plan, self.q, self.k_pool, self.v_pool, self.k_scale, self.v_scale,
                                          self.block_table, self.out_o, self.out_lse, self.workspace, tile_clock)
        return self.out_o, self.out_lse

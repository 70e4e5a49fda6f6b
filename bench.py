#!/usr/bin/env python3
"""Benchmark of the DCP decode-attention hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch already resident in HBM:
    nanocp_decode_attn_partial (tile kernel + tile reduce)  ->  nanocp_merge_partials.
The plan (host tile work-list) is built and uploaded once, outside the timed region, as the paper
amortises scheduling over decode iterations.  Default workload: config 3, the mixed long-tail DCP
batch the headline metric is quoted on.  Successive steps alternate between two copies of the KV
pools so that no step can be served from the 256 MB last-level cache.

Prints ONE JSON line (last line of stdout).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the tile kernel, from rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by a 1 GiB copy
# (summaries and commands under profiles/); valid for the default plan of the named config only.
MEASURED_TRAFFIC_BYTES = {3: (1203400000, "profiles/gqa_mfma_bf16_config3_mixed_dcp.md"),
                          5: (764320000, "profiles/gqa_mfma_fp8_config5_long_shard.md"),
                          2: (656040000, "profiles/gqa_mfma_bf16_config2_local.md"),
                          4: (1585600000, "profiles/mla_mfma_bf16_config4.md"),
                          6: (677260000, "profiles/gqa_mfma_bf16_config6_microbench.md"),   # 3 long requests per node
                          7: (1468300000, "profiles/mla64_mfma_bf16_config7.md")}
METRIC = "decode-attention KV GB/s (% of HBM peak) + µs/step, mixed ragged DCP batch"
WORKLOAD_NAMES = {1: "config1: tiny fp32 GQA", 2: "config2: bf16 GQA 64 local requests U[1024,8192]",
                  3: "config3: mixed long-tail DCP batch, 128 requests lognormal(median 2048, sigma 1.2), bf16 GQA 64q/4kv d128",
                  4: "config4: MLA-absorbed bf16, 128 heads, 576/512, 64 requests U[4096,32768], half split CP=2",
                  5: "config5: fp8 KV, 131072-token shard (CP=8 of 1,048,576) + 256 short requests",
                  6: "config6: the paper's micro-benchmark batch, 64 x 2048-token requests + a 1/8 slice of each of "
                     "{n} 524288-token requests, bf16 GQA 64q/4kv d128",
                  7: "config7: config 4's recipe with 64 query heads (MLA-absorbed bf16, 576/512)"}


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_pass(batch, order, lens, budget_s):
    """Run the float64 checker over shard entries (longest first, repeated) for about budget_s seconds."""
    import oracle
    done_tokens, picked, passes = 0, 0, 0
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < budget_s / 2:           # repeat the pass until about half the budget is spent
        for s in order:
            oracle.attn_partial_paged(batch.desc, batch.q, batch.k_pool, batch.v_pool, batch.k_scale, batch.v_scale,
                                      batch.block_table, batch.shards[s])
            done_tokens += int(lens[s])
            picked += 1
            if time.perf_counter() - t0 > budget_s:
                break
        passes += 1
    return done_tokens, picked, passes, time.perf_counter() - t0


def cpu_baseline(batch, budget_s=12.0):
    """Time the float64 checker (as it stands) on a bounded sample of the same workload's shard entries: once with the
    threads numpy's BLAS takes by itself (all host cores of the box's share), once limited to one thread."""
    from threadpoolctl import threadpool_info, threadpool_limits
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    lens = batch.shards[:, 3] - batch.shards[:, 2]
    order = np.argsort(-lens)            # longest first: the sample keeps the workload's long tail
    bpt = batch.desc.kv_bytes_per_token
    tok, picked, passes, dt = _oracle_pass(batch, order, lens, budget_s)
    with threadpool_limits(limits=1):
        tok1, picked1, passes1, dt1 = _oracle_pass(batch, order, lens, budget_s)
    return {"value": tok * bpt / dt / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "single_thread": {"value": tok1 * bpt / dt1 / 1e9, "unit": "GB/s", "cores": 1,
                              "sample": f"{picked1} shard entries, longest first, in {passes1} pass(es) "
                                        f"({tok1} tokens, {dt1:.1f} s)"},
            "cpu_model": _cpu_model(), "host_cpus_visible": os.cpu_count(),
            "sample": f"{picked} shard entries, longest first, in {passes} pass(es) over the {len(lens)} entries of the "
                      f"workload ({tok} tokens, {dt:.1f} s), float64 numpy partial attention"}


def quick_config(cid, steps, warmup):
    """One workload's step time and event-timed attention launch, in the default launch configuration (automatic
    tiling, final rows from the kernel, two pool copies alternated).  Used for the per-config table."""
    import torch
    import paper_2605_21100_amd as nanocp
    import workloads as W
    from workloads.device import DeviceBatch
    batch = W.FULL[cid](with_remote_kv=False)
    d = batch.desc
    db = DeviceBatch(batch, final_rows=True)
    pools = [(db.k_pool, db.v_pool, db.k_scale, db.v_scale)]
    pools.append(tuple(None if t is None else t.clone() for t in pools[0]))
    S, R = batch.num_shards, batch.num_requests
    rem_o, rem_lse = W.synthetic_remote_partials(batch)
    n_rem = rem_o.shape[0]
    parts_o = torch.empty((S + n_rem, d.num_q_heads, d.head_dim_v), dtype=torch.float32, device="cuda")
    parts_lse = torch.empty((S + n_rem, d.num_q_heads), dtype=torch.float32, device="cuda")
    if n_rem:
        parts_o[S:] = torch.from_numpy(rem_o).cuda()
        parts_lse[S:] = torch.from_numpy(rem_lse).cuda()
    out = torch.empty((R, d.num_q_heads, d.head_dim_v), dtype=torch.bfloat16, device="cuda")
    n_rest = len(db.rest_rows)
    rest_offsets, rest_index = torch.from_numpy(db.rest_offsets).cuda(), torch.from_numpy(db.rest_index).cuda()
    rest_rows = torch.from_numpy(db.rest_rows).cuda()

    def step(i, ev=None):
        k, v, ks, vs = pools[i & 1]
        if ev:
            ev[0].record()
        nanocp.nanocp_decode_attn_partial(db.plan, db.q, k, v, ks, vs, db.block_table, parts_o[:S], parts_lse[:S],
                                          db.workspace, final_out=out)
        if ev:
            ev[1].record()
        if n_rest:
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, rest_offsets, rest_index, n_rest, out,
                                         out_rows=rest_rows)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    n_ev = min(steps, 100)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for i in range(n_ev):
        step(i, evs[i])
    torch.cuda.synchronize()
    launch_us = float(np.mean([a.elapsed_time(b) for a, b in evs]) * 1e3)
    res = {"workload": WORKLOAD_NAMES[cid].format(n=3), "kernel": db.plan.kernel, "kv_bytes": int(batch.kv_bytes),
           "us_per_step": us, "kv_GBs": batch.kv_bytes / us / 1e3, "pct_of_hbm_peak": batch.kv_bytes / us / 1e3 / 80.0,
           "launch_us_mean": launch_us, "frac": batch.kv_bytes / launch_us / 1e3 / HBM_PEAK_GBS,
           "tiles": int(db.plan.num_tiles), "rows_merged": int(n_rest)}
    if d.kind == "mla":
        flops = 2.0 * (d.head_dim_qk + d.head_dim_v) * d.num_q_heads * batch.local_tokens
        res["mfma_frac"] = flops / (launch_us * 1e-6) / 1e12 / 2500.0
    db.plan.close()
    del db, pools, parts_o, parts_lse, out
    torch.cuda.empty_cache()
    return res


def time_kv_append(batch, db, workload):
    """nanocp_kv_append (pure data movement) on the workload's shapes: (a) a decode step's append, one token per
    shard entry at its last position; (b) a bulk append of up to 65536 tokens.  Payload rows are random bytes."""
    import torch
    import paper_2605_21100_amd as nanocp
    d = batch.desc
    mla = d.kind == "mla"
    es = db.k_pool.element_size()
    res = {"metric": "nanocp_kv_append", "workload": workload,
           "kv_dtype": d.kv_dtype, "kind": d.kind}
    last_rows = np.array([bt for _, bt, lo, hi in batch.shards if hi > lo], np.int32)
    last_pos = np.array([hi - 1 for _, bt, lo, hi in batch.shards if hi > lo], np.int32)
    rows, pos = [], []
    for _, bt, lo, hi in batch.shards:
        rows.append(np.full(hi - lo, bt, np.int32))
        pos.append(np.arange(lo, hi, dtype=np.int32))
    rows, pos = np.concatenate(rows)[:65536], np.concatenate(pos)[:65536]
    for name, r_, p_ in (("decode_step", last_rows, last_pos), ("bulk", rows, pos)):
        n = len(r_)
        kshape = (n, d.head_dim_qk) if mla else (n, d.num_kv_heads, d.head_dim_qk)
        k_new = torch.empty(kshape, dtype=db.k_pool.dtype, device="cuda")
        k_new.view(torch.uint8).random_(0, 120)
        v_new = None
        if not mla:
            v_new = torch.empty((n, d.num_kv_heads, d.head_dim_v), dtype=db.v_pool.dtype, device="cuda")
            v_new.view(torch.uint8).random_(0, 120)
        rt, pt = torch.from_numpy(r_).cuda(), torch.from_numpy(p_).cuda()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(30)]
        for a, b in evs:
            a.record()
            nanocp.nanocp_kv_append(db.desc, k_new, v_new, rt, pt, db.k_pool, db.v_pool, db.block_table)
            b.record()
        torch.cuda.synchronize()
        us = np.array([a.elapsed_time(b) for a, b in evs])[5:] * 1e3
        nbytes = n * (d.head_dim_qk if mla else d.num_kv_heads * (d.head_dim_qk + d.head_dim_v)) * es
        res[name] = {"tokens": int(n), "bytes": int(nbytes), "us_mean": float(us.mean()), "us_min": float(us.min()),
                     "GBs_written": nbytes / (us.mean() * 1e-6) / 1e9}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--num-long", type=int, default=3, help="config 6 only: long requests per node (1, 3, 5, 7)")
    ap.add_argument("--tile-tokens", type=int, default=0)
    ap.add_argument("--merge-all", action="store_true",
                    help="every output row goes through nanocp_merge_partials (default: requests whose only partial "
                         "is a local shard are written in final form by the attention kernel itself)")
    ap.add_argument("--graph", action="store_true",
                    help="bucket mode: the step is recorded once as a HIP graph over a plan image; every timed step "
                         "re-injects the image (pack + asynchronous copy) and replays the graph")
    ap.add_argument("--image-eager", action="store_true",
                    help="with --graph: do not record a graph, launch the image-driven step eagerly every time")
    ap.add_argument("--inject-once", action="store_true",
                    help="with --graph: inject the plan image once instead of before every step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per_config table (step time and event-timed launch of the other workloads)")
    ap.add_argument("--no-straggle", action="store_true")
    ap.add_argument("--dump-tiles", default="", help="write the tile list and per-tile device clocks to this .npz")
    ap.add_argument("--kv-append", action="store_true",
                    help="time nanocp_kv_append on the workload's shapes instead of the attention step: one token per "
                         "shard entry (what a decode step appends) and a bulk rebuild of 65536 tokens")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of known size (1 GiB read + 1 GiB written per launch); "
                         "used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of a DCP decode step; this build has no multi-GPU path "
              "(--gpus must be 1).", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2605_21100_amd as nanocp
    import workloads as W
    from workloads.device import DeviceBatch

    torch.cuda.set_device(0)
    print("[bench] start", file=sys.stderr, flush=True)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for a, b in evs:
            a.record()
            dst.copy_(src)
            b.record()
        torch.cuda.synchronize()
        ms = np.array([a.elapsed_time(b) for a, b in evs])[2:]
        print(json.dumps({"calibrate_copy_bytes_each_way": 1 << 30, "launches": 20, "ms_mean": float(ms.mean()),
                          "read_plus_write_GBs": 2 * (1 << 30) / (ms.mean() * 1e-3) / 1e9}))
        return
    kw = {"num_long": args.num_long} if args.config == 6 else {}
    batch = W.FULL[args.config](with_remote_kv=False, **kw)
    d = batch.desc
    db = DeviceBatch(batch, tile_tokens=args.tile_tokens, final_rows=not args.merge_all)
    if args.kv_append:
        print(json.dumps(time_kv_append(batch, db, WORKLOAD_NAMES[args.config].format(n=args.num_long))))
        return
    pools = [(db.k_pool, db.v_pool, db.k_scale, db.v_scale)]
    pools.append(tuple(None if t is None else t.clone() for t in pools[0]))
    S, R = batch.num_shards, batch.num_requests
    rem_o, rem_lse = W.synthetic_remote_partials(batch)
    n_rem = rem_o.shape[0]
    # pooled partial list: [local partials (written by the kernel) | remote partials (received)]
    parts_o = torch.empty((S + n_rem, d.num_q_heads, d.head_dim_v), dtype=torch.float32, device="cuda")
    parts_lse = torch.empty((S + n_rem, d.num_q_heads), dtype=torch.float32, device="cuda")
    if n_rem:
        parts_o[S:] = torch.from_numpy(rem_o).cuda()
        parts_lse[S:] = torch.from_numpy(rem_lse).cuda()
    part_offsets = torch.from_numpy(batch.part_offsets).cuda()
    part_index = torch.from_numpy(batch.part_index).cuda()
    out = torch.empty((R, d.num_q_heads, d.head_dim_v), dtype=torch.bfloat16 if d.q_dtype == "bf16" else torch.float32,
                      device="cuda")
    local_o, local_lse = parts_o[:S], parts_lse[:S]
    if not args.merge_all:
        n_rest = len(db.rest_rows)
        rest_offsets, rest_index = torch.from_numpy(db.rest_offsets).cuda(), torch.from_numpy(db.rest_index).cuda()
        rest_rows = torch.from_numpy(db.rest_rows).cuda()

    def step(i, ev=None):
        k, v, ks, vs = pools[i & 1]
        if ev:
            ev[0].record()
        if args.merge_all:
            nanocp.nanocp_decode_attn_partial(db.plan, db.q, k, v, ks, vs, db.block_table, local_o, local_lse,
                                              db.workspace)
        else:
            nanocp.nanocp_decode_attn_partial(db.plan, db.q, k, v, ks, vs, db.block_table, local_o, local_lse,
                                              db.workspace, final_out=out)
        if ev:
            ev[1].record()
        if args.merge_all:
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, part_offsets, part_index, R, out)
        elif n_rest:
            nanocp.nanocp_merge_partials(db.desc, parts_o, parts_lse, rest_offsets, rest_index, n_rest, out,
                                         out_rows=rest_rows)

    graph_info = {}
    if args.graph:
        if args.merge_all:
            print("--graph uses the final-row path; drop --merge-all", file=sys.stderr)
            sys.exit(2)
        nt = db.plan.num_tiles
        bucket = nanocp.Bucket(nt + nt // 4 + 64, db.plan.num_chunks + db.plan.num_chunks // 4 + 64,
                               nt + 64 + d.num_kv_heads * S, nt + 64)
        img_bytes = nanocp.bucket_plan_bytes(bucket)
        # two images: while the step of one parity runs, the image of the other is injected on a copy stream
        host_imgs = [torch.empty(img_bytes, dtype=torch.uint8).pin_memory() for _ in range(2)]
        dev_imgs = [torch.zeros(img_bytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
        host_img = host_imgs[0]
        ws_b = torch.empty(max(nanocp.bucket_workspace_bytes(db.desc, bucket), 16), dtype=torch.uint8, device="cuda")
        m_count = torch.tensor([n_rest], dtype=torch.int32, device="cuda")
        m_offs = torch.zeros(R + 1, dtype=torch.int32, device="cuda")
        m_idx = torch.zeros(max(len(db.rest_index), 1), dtype=torch.int32, device="cuda")
        m_rows = torch.zeros(R, dtype=torch.int32, device="cuda")
        m_offs[: len(db.rest_offsets)] = rest_offsets
        m_idx[: len(db.rest_index)] = rest_index
        m_rows[:n_rest] = rest_rows
        mb = batch.block_table.shape[1]
        # host side of an iteration whose batch composition changed: new plan, final rows, image
        t_h = time.perf_counter()
        reps = 20
        for _ in range(reps):
            pl = nanocp.Plan(db.desc, batch.shards, batch.q.shape[0], batch.block_table.shape[0], mb, args.tile_tokens)
            pl.set_final_rows(db.shard_final_row, R)
            pl.pack(bucket, host_img)
            pl.close()
        graph_info["host_us_plan_create_and_pack"] = (time.perf_counter() - t_h) / reps * 1e6
        t_h = time.perf_counter()
        for _ in range(200):
            db.plan.pack(bucket, host_img)
        graph_info["host_us_pack"] = (time.perf_counter() - t_h) / 200 * 1e6
        graph_info["image_bytes"] = img_bytes

        def gstep(i):
            k, v, ks, vs = pools[i & 1]
            nanocp.nanocp_decode_attn_partial_image(db.desc, bucket, dev_imgs[i & 1], 0, mb, db.q, k, v, ks, vs,
                                                    db.block_table, local_o, local_lse, ws_b, final_out=out)
            nanocp.nanocp_merge_partials_dyn(db.desc, parts_o, parts_lse, m_offs, m_idx, R, m_count, m_rows, out)

        for par in (0, 1):
            db.plan.pack(bucket, host_imgs[par])
            dev_imgs[par].copy_(host_imgs[par], non_blocking=True)
        gstep(0)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        copy_stream = torch.cuda.Stream()
        done_ev = [torch.cuda.Event(), torch.cuda.Event()]
        copied_ev = [torch.cuda.Event(), torch.cuda.Event()]
        for e in done_ev:
            e.record()
        graphs = []
        for par in (0, 1):                       # one graph per KV pool copy (the pools alternate to defeat the cache)
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                gstep(par)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                gstep(par)
            graphs.append(g)
        eager_step = step

        def step(i, ev=None):                    # noqa: F811  (replaces the eager step in the timed loops below)
            par = i & 1
            if not args.inject_once:
                done_ev[par].synchronize()        # the step that last used this image (two steps back) has finished
                db.plan.pack(bucket, host_imgs[par])
                with torch.cuda.stream(copy_stream):
                    dev_imgs[par].copy_(host_imgs[par], non_blocking=True)
                    copied_ev[par].record()
                torch.cuda.current_stream().wait_event(copied_ev[par])
            if ev:
                ev[0].record()
            if args.image_eager:
                gstep(i)
            else:
                graphs[par].replay()
            if ev:
                ev[1].record()
            done_ev[par].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # dominant kernel: the tile kernel inside nanocp_decode_attn_partial, timed with events on the launch stream
    # (torch's current stream is the one handed to the library)
    n_ev = min(args.steps, 100)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for i in range(n_ev):
        step(i, evs[i])
    torch.cuda.synchronize()
    part_ms = np.array([a.elapsed_time(b) for a, b in evs])
    kv_bytes = batch.kv_bytes
    achieved = kv_bytes / (part_ms.mean() * 1e-3) / 1e9

    extra = {}
    if not args.no_straggle:
        # per tile: device clock at start / end and the workgroup that ran it (instrumented entry point)
        # (same work-list; the instrumented entry point writes per-shard partials, so it gets a plan of its own)
        plan_t = nanocp.Plan(db.desc, batch.shards, batch.q.shape[0], batch.block_table.shape[0],
                             batch.block_table.shape[1], args.tile_tokens).upload()
        ws_t = torch.empty(max(plan_t.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
        clk = torch.zeros((max(plan_t.num_tiles, 1), 3), dtype=torch.int64, device="cuda")
        for rep in range(3):
            nanocp.nanocp_decode_attn_partial(plan_t, db.q, *[pools[rep & 1][j] for j in range(4)], db.block_table,
                                              local_o, local_lse, ws_t, tile_clock=clk)
        torch.cuda.synchronize()
        c = clk.cpu().numpy().astype(np.int64)
        tiles = plan_t.tiles()
        if args.dump_tiles:
            np.savez(args.dump_tiles, tiles=tiles, clock=c)
        t0 = c[:, 0].min()
        wg = c[:, 2]
        n_wg = int(wg.max()) + 1
        finish = np.zeros(n_wg)
        np.maximum.at(finish, wg, (c[:, 1] - t0) / 100.0)            # 100 MHz clock -> microseconds
        # the first n_wg chunks of the queue are the big, statically sized ones (equal cost up to the planner's
        # boundary snapping, +-12 %): their run times, raw and per token, are the "tile times" whose spread says
        # how much one piece of the work-list can straggle
        nch = plan_t.num_chunks
        c_start = np.full(nch, np.iinfo(np.int64).max)
        c_end = np.zeros(nch, np.int64)
        np.minimum.at(c_start, tiles["chunk"], c[:, 0])
        np.maximum.at(c_end, tiles["chunk"], c[:, 1])
        head = ((c_end - c_start) / 100.0)[:min(n_wg, nch)]
        c_tok = np.zeros(nch)
        np.add.at(c_tok, tiles["chunk"], tiles["tok_end"] - tiles["tok_begin"])
        rate = head / np.maximum(c_tok[:len(head)], 1)               # microseconds per token of the chunk
        # per tile: run time per token over the full-size tiles (at least half the largest tile's tokens); cuts snap
        # to boundaries, so tile sizes differ by design and only the per-token time is comparable between them
        t_tok = (tiles["tok_end"] - tiles["tok_begin"]).astype(np.float64)
        t_us = (c[:, 1] - c[:, 0]) / 100.0
        big = t_tok >= 0.5 * t_tok.max()
        t_rate = t_us[big] / t_tok[big]
        extra = {"chunks": int(nch), "tiles": int(db.plan.num_tiles), "workgroups": n_wg,
                 "wg_finish_us_mean": float(finish.mean()), "wg_finish_us_max": float(finish.max()),
                 "straggle_wg_finish_max_over_mean": float(finish.max() / finish.mean()),
                 "equal_chunk_us_mean": float(head.mean()), "equal_chunk_us_max": float(head.max()),
                 "straggle_equal_chunk_max_over_mean": float(head.max() / head.mean()),
                 "straggle_equal_chunk_per_token_max_over_mean": float(rate.max() / rate.mean()),
                 "full_size_tiles": int(big.sum()),
                 "straggle_full_size_tile_per_token_max_over_mean": float(t_rate.max() / t_rate.mean())}

    default_plan = (args.tile_tokens == 0 and not args.merge_all and not args.graph and args.num_long == 3 and
                    not any(k.startswith("NANOCP_") for k in os.environ))
    traffic, traffic_src = (MEASURED_TRAFFIC_BYTES.get(args.config, (None, None)) if default_plan else (None, None))
    result = {
        "metric": METRIC, "value": kv_bytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16", "fp8": "fp8_e4m3"}[d.kv_dtype], "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.config].format(n=args.num_long), "seed": int(batch.seed), "shard_entries": S,
                   "requests": R, "local_kv_tokens": batch.local_tokens, "kv_bytes": kv_bytes,
                   "remote_partials": int(n_rem), "kernel": db.plan.kernel,
                   "rows_final_from_kernel": 0 if args.merge_all else int(len(set(db.shard_final_row[db.shard_final_row >= 0].tolist()))),
                   "rows_merged": int(R) if args.merge_all else int(n_rest),
                   "mode": "graph replay over a plan image, re-injected every step" if args.graph else "eager launches",
                   **graph_info, "us_per_step": ms_per_step * 1e3,
                   "pct_of_hbm_peak": 100.0 * kv_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, **extra},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": db.plan.kernel, "launch_us_mean": float(part_ms.mean() * 1e3),
                     "launch_us_min": float(part_ms.min() * 1e3), "traffic_source": traffic_src,
                     "note": "events on the launch stream bracket nanocp_decode_attn_partial, which is one kernel "
                             "for the MFMA variants (tile kernel with fused tile reduction)"},
    }
    if d.kind == "mla":
        # MLA is co-limited: 2*(Dk+Dv)*Hq flop per token against Dk*2 bytes; the HBM term is the larger one at the
        # published peaks, the matrix-core fraction is reported beside it (useful flops: the second bf16 term of P
        # that the kernel also multiplies is not counted)
        flops = 2.0 * (d.head_dim_qk + d.head_dim_v) * d.num_q_heads * batch.local_tokens
        tf = flops / (part_ms.mean() * 1e-3) / 1e12
        result["roofline"]["mfma"] = {"bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s",
                                      "frac": tf / 2500.0}
        result["roofline"]["note"] = ("events on the launch stream bracket nanocp_decode_attn_partial = the tile "
                                      "kernel plus the tile-reduction kernel")
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(batch)
    if not args.no_per_config and args.config == 3 and default_plan:
        # the other workloads at the same --steps / --warmup, each in its default launch configuration
        del db, pools, parts_o, parts_lse, out, local_o, local_lse
        torch.cuda.empty_cache()
        result["per_config"] = {}
        for cid in (2, 4, 5, 6, 7):
            result["per_config"][str(cid)] = quick_config(cid, args.steps, args.warmup)
            print(f"[bench] config {cid}: {result['per_config'][str(cid)]['us_per_step']:.1f} us/step", file=sys.stderr,
                  flush=True)
    print(json.dumps(result))


if __name__ == "__main__":
    main()

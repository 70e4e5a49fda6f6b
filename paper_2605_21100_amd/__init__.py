"""Thin ctypes binding of libnanocp.so (the C ABI in include/nanocp.h).

Argument marshalling only: every step of the decode path runs in the HIP kernels of the
library.  torch tensors are used as device memory; their data pointers are handed to the
C functions together with the current torch stream.  If the library has not been built
the import fails loudly -- there is no fallback path.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnanocp.so")

OK, EINVAL, ESHAPE, EBOUNDS, EUNSUPPORTED, ENOMEM, EHIP, ESTATE = range(8)
F32, BF16, FP8_E4M3 = 0, 1, 2
GQA, MLA = 0, 1
_DTYPES = {"f32": F32, "bf16": BF16, "fp8": FP8_E4M3}
_KINDS = {"gqa": GQA, "mla": MLA}


class AttnDesc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("q_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim_qk", ctypes.c_int32), ("head_dim_v", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("out_scale", ctypes.c_float)]


class Shard(ctypes.Structure):
    _fields_ = [("q_row", ctypes.c_int32), ("bt_row", ctypes.c_int32),
                ("kv_begin", ctypes.c_int32), ("kv_end", ctypes.c_int32)]


class Tile(ctypes.Structure):
    _fields_ = [("shard", ctypes.c_int32), ("kv_head", ctypes.c_int32), ("q_row", ctypes.c_int32),
                ("bt_row", ctypes.c_int32), ("tok_begin", ctypes.c_int32), ("tok_end", ctypes.c_int32),
                ("dst", ctypes.c_int32), ("chunk", ctypes.c_int32)]


TILE_DTYPE = np.dtype([(n, np.int32) for n, _ in Tile._fields_])

EXPORTS = ["nanocp_plan_create", "nanocp_plan_query", "nanocp_plan_tiles", "nanocp_plan_kernel",
           "nanocp_plan_upload", "nanocp_plan_destroy", "nanocp_decode_attn_partial",
           "nanocp_merge_partials", "nanocp_status_str",
           "nanocp_plan_set_final_rows", "nanocp_decode_attn_partial_final", "nanocp_merge_partials_rows",
           "nanocp_bucket_plan_bytes", "nanocp_bucket_workspace_bytes", "nanocp_plan_pack",
           "nanocp_decode_attn_partial_image", "nanocp_merge_partials_dyn", "nanocp_kv_append",
           "nanocp_decode_attn_partial_image_static"]
DEBUG_EXPORTS = ["nanocp_decode_attn_partial_timed"]          # include/nanocp_debug.h
STATIC_SCRATCH_BYTES = 32 << 20


class Bucket(ctypes.Structure):
    """Capacities of a bucket of batch compositions (see include/nanocp.h)."""
    _fields_ = [("max_tiles", ctypes.c_int32), ("max_chunks", ctypes.c_int32), ("max_segs", ctypes.c_int32),
                ("max_slots", ctypes.c_int32)]



def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2605_21100_amd/build.py)")
    import torch  # noqa: F401  -- first, so that the library binds to the HIP runtime torch has loaded (two
    #                               runtimes in one process do not share devices, streams or memory)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.nanocp_plan_create.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(Shard), i32, i32, i32, i32, i32, i32,
                                       ctypes.POINTER(vp)]
    lib.nanocp_plan_query.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(sz)]
    lib.nanocp_plan_tiles.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(i32)]
    lib.nanocp_plan_kernel.argtypes = [vp]
    lib.nanocp_plan_kernel.restype = ctypes.c_char_p
    lib.nanocp_plan_upload.argtypes = [vp, vp]
    lib.nanocp_plan_destroy.argtypes = [vp]
    lib.nanocp_plan_destroy.restype = None
    lib.nanocp_decode_attn_partial.argtypes = [vp] * 9 + [vp, sz, vp]
    lib.nanocp_decode_attn_partial_timed.argtypes = [vp] * 9 + [vp, sz, vp, vp]
    lib.nanocp_merge_partials.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, i32, vp, i32, vp, vp]
    lib.nanocp_plan_set_final_rows.argtypes = [vp, vp, i32]
    lib.nanocp_decode_attn_partial_final.argtypes = [vp] * 9 + [vp, sz, vp, i32, vp, vp]
    lib.nanocp_merge_partials_rows.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, i32, vp, vp, i32, vp, vp]
    lib.nanocp_bucket_plan_bytes.argtypes = [ctypes.POINTER(Bucket)]
    lib.nanocp_bucket_plan_bytes.restype = sz
    lib.nanocp_bucket_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(Bucket)]
    lib.nanocp_bucket_workspace_bytes.restype = sz
    lib.nanocp_plan_pack.argtypes = [vp, ctypes.POINTER(Bucket), vp, sz]
    lib.nanocp_decode_attn_partial_image.argtypes = ([ctypes.POINTER(AttnDesc), ctypes.POINTER(Bucket), vp, i32, i32] +
                                                     [vp] * 8 + [vp, sz, vp, i32, vp, vp])
    lib.nanocp_decode_attn_partial_image_static.argtypes = ([ctypes.POINTER(AttnDesc), ctypes.POINTER(Bucket), vp, i32,
                                                             i32] + [vp] * 8 + [vp, i32, vp, vp])
    lib.nanocp_merge_partials_dyn.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, i32, vp, vp, vp, i32, vp, vp]
    lib.nanocp_kv_append.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, i32, vp, vp, vp, i32, vp]
    lib.nanocp_status_str.argtypes = [ctypes.c_int]
    lib.nanocp_status_str.restype = ctypes.c_char_p
    return lib


_lib = _load()


class NanocpError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {_lib.nanocp_status_str(self.status).decode()} ({self.status})")


def _check(status, where):
    if status != OK:
        raise NanocpError(status, where)


def make_desc(kind, q_dtype, kv_dtype, num_q_heads, num_kv_heads, head_dim_qk, head_dim_v, page_size,
              softmax_scale, out_scale=0.0):
    return AttnDesc(_KINDS.get(kind, kind), _DTYPES.get(q_dtype, q_dtype), _DTYPES.get(kv_dtype, kv_dtype),
                    num_q_heads, num_kv_heads, head_dim_qk, head_dim_v, page_size, softmax_scale, out_scale)


def _out_dtype(t, where):
    """nanocp_dtype of an output tensor: float32, bfloat16, or one byte per element (uint8 / float8_e4m3fn) for fp8."""
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.uint8 or t.dtype == getattr(torch, "float8_e4m3fn", None):
        return FP8_E4M3
    raise NanocpError(EUNSUPPORTED, where)


def _ptr(t):
    """Device (or None) pointer of a torch tensor."""
    if t is None:
        return None
    assert t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(stream)
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Plan:
    """nanocp_plan: the tile work-list of one batch composition (host object + device copy)."""

    def __init__(self, desc, shards, num_q_rows, num_bt_rows, max_blocks_per_row, tile_tokens=0, num_cus=0):
        self.desc = desc
        shards = np.ascontiguousarray(shards, dtype=np.int32).reshape(-1, 4)
        self.num_shards = shards.shape[0]
        self._h = ctypes.c_void_p()
        sp = shards.ctypes.data_as(ctypes.POINTER(Shard)) if self.num_shards else None
        _check(_lib.nanocp_plan_create(ctypes.byref(desc), sp, self.num_shards, num_q_rows, num_bt_rows,
                                       max_blocks_per_row, tile_tokens, num_cus, ctypes.byref(self._h)),
               "nanocp_plan_create")
        self._query()
        self.uploaded = False

    def _query(self):
        nt, nc, ws = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_size_t()
        _check(_lib.nanocp_plan_query(self._h, ctypes.byref(nt), ctypes.byref(nc), ctypes.byref(ws)),
               "nanocp_plan_query")
        self.num_tiles, self.num_chunks, self.workspace_bytes = nt.value, nc.value, ws.value

    @property
    def kernel(self):
        return _lib.nanocp_plan_kernel(self._h).decode()

    def tiles(self):
        """Host copy of the tile list as a numpy structured array."""
        p, n = ctypes.c_void_p(), ctypes.c_int32()
        _check(_lib.nanocp_plan_tiles(self._h, ctypes.byref(p), ctypes.byref(n)), "nanocp_plan_tiles")
        if n.value == 0:
            return np.zeros(0, TILE_DTYPE)
        buf = (ctypes.c_char * (n.value * ctypes.sizeof(Tile))).from_address(p.value)
        return np.frombuffer(buf, dtype=TILE_DTYPE).copy()

    def set_final_rows(self, shard_final_row, num_out):
        """shard_final_row[s] = r >= 0: shard s is the only partial of output row r (before upload)."""
        rows = np.ascontiguousarray(shard_final_row, dtype=np.int32)
        assert rows.shape == (self.num_shards,)
        _check(_lib.nanocp_plan_set_final_rows(self._h, rows.ctypes.data, int(num_out)), "nanocp_plan_set_final_rows")
        self._query()       # the partial slots (workspace size) were re-derived
        return self

    def pack(self, bucket, host_image):
        """Serialise into host_image (a pinned uint8 torch tensor or numpy array of bucket_plan_bytes(bucket))."""
        ptr = host_image.data_ptr() if hasattr(host_image, "data_ptr") else host_image.ctypes.data
        nbytes = host_image.numel() if hasattr(host_image, "numel") else host_image.nbytes
        _check(_lib.nanocp_plan_pack(self._h, ctypes.byref(bucket), ctypes.c_void_p(ptr), nbytes), "nanocp_plan_pack")

    def upload(self, stream=None):
        _check(_lib.nanocp_plan_upload(self._h, _stream(stream)), "nanocp_plan_upload")
        self.uploaded = True
        return self

    def close(self):
        if self._h:
            _lib.nanocp_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def nanocp_plan(desc, shards, num_q_rows, num_bt_rows, max_blocks_per_row, tile_tokens=0, num_cus=0):
    return Plan(desc, shards, num_q_rows, num_bt_rows, max_blocks_per_row, tile_tokens, num_cus)


def nanocp_decode_attn_partial(plan, q, k_pool, v_pool, k_scale, v_scale, block_table, out_o, out_lse,
                               workspace, tile_clock=None, stream=None, final_out=None, final_lse=None):
    """Phase 2 on the given torch device tensors; results land in out_o / out_lse (float32).  With final_out
    (float32, bfloat16 or fp8 bytes, [num_out, Hq, Dv]) shards that are a whole output row write it directly."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    args = [plan._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale), _ptr(v_scale), _ptr(block_table),
            _ptr(out_o), _ptr(out_lse), _ptr(workspace), ws_bytes]
    if final_out is not None:
        assert tile_clock is None
        _check(_lib.nanocp_decode_attn_partial_final(*args, _ptr(final_out),
                                                     _out_dtype(final_out, "nanocp_decode_attn_partial_final"),
                                                     _ptr(final_lse), _stream(stream)),
               "nanocp_decode_attn_partial_final")
    elif tile_clock is None:
        _check(_lib.nanocp_decode_attn_partial(*args, _stream(stream)), "nanocp_decode_attn_partial")
    else:
        _check(_lib.nanocp_decode_attn_partial_timed(*args, _ptr(tile_clock), _stream(stream)),
               "nanocp_decode_attn_partial_timed")


def nanocp_merge_partials(desc, o_parts, lse_parts, part_offsets, part_index, num_out, out, out_lse=None,
                          stream=None, out_rows=None):
    """Phase 4 on device tensors; out is float32, bfloat16 or fp8 bytes [rows, Hq, Dv].  With out_rows (int32
    [num_out]) list i of the CSR produces row out_rows[i] instead of row i."""
    out_dtype = _out_dtype(out, "nanocp_merge_partials")
    if out_rows is None:
        _check(_lib.nanocp_merge_partials(ctypes.byref(desc), _ptr(o_parts), _ptr(lse_parts), _ptr(part_offsets),
                                          _ptr(part_index), num_out, _ptr(out), out_dtype, _ptr(out_lse),
                                          _stream(stream)), "nanocp_merge_partials")
    else:
        _check(_lib.nanocp_merge_partials_rows(ctypes.byref(desc), _ptr(o_parts), _ptr(lse_parts), _ptr(part_offsets),
                                               _ptr(part_index), num_out, _ptr(out_rows), _ptr(out), out_dtype,
                                               _ptr(out_lse), _stream(stream)), "nanocp_merge_partials_rows")


def bucket_plan_bytes(bucket):
    return int(_lib.nanocp_bucket_plan_bytes(ctypes.byref(bucket)))


def bucket_workspace_bytes(desc, bucket):
    return int(_lib.nanocp_bucket_workspace_bytes(ctypes.byref(desc), ctypes.byref(bucket)))


def nanocp_decode_attn_partial_image(desc, bucket, image, num_cus, max_blocks_per_row, q, k_pool, v_pool, k_scale,
                                     v_scale, block_table, out_o, out_lse, workspace, final_out=None, final_lse=None,
                                     stream=None):
    """Phase 2 driven by a plan image on the device (same call for every plan of the bucket: graph-capturable)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fdt = F32 if final_out is None else _out_dtype(final_out, "nanocp_decode_attn_partial_image")
    _check(_lib.nanocp_decode_attn_partial_image(ctypes.byref(desc), ctypes.byref(bucket), _ptr(image), num_cus,
                                                 max_blocks_per_row, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale),
                                                 _ptr(v_scale), _ptr(block_table), _ptr(out_o), _ptr(out_lse),
                                                 _ptr(workspace), ws_bytes, _ptr(final_out), fdt, _ptr(final_lse),
                                                 _stream(stream)), "nanocp_decode_attn_partial_image")


def nanocp_decode_attn_partial_image_static(desc, bucket, image, num_cus, max_blocks_per_row, q, k_pool, v_pool,
                                            k_scale, v_scale, block_table, out_o, out_lse, final_out=None,
                                            final_lse=None, stream=None):
    """nanocp_decode_attn_partial_image with the tile partials in the library's own static scratch (no workspace
    argument, no allocation, no device query: num_cus must be given)."""
    fdt = F32 if final_out is None else _out_dtype(final_out, "nanocp_decode_attn_partial_image_static")
    _check(_lib.nanocp_decode_attn_partial_image_static(ctypes.byref(desc), ctypes.byref(bucket), _ptr(image), num_cus,
                                                        max_blocks_per_row, _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                        _ptr(k_scale), _ptr(v_scale), _ptr(block_table), _ptr(out_o),
                                                        _ptr(out_lse), _ptr(final_out), fdt, _ptr(final_lse),
                                                        _stream(stream)), "nanocp_decode_attn_partial_image_static")


def nanocp_merge_partials_dyn(desc, o_parts, lse_parts, part_offsets, part_index, max_out, num_out_dev, out_rows, out,
                              out_lse=None, stream=None):
    """Row-indexed merge over at most max_out lists; the count is read from num_out_dev (int32 [1]) on the device."""
    out_dtype = _out_dtype(out, "nanocp_merge_partials_dyn")
    _check(_lib.nanocp_merge_partials_dyn(ctypes.byref(desc), _ptr(o_parts), _ptr(lse_parts), _ptr(part_offsets),
                                          _ptr(part_index), max_out, _ptr(num_out_dev), _ptr(out_rows), _ptr(out),
                                          out_dtype, _ptr(out_lse), _stream(stream)), "nanocp_merge_partials_dyn")


def split_final_rows(part_offsets, part_index, num_local, single_only=False):
    """Host helper.  From the pooled partial lists ([local shards | received partials], CSR per output row):
    shard_final_row [num_local] (row r for the local shards of a row all of whose partials are local -- with
    single_only, only rows with exactly one partial -- else -1) and the CSR (offsets, index, rows) of the
    remaining rows, which still need nanocp_merge_partials."""
    part_offsets = np.asarray(part_offsets, np.int64)
    part_index = np.asarray(part_index, np.int64)
    final = np.full(num_local, -1, np.int32)
    offs, idx, rows = [0], [], []
    for r in range(len(part_offsets) - 1):
        parts = part_index[part_offsets[r]:part_offsets[r + 1]]
        if len(parts) >= 1 and (parts < num_local).all() and (len(parts) == 1 or not single_only):
            final[parts] = r
        else:
            idx.extend(parts.tolist())
            offs.append(len(idx))
            rows.append(r)
    return final, np.asarray(offs, np.int32), np.asarray(idx, np.int32), np.asarray(rows, np.int32)


def nanocp_kv_append(desc, k_new, v_new, bt_row, position, k_pool, v_pool, block_table, stream=None):
    """Store n tokens' K / V rows at (block-table row, position) into the paged pools (the layouts' writer)."""
    _check(_lib.nanocp_kv_append(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _ptr(bt_row), _ptr(position),
                                 int(bt_row.numel()), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                 int(block_table.shape[1]), _stream(stream)), "nanocp_kv_append")


# --------------------------------------------------------------------------- host scheduler (include/nanocp_sched.h)

SCHED_MAX_CP = 8
SCHED_EXPORTS = ["nanocp_sched_water_fill", "nanocp_sched_rebalance", "nanocp_sched_place"]


class SchedConfig(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int32), ("node_offsets", ctypes.POINTER(ctypes.c_int32)),
                ("kv_capacity", ctypes.c_int64), ("num_buckets", ctypes.c_int32),
                ("bucket_max_len", ctypes.POINTER(ctypes.c_int64)), ("bucket_degree", ctypes.POINTER(ctypes.c_int32))]


class SchedDecision(ctypes.Structure):
    _fields_ = [("scheduled", ctypes.c_int32), ("node", ctypes.c_int32), ("moe_instance", ctypes.c_int32),
                ("num_participants", ctypes.c_int32), ("participants", ctypes.c_int32 * SCHED_MAX_CP),
                ("split", ctypes.c_int64 * SCHED_MAX_CP)]


_lib.nanocp_sched_water_fill.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
_lib.nanocp_sched_rebalance.argtypes = [ctypes.POINTER(SchedConfig), ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p]
_lib.nanocp_sched_place.argtypes = [ctypes.POINTER(SchedConfig), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                    ctypes.c_void_p, ctypes.POINTER(SchedDecision)]


class Scheduler:
    """Dual-balanced scheduler state for a cluster: nodes[n] = number of instances of node n."""

    def __init__(self, instances_per_node, kv_capacity, bucket_max_len, bucket_degree):
        self._offsets = np.concatenate([[0], np.cumsum(instances_per_node)]).astype(np.int32)
        self._blen = np.ascontiguousarray(bucket_max_len, dtype=np.int64)
        self._bdeg = np.ascontiguousarray(bucket_degree, dtype=np.int32)
        self.num_instances = int(self._offsets[-1])
        self.cfg = SchedConfig(len(instances_per_node), self._offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                               int(kv_capacity), len(self._blen),
                               self._blen.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                               self._bdeg.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
        self.kv_load = np.zeros(self.num_instances, np.int64)
        self.moe_load = np.zeros(self.num_instances, np.int32)

    def rebalance(self, participants):
        """participants: list of lists of instance ids (P_r of the active requests).  Returns m_r per request."""
        offs = np.concatenate([[0], np.cumsum([len(p) for p in participants])]).astype(np.int32)
        inst = np.asarray([s for p in participants for s in p], np.int32)
        m = np.zeros(len(participants), np.int32)
        _check(_lib.nanocp_sched_rebalance(ctypes.byref(self.cfg), len(participants), offs.ctypes.data,
                                           inst.ctypes.data if len(inst) else None, m.ctypes.data,
                                           self.moe_load.ctypes.data), "nanocp_sched_rebalance")
        return m

    def place(self, lengths):
        lengths = np.ascontiguousarray(lengths, dtype=np.int64)
        out = (SchedDecision * max(len(lengths), 1))()
        _check(_lib.nanocp_sched_place(ctypes.byref(self.cfg), self.kv_load.ctypes.data, self.moe_load.ctypes.data,
                                       len(lengths), lengths.ctypes.data, out), "nanocp_sched_place")
        res = []
        for i in range(len(lengths)):
            d = out[i]
            k = d.num_participants
            res.append({"scheduled": bool(d.scheduled), "node": d.node, "m": d.moe_instance,
                        "P": list(d.participants[:k]), "split": list(d.split[:k])})
        return res


def nanocp_sched_water_fill(loads, length):
    loads = np.ascontiguousarray(loads, dtype=np.int64)
    split = np.zeros(len(loads), np.int64)
    _check(_lib.nanocp_sched_water_fill(len(loads), loads.ctypes.data, int(length), split.ctypes.data),
           "nanocp_sched_water_fill")
    return split.tolist()

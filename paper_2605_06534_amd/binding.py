"""Thin ctypes binding of librose_delta.so (declared in include/rose_delta.h).

Argument marshalling only: every step of the path (diff, compaction, shard routing, apply)
runs in the library's HIP kernels.  torch tensors are used as device memory; this module reads
their ``data_ptr()`` and the current HIP stream, nothing else.  There is no fallback: if the
library has not been built, importing this module fails.
"""
import ctypes
import os

import torch

ROSE_MAX_TP = 16
ROSE_MAX_SECTIONS = 4
REPLICATED, SPLIT_ROWS, SPLIT_COLS, FUSED_ROWS = 0, 1, 2, 3
BF16, FP32_RNE = 0, 1
OK, ERR_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_ALIGN, ERR_HIP, ERR_UNSUPPORTED, ERR_SCRATCH = range(8)
LAYER_FIRST, LAYER_LAST = -1, -2
TILE_ORDER_AUTO, TILE_ORDER_SPREAD, TILE_ORDER_NEIGHBOURS, TILE_ORDER_TIMED = 0, 1, 2, 3
STATIC_SCRATCH_BYTES = 48 << 20

_LIB_PATH = os.environ.get("ROSE_DELTA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                            "librose_delta.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError("%s is not built: run `python -m paper_2605_06534_amd.build` "
                      "(there is no CPU fallback)" % _LIB_PATH)


class TensorDesc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("rule", ctypes.c_int32),
                ("n_sections", ctypes.c_int32), ("section_rows", ctypes.c_int64 * ROSE_MAX_SECTIONS),
                ("src_groups", ctypes.c_int32), ("layer", ctypes.c_int32)]


class CBucket(ctypes.Structure):
    _fields_ = [("idx", ctypes.c_void_p), ("val", ctypes.c_void_p), ("capacity", ctypes.c_int64),
                ("seg_off", ctypes.c_void_p)]


_vp, _i32, _i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
_P = ctypes.POINTER
_SIGS = {
    "rose_shard_plan_create": (_i32, [_P(TensorDesc), _i32, _i32, _P(_vp)]),
    "rose_shard_plan_create_src": (_i32, [_P(TensorDesc), _i32, _i32, _i32, _i32, _P(_vp)]),
    "rose_shard_plan_create_pp": (_i32, [_P(TensorDesc), _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _P(_vp)]),
    "rose_shard_plan_destroy": (None, [_vp]),
    "rose_plan_upload": (_i32, [_vp]),
    "rose_plan_set_worker_cap": (_i32, [_vp, _i32]),
    "rose_plan_set_tile_order": (_i32, [_vp, _i32]),
    "rose_plan_n_tensors": (_i32, [_vp]),
    "rose_plan_tp": (_i32, [_vp]),
    "rose_plan_n_buckets": (_i32, [_vp]),
    "rose_plan_pick_tile_order": (_i32, [_vp, _vp, _P(_i32)]),
    "rose_plan_stage_of": (_i32, [_vp, _i32, _P(_i32), _P(_i32)]),
    "rose_plan_tensor_is_read": (_i32, [_vp, _i32, ctypes.c_uint32, _P(_i32)]),
    "rose_plan_tensor_base": (_i32, [_vp, _i32, _P(_i64)]),
    "rose_plan_local_numel": (_i32, [_vp, _i32, _i32, _P(_i64)]),
    "rose_plan_src_numel": (_i32, [_vp, _i32, _P(_i64)]),
    "rose_plan_map_index": (_i32, [_vp, _i32, _i64, _P(_i32), _P(_i32), _P(_i32)]),
    "rose_plan_bucket_capacity": (_i32, [_vp, _i32, _P(_i64)]),
    "rose_plan_workspace_bytes": (_i32, [_vp, _P(ctypes.c_size_t)]),
    "rose_plan_n_tiles": (_i32, [_vp, _P(_i64)]),
    "rose_delta_encode": (_i32, [_vp, _vp, _vp, _i32, _P(CBucket), _vp, ctypes.c_size_t, _vp]),
    "rose_delta_encode_refresh": (_i32, [_vp, _vp, _vp, _i32, _P(CBucket), _vp, ctypes.c_size_t, _vp]),
    "rose_delta_encode_ex": (_i32, [_vp, _vp, _vp, _i32, ctypes.c_uint32, _P(CBucket), _vp, ctypes.c_size_t, _vp]),
    "rose_delta_encode_static": (_i32, [_vp, _vp, _vp, _i32, ctypes.c_uint32, _P(CBucket), _vp]),
    "rose_delta_apply": (_i32, [_vp, _i32, _P(CBucket), _vp, _vp]),
    "rose_delta_apply_ex": (_i32, [_vp, _i32, _P(CBucket), _i32, _vp, _vp]),
    "rose_dense_copy": (_i32, [_vp, _i32, _vp, _i32, _vp, _vp]),
    "rose_bucket_check": (_i32, [_vp, _P(CBucket), _vp, _P(_i64)]),
    "rose_object_bytes": (_i32, [_vp, _i64, _P(ctypes.c_size_t)]),
    "rose_bucket_pack": (_i32, [_vp, _i32, _P(CBucket), _i64, _i64, _vp, ctypes.c_size_t, _vp]),
    "rose_bucket_pack_ex": (_i32, [_vp, _i32, _P(CBucket), _i32, _i64, _i64, _vp, ctypes.c_size_t, _vp]),
    "rose_object_apply": (_i32, [_vp, _vp, ctypes.c_size_t, _vp, _vp]),
    "rose_object_check": (_i32, [_vp, _vp, ctypes.c_size_t, _vp, _P(_i32), _P(_i64), _P(_i64), _P(_i32)]),
    "rose_bw_probe": (_i32, [_vp, _vp, ctypes.c_size_t, _vp, _vp]),
    "rose_bw_probe_mixed": (_i32, [_vp, _vp, _vp, ctypes.c_size_t, ctypes.c_size_t, _vp, _vp]),
    "rose_bw_probe_mixed_timed": (_i32, [_vp, _vp, _vp, ctypes.c_size_t, ctypes.c_size_t, _vp, _vp]),
    "rose_bw_probe_lines": (_i32, [_vp, ctypes.c_size_t, ctypes.c_uint32, _vp]),
    "rose_status_str": (ctypes.c_char_p, [_i32]),
}


def _bind(path):
    lib = ctypes.CDLL(path)
    for name, (res, args) in _SIGS.items():
        f = getattr(lib, name)
        f.restype, f.argtypes = res, args
    return lib


_lib = _bind(_LIB_PATH)

EXPORTS = tuple(_SIGS)


class RoseError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s" % (what, _lib.rose_status_str(status).decode()))


def _check(status, what):
    if status != OK:
        raise RoseError(status, what)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class Plan:
    """Handle of a shard plan (rose_shard_plan_create)."""

    def __init__(self, handle, tensors):
        self._h = handle
        self.tensors = tensors

    def __del__(self):
        # at interpreter shutdown the module's globals may be gone already: then the process's end frees the plan
        h, lib = getattr(self, "_h", None), globals().get("_lib")
        if h and lib is not None:
            lib.rose_shard_plan_destroy(h)
            self._h = None

    @property
    def n_tensors(self):
        return _lib.rose_plan_n_tensors(self._h)

    @property
    def tp(self):
        return _lib.rose_plan_tp(self._h)

    @property
    def n_buckets(self):
        return _lib.rose_plan_n_buckets(self._h)

    def upload(self):
        _check(_lib.rose_plan_upload(self._h), "plan_upload")

    def set_worker_cap(self, workers):
        _check(_lib.rose_plan_set_worker_cap(self._h, workers), "plan_set_worker_cap")

    def set_tile_order(self, order):
        _check(_lib.rose_plan_set_tile_order(self._h, order), "plan_set_tile_order")

    def pick_tile_order(self, capacities):
        """The tile order a launch into buckets of these capacities would use now (host only)."""
        cb = (CBucket * self.n_buckets)(*[CBucket(None, None, int(c), None) for c in capacities])
        v = _i32()
        _check(_lib.rose_plan_pick_tile_order(self._h, cb, ctypes.byref(v)), "plan_pick_tile_order")
        return v.value

    def stage_of(self, t):
        a, b = _i32(), _i32()
        _check(_lib.rose_plan_stage_of(self._h, t, ctypes.byref(a), ctypes.byref(b)), "plan_stage_of")
        return a.value, b.value

    def tensor_is_read(self, t, flags=0):
        v = _i32()
        _check(_lib.rose_plan_tensor_is_read(self._h, t, flags, ctypes.byref(v)), "plan_tensor_is_read")
        return bool(v.value)

    def tensor_base(self, t):
        v = _i64()
        _check(_lib.rose_plan_tensor_base(self._h, t, ctypes.byref(v)), "plan_tensor_base")
        return v.value

    def src_numel(self, t):
        v = _i64()
        _check(_lib.rose_plan_src_numel(self._h, t, ctypes.byref(v)), "plan_src_numel")
        return v.value

    def local_numel(self, t, d):
        v = _i64()
        _check(_lib.rose_plan_local_numel(self._h, t, d, ctypes.byref(v)), "plan_local_numel")
        return v.value

    def map_index(self, t, g):
        a, b, c = _i32(), _i32(), _i32()
        _check(_lib.rose_plan_map_index(self._h, t, g, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
               "plan_map_index")
        return a.value, b.value, c.value

    def bucket_capacity(self, d):
        v = _i64()
        _check(_lib.rose_plan_bucket_capacity(self._h, d, ctypes.byref(v)), "plan_bucket_capacity")
        return v.value

    def workspace_bytes(self):
        v = ctypes.c_size_t()
        _check(_lib.rose_plan_workspace_bytes(self._h, ctypes.byref(v)), "plan_workspace_bytes")
        return v.value

    def n_tiles(self):
        v = _i64()
        _check(_lib.rose_plan_n_tiles(self._h, ctypes.byref(v)), "plan_n_tiles")
        return v.value


def shard_plan(tensors, tp, tp_src=1, src_rank=0, n_layers=0, pp_src=1, stage_src=0, pp_dst=1):
    """tensors: list of dicts with rows, cols, rule and (fused rows) sections.  With tp_src > 1 the
    plan is for the sender that holds shard src_rank of tp_src of every tensor; with pp_src / pp_dst
    > 1 (each tensor then names its "layer") for the sender in stage stage_src of pp_src feeding
    pp_dst stages of tp shards."""
    arr = (TensorDesc * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i].rows, arr[i].cols, arr[i].rule = t["rows"], t["cols"], t["rule"]
        sec = t.get("sections") or []
        if len(sec) > ROSE_MAX_SECTIONS:
            raise RoseError(ERR_ARG, "shard_plan")
        arr[i].n_sections = len(sec)
        for j, s in enumerate(sec):
            arr[i].section_rows[j] = s
        arr[i].src_groups = int(t.get("src_groups") or 0)
        arr[i].layer = int(t.get("layer") or 0)
    h = _vp()
    if pp_src != 1 or pp_dst != 1 or stage_src != 0 or n_layers != 0:
        _check(_lib.rose_shard_plan_create_pp(arr, len(tensors), tp, tp_src, src_rank, n_layers, pp_src, stage_src,
                                              pp_dst, ctypes.byref(h)), "shard_plan")
    elif tp_src == 1 and src_rank == 0:
        _check(_lib.rose_shard_plan_create(arr, len(tensors), tp, ctypes.byref(h)), "shard_plan")
    else:
        _check(_lib.rose_shard_plan_create_src(arr, len(tensors), tp, tp_src, src_rank, ctypes.byref(h)), "shard_plan")
    return Plan(h, list(tensors))


class Bucket:
    """Device arrays of one destination shard's COO data (caller-owned torch tensors)."""

    def __init__(self, capacity, n_tensors, device="cuda"):
        self.capacity = int(capacity)
        self.idx = torch.empty(max(self.capacity, 4), dtype=torch.int32, device=device)
        self.val = torch.empty(max(self.capacity, 8), dtype=torch.int16, device=device)
        self.seg_off = torch.zeros(n_tensors + 1, dtype=torch.int64, device=device)

    def c(self):
        return CBucket(self.idx.data_ptr(), self.val.data_ptr(), self.capacity, self.seg_off.data_ptr())


def ptr_table(tensors, device="cuda"):
    """Device array of the tensors' device pointers (keep the tensors alive yourself)."""
    return torch.tensor([t.data_ptr() for t in tensors], dtype=torch.int64, device=device)


def workspace(plan, device="cuda"):
    return torch.empty((plan.workspace_bytes() + 7) // 8, dtype=torch.int64, device=device)


def delta_encode(plan, old_tab, new_tab, new_dtype, buckets, ws, stream=None):
    cb = (CBucket * plan.n_buckets)(*[b.c() for b in buckets])
    _check(_lib.rose_delta_encode(plan._h, old_tab.data_ptr(), new_tab.data_ptr(), new_dtype, cb,
                                  ws.data_ptr(), ws.numel() * ws.element_size(), _stream(stream)),
           "delta_encode")


def delta_encode_refresh(plan, old_tab, new_tab, new_dtype, buckets, ws, stream=None):
    """delta_encode that also makes the old tensors equal to the new ones (as bf16)."""
    cb = (CBucket * plan.n_buckets)(*[b.c() for b in buckets])
    _check(_lib.rose_delta_encode_refresh(plan._h, old_tab.data_ptr(), new_tab.data_ptr(), new_dtype, cb,
                                          ws.data_ptr(), ws.numel() * ws.element_size(), _stream(stream)),
           "delta_encode_refresh")


ENCODE_REFRESH, ENCODE_ARITH = 1, 2
PAYLOAD_NEW, PAYLOAD_ARITH = 0, 1


def delta_encode_ex(plan, old_tab, new_tab, new_dtype, flags, buckets, ws, stream=None):
    """delta_encode with flags: ENCODE_REFRESH (old tensors are written), ENCODE_ARITH (arithmetic payloads)."""
    cb = (CBucket * plan.n_buckets)(*[b.c() for b in buckets])
    _check(_lib.rose_delta_encode_ex(plan._h, old_tab.data_ptr(), new_tab.data_ptr(), new_dtype, flags, cb,
                                     ws.data_ptr(), ws.numel() * ws.element_size(), _stream(stream)),
           "delta_encode_ex")


def delta_encode_static(plan, old_tab, new_tab, new_dtype, flags, buckets, stream=None):
    """delta_encode_ex on the library's built-in scratch: no workspace, no allocation (plan.upload() first)."""
    cb = (CBucket * plan.n_buckets)(*[b.c() for b in buckets])
    _check(_lib.rose_delta_encode_static(plan._h, old_tab.data_ptr(), new_tab.data_ptr(), new_dtype, flags, cb,
                                         _stream(stream)), "delta_encode_static")


def delta_apply_ex(plan, d, bucket, payload, dst_tab, stream=None):
    cb = bucket.c()
    _check(_lib.rose_delta_apply_ex(plan._h, d, ctypes.byref(cb), payload, dst_tab.data_ptr(), _stream(stream)),
           "delta_apply_ex")


def bucket_pack_ex(plan, d, bucket, payload, first_entry, n_entries, obj, stream=None):
    cb = bucket.c()
    _check(_lib.rose_bucket_pack_ex(plan._h, d, ctypes.byref(cb), payload, first_entry, n_entries, obj.data_ptr(),
                                    obj.numel() * obj.element_size(), _stream(stream)), "bucket_pack_ex")


def delta_apply(plan, d, bucket, dst_tab, stream=None):
    cb = bucket.c()
    _check(_lib.rose_delta_apply(plan._h, d, ctypes.byref(cb), dst_tab.data_ptr(), _stream(stream)),
           "delta_apply")


def dense_copy(plan, d, new_tab, new_dtype, dst_tab, stream=None):
    _check(_lib.rose_dense_copy(plan._h, d, new_tab.data_ptr(), new_dtype, dst_tab.data_ptr(),
                                _stream(stream)), "dense_copy")


def bucket_check(plan, bucket, stream=None):
    """-> number of entries the bucket needs; raises RoseError(ERR_CAPACITY) if it overflowed."""
    cb, req = bucket.c(), _i64()
    st = _lib.rose_bucket_check(plan._h, ctypes.byref(cb), _stream(stream), ctypes.byref(req))
    if st == ERR_CAPACITY:
        e = RoseError(st, "bucket_check")
        e.required = req.value
        raise e
    _check(st, "bucket_check")
    return req.value


def bw_probe(src, dst=None, sink=None, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(_lib.rose_bw_probe(src.data_ptr(), dst.data_ptr() if dst is not None else None, nbytes,
                              sink.data_ptr() if sink is not None else None, _stream(stream)), "bw_probe")


def bw_probe_mixed(src_a, src_b, dst, write_bytes_per_chunk, sink, stream=None, timed=False):
    """timed: the writes go out in the windows of time of the timed tile order"""
    nbytes = src_a.numel() * src_a.element_size()
    f = _lib.rose_bw_probe_mixed_timed if timed else _lib.rose_bw_probe_mixed
    _check(f(src_a.data_ptr(), src_b.data_ptr(), dst.data_ptr(), nbytes, write_bytes_per_chunk, sink.data_ptr(),
             _stream(stream)), "bw_probe_mixed")


def bw_probe_lines(dst, touched_fraction, stream=None):
    """read-modify-write of about `touched_fraction` of the 64-byte lines of dst"""
    thr = min(0xFFFFFFFF, max(0, int(round(touched_fraction * 4294967296.0))))
    _check(_lib.rose_bw_probe_lines(dst.data_ptr(), dst.numel() * dst.element_size(), thr, _stream(stream)),
           "bw_probe_lines")


def object_bytes(plan, n_entries):
    v = ctypes.c_size_t()
    _check(_lib.rose_object_bytes(plan._h, n_entries, ctypes.byref(v)), "object_bytes")
    return v.value


def bucket_pack(plan, d, bucket, first_entry, n_entries, obj, stream=None):
    """obj: uint8 device tensor of at least object_bytes(plan, n_entries)."""
    cb = bucket.c()
    _check(_lib.rose_bucket_pack(plan._h, d, ctypes.byref(cb), first_entry, n_entries, obj.data_ptr(),
                                 obj.numel() * obj.element_size(), _stream(stream)), "bucket_pack")


def object_apply(plan, obj, dst_tab, stream=None):
    _check(_lib.rose_object_apply(plan._h, obj.data_ptr(), obj.numel() * obj.element_size(), dst_tab.data_ptr(),
                                  _stream(stream)), "object_apply")


def object_check(plan, obj, stream=None, with_payload=False):
    """-> (shard, first_entry, n_entries), with the payload kind appended if asked for."""
    d, first, n, kind = _i32(), _i64(), _i64(), _i32()
    _check(_lib.rose_object_check(plan._h, obj.data_ptr(), obj.numel() * obj.element_size(), _stream(stream),
                                  ctypes.byref(d), ctypes.byref(first), ctypes.byref(n), ctypes.byref(kind)),
           "object_check")
    return (d.value, first.value, n.value, kind.value) if with_payload else (d.value, first.value, n.value)

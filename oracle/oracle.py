"""ctypes front end of the CPU oracle (``rose_oracle.c``).

TEST INFRASTRUCTURE: imported only by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports
this module and this module never imports the GPU library.

A *tensor record* is a dict with keys
  ``old``   numpy uint16 array of R*C bf16 bit patterns (W_{t-1})
  ``new``   numpy uint16 array (bf16 patterns) or uint32/float32 array (fp32 master)
  ``rows``, ``cols``, ``rule`` (0 replicated, 1 split rows, 2 split cols,
  3 fused rows) and, for rule 3, ``sections`` (row count of each stacked part).

A *bucket* (Sec. 4.2, COO data of one destination shard) is a dict with
  ``idx``     int32 local indices, ``val`` uint16 new bit patterns,
  ``seg_off`` int64 [n_tensors+1]: entries of tensor t are seg_off[t]:seg_off[t+1].
"""
import ctypes
import os
import subprocess

import numpy as np

REPLICATED, SPLIT_ROWS, SPLIT_COLS, FUSED_ROWS = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rose_oracle.c")
_LIB = os.path.join(_HERE, "librose_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain C, no special flags beyond -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32 = ctypes.c_int64, ctypes.c_int
        vp = ctypes.c_void_p
        lib.orc_rne_bf16.restype = ctypes.c_uint16
        lib.orc_rne_bf16.argtypes = [ctypes.c_uint32]
        lib.orc_rne_bf16_array.restype = None
        lib.orc_rne_bf16_array.argtypes = [vp, vp, i64]
        lib.orc_local_numel.restype = i64
        lib.orc_local_numel.argtypes = [i32, i64, i64, i32]
        lib.orc_shard_map.restype = i32
        lib.orc_shard_map.argtypes = [i32, i64, i64, i32, vp, i32, i64, i64, vp, vp, vp]
        lib.orc_encode_tensor.restype = i32
        lib.orc_encode_tensor.argtypes = [vp, vp, i32, i32, i64, i64, i32, vp, i32, vp, vp, vp]
        lib.orc_encode_tensor_src.restype = i32
        lib.orc_encode_tensor_src.argtypes = [vp, vp, i32, i32, i64, i64, i32, vp, i32, i32, i32, i32, i32, vp, vp, vp]
        lib.orc_apply.restype = i32
        lib.orc_apply.argtypes = [vp, vp, i64, vp, i64]
        lib.orc_stage_of.restype = i32
        lib.orc_stage_of.argtypes = [i32, i32, i32]
        u16 = ctypes.c_uint16
        lib.orc_bf16_nearest.restype = u16
        lib.orc_bf16_nearest.argtypes = [ctypes.c_double]
        lib.orc_bf16_add.restype = u16
        lib.orc_bf16_add.argtypes = [u16, u16]
        lib.orc_bf16_sub.restype = u16
        lib.orc_bf16_sub.argtypes = [u16, u16]
        lib.orc_arith_payload.restype = i32
        lib.orc_arith_payload.argtypes = [u16, u16, vp]
        lib.orc_arith_from_overwrite.restype = i32
        lib.orc_arith_from_overwrite.argtypes = [vp, vp, i64, vp, i64]
        lib.orc_apply_arith.restype = i32
        lib.orc_apply_arith.argtypes = [vp, vp, i64, vp, i64]
        lib.orc_dense_shard.restype = i32
        lib.orc_dense_shard.argtypes = [vp, i32, i64, i64, i32, vp, i32, i32, vp]
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    pass


def _check(rc, what):
    if rc != 0:
        names = {1: "bad argument", 2: "bad shape", 3: "out of range", 4: "order violated"}
        raise OracleError("%s: %s" % (what, names.get(rc, rc)))


def _sections(sections):
    sec = np.ascontiguousarray(np.asarray(sections if sections is not None else [], dtype=np.int64))
    return sec, (sec.ctypes.data if sec.size else None)


def rne_bf16(bits32):
    """fp32 bit pattern(s) -> bf16 bit pattern(s), round to nearest even."""
    lib = _load()
    if np.isscalar(bits32):
        return int(lib.orc_rne_bf16(int(bits32) & 0xFFFFFFFF))
    a = np.ascontiguousarray(bits32).view(np.uint32).ravel()
    out = np.empty(a.size, dtype=np.uint16)
    lib.orc_rne_bf16_array(a.ctypes.data, out.ctypes.data, a.size)
    return out


def local_numel(rule, rows, cols, tp):
    return int(_load().orc_local_numel(rule, rows, cols, tp))


def shard_map(rule, rows, cols, sections, tp, r, c):
    """-> (d_first, n_dest, local) of element (r, c)."""
    sec, secp = _sections(sections)
    d_first, n_dest, local = ctypes.c_int(), ctypes.c_int(), ctypes.c_int64()
    rc = _load().orc_shard_map(rule, rows, cols, sec.size, secp, tp, r, c,
                               ctypes.addressof(d_first), ctypes.addressof(n_dest),
                               ctypes.addressof(local))
    _check(rc, "shard_map")
    return d_first.value, n_dest.value, local.value


def encode_tensor(old, new, rows, cols, rule, sections, tp):
    """Dense-to-sparse of one tensor -> list over shards of (idx int32, val uint16)."""
    lib = _load()
    old = np.ascontiguousarray(old).view(np.uint16).ravel()
    new = np.ascontiguousarray(new).ravel()
    if new.dtype.itemsize == 4:
        new, is_f32 = new.view(np.uint32), 1
    elif new.dtype.itemsize == 2:
        new, is_f32 = new.view(np.uint16), 0
    else:
        raise OracleError("new must hold 16-bit or 32-bit patterns")
    if old.size != rows * cols or new.size != rows * cols:
        raise OracleError("array sizes do not match rows*cols")
    sec, secp = _sections(sections)
    counts = np.zeros(tp, dtype=np.int64)
    rc = lib.orc_encode_tensor(old.ctypes.data, new.ctypes.data, is_f32, rule, rows, cols,
                               sec.size, secp, tp, counts.ctypes.data, None, None)
    _check(rc, "encode_tensor(count)")
    idx = [np.empty(int(n), dtype=np.int32) for n in counts]
    val = [np.empty(int(n), dtype=np.uint16) for n in counts]
    pi = (ctypes.c_void_p * tp)(*[a.ctypes.data for a in idx])
    pv = (ctypes.c_void_p * tp)(*[a.ctypes.data for a in val])
    counts2 = np.zeros(tp, dtype=np.int64)
    rc = lib.orc_encode_tensor(old.ctypes.data, new.ctypes.data, is_f32, rule, rows, cols,
                               sec.size, secp, tp, counts2.ctypes.data, pi, pv)
    _check(rc, "encode_tensor(fill)")
    assert (counts == counts2).all()
    return list(zip(idx, val))


def encode_tensor_src(old_slice, new_slice, rows, cols, rule, sections, tp_dst, tp_src, src_rank,
                      sends_replicated=True, src_groups=0):
    """Dense-to-sparse of one tensor by the sender that holds shard `src_rank` of `tp_src` of it
    (rows, cols are the FULL tensor's) -> list over destination shards of (idx int32, val uint16).
    src_groups = G > 0: the sender side keeps a fused tensor interleaved by G head groups."""
    lib = _load()
    old = np.ascontiguousarray(old_slice).view(np.uint16).ravel()
    new = np.ascontiguousarray(new_slice).ravel()
    if new.dtype.itemsize == 4:
        new, is_f32 = new.view(np.uint32), 1
    elif new.dtype.itemsize == 2:
        new, is_f32 = new.view(np.uint16), 0
    else:
        raise OracleError("new must hold 16-bit or 32-bit patterns")
    want = local_numel(rule, rows, cols, tp_src)
    if old.size != want or new.size != want:
        raise OracleError("slice sizes do not match the sender's shard")
    sec, secp = _sections(sections)
    args = (is_f32, rule, rows, cols, sec.size, secp, tp_dst, tp_src, src_rank, 1 if sends_replicated else 0,
            src_groups)
    counts = np.zeros(tp_dst, dtype=np.int64)
    _check(lib.orc_encode_tensor_src(old.ctypes.data, new.ctypes.data, *args, counts.ctypes.data, None, None),
           "encode_tensor_src(count)")
    idx = [np.empty(int(n), dtype=np.int32) for n in counts]
    val = [np.empty(int(n), dtype=np.uint16) for n in counts]
    pi = (ctypes.c_void_p * tp_dst)(*[a.ctypes.data for a in idx])
    pv = (ctypes.c_void_p * tp_dst)(*[a.ctypes.data for a in val])
    counts2 = np.zeros(tp_dst, dtype=np.int64)
    _check(lib.orc_encode_tensor_src(old.ctypes.data, new.ctypes.data, *args, counts2.ctypes.data, pi, pv),
           "encode_tensor_src(fill)")
    assert (counts == counts2).all()
    return list(zip(idx, val))


def encode_model(tensors, tp):
    """All tensors -> one bucket per destination shard, segments in tensor order."""
    per_tensor = [encode_tensor(t["old"], t["new"], t["rows"], t["cols"], t["rule"],
                                t.get("sections"), tp) for t in tensors]
    buckets = []
    for d in range(tp):
        seg_off = np.zeros(len(tensors) + 1, dtype=np.int64)
        for i, segs in enumerate(per_tensor):
            seg_off[i + 1] = seg_off[i] + segs[d][0].size
        idx = np.concatenate([segs[d][0] for segs in per_tensor]) if tensors else np.empty(0, np.int32)
        val = np.concatenate([segs[d][1] for segs in per_tensor]) if tensors else np.empty(0, np.uint16)
        buckets.append({"idx": idx, "val": val, "seg_off": seg_off})
    return buckets


LAYER_FIRST, LAYER_LAST = -1, -2


def stage_of(layer, n_layers, pp):
    """Pipeline stage (of pp) that holds a tensor of decoder layer `layer` (LAYER_FIRST: in front of
    the layers, LAYER_LAST: behind them)."""
    s = _load().orc_stage_of(int(layer), int(n_layers), int(pp))
    if s < 0:
        raise OracleError("stage_of(%d, %d, %d)" % (layer, n_layers, pp))
    return s


def encode_model_pp(tensors, tp, tp_src, src_rank, n_layers, pp_src, stage_src, pp_dst):
    """Dense-to-sparse by the sender that is rank `src_rank` of `tp_src` in pipeline stage `stage_src`
    of `pp_src`, towards `pp_dst` receiving stages of `tp` shards each.  `tensors` lists the whole
    model (each with "layer"); "old" / "new" are the sender's slices and are looked at only for
    tensors of its own stage.  -> pp_dst * tp buckets, bucket stage * tp + d for shard d of a
    receiving stage; every bucket's seg_off counts all tensors of the model (segments of tensors that
    the sender does not hold, or that belong to another receiving stage, are empty)."""
    empty = (np.empty(0, np.int32), np.empty(0, np.uint16))
    per = []                                           # per tensor: receiving stage, per-shard (idx, val)
    for i, t in enumerate(tensors):
        to = stage_of(t["layer"], n_layers, pp_dst)
        if stage_of(t["layer"], n_layers, pp_src) != stage_src:
            per.append((to, [empty] * tp))
            continue
        per.append((to, encode_tensor_src(t["old"], t["new"], t["rows"], t["cols"], t["rule"], t.get("sections"),
                                          tp, tp_src, src_rank, sends_replicated=(i % tp_src == src_rank),
                                          src_groups=t.get("src_groups") or 0)))
    buckets = []
    for stage in range(pp_dst):
        for d in range(tp):
            segs = [s[d] if to == stage else empty for to, s in per]
            seg_off = np.zeros(len(tensors) + 1, dtype=np.int64)
            seg_off[1:] = np.cumsum([a.size for a, _ in segs])
            buckets.append({"idx": np.concatenate([a for a, _ in segs]) if segs else empty[0],
                            "val": np.concatenate([v for _, v in segs]) if segs else empty[1],
                            "seg_off": seg_off})
    return buckets


def apply_segment(idx, val, dst):
    """Sparse-to-dense of one segment, in place on ``dst`` (uint16, flat local copy)."""
    assert dst.dtype == np.uint16 and dst.flags["C_CONTIGUOUS"]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.uint16)
    rc = _load().orc_apply(idx.ctypes.data, val.ctypes.data, idx.size, dst.ctypes.data, dst.size)
    _check(rc, "apply")


def apply_bucket(bucket, dsts):
    """Apply every segment of a bucket onto the receiver's local copies ``dsts[t]``."""
    so = bucket["seg_off"]
    for t, dst in enumerate(dsts):
        a, b = int(so[t]), int(so[t + 1])
        apply_segment(bucket["idx"][a:b], bucket["val"][a:b], dst)


# ---------------------------------------------------------------------------------------------
# Arithmetic payload (Sec. 4.2 writes the update as W_t = W_{t-1} + dW_t): an entry carries the
# bf16-rounded difference where adding it back to the old pattern reproduces the new one, and
# otherwise the new pattern itself with bit 31 of its index set (int32: a negative index).
# ---------------------------------------------------------------------------------------------
ESCAPE = np.int32(-2**31)


def bf16_nearest(x):
    """bf16 pattern nearest to the double x (ties to even)."""
    return int(_load().orc_bf16_nearest(float(x)))


def bf16_add(a, b):
    return int(_load().orc_bf16_add(int(a), int(b)))


def bf16_sub(a, b):
    return int(_load().orc_bf16_sub(int(a), int(b)))


def arith_payload(old_bits, new_bits):
    """(escape, val) of one entry."""
    v = ctypes.c_uint16(0)
    esc = _load().orc_arith_payload(int(old_bits), int(new_bits), ctypes.addressof(v))
    return bool(esc), int(v.value)


def arith_bucket(bucket, old_locals):
    """The bucket with arithmetic payloads; ``old_locals[t]`` is the receiver's resident copy
    (uint16, flat) of tensor t, the value it will add to.  Returns a new bucket."""
    idx = np.array(bucket["idx"], dtype=np.int32, copy=True)
    val = np.array(bucket["val"], dtype=np.uint16, copy=True)
    so = bucket["seg_off"]
    for t, old in enumerate(old_locals):
        a, b = int(so[t]), int(so[t + 1])
        old = np.ascontiguousarray(old).view(np.uint16).ravel()
        si, sv = idx[a:b], val[a:b]          # contiguous views: converted in place
        _check(_load().orc_arith_from_overwrite(si.ctypes.data, sv.ctypes.data, b - a, old.ctypes.data, old.size),
               "arith_from_overwrite")
    return {"idx": idx, "val": val, "seg_off": np.array(so, dtype=np.int64, copy=True)}


def apply_segment_arith(idx, val, dst):
    assert dst.dtype == np.uint16 and dst.flags["C_CONTIGUOUS"]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.uint16)
    _check(_load().orc_apply_arith(idx.ctypes.data, val.ctypes.data, idx.size, dst.ctypes.data, dst.size),
           "apply_arith")


def apply_bucket_arith(bucket, dsts):
    so = bucket["seg_off"]
    for t, dst in enumerate(dsts):
        a, b = int(so[t]), int(so[t + 1])
        apply_segment_arith(bucket["idx"][a:b], bucket["val"][a:b], dst)


def dense_shard(full, rows, cols, rule, sections, tp, d):
    """Shard d's local copy of a full tensor, through the shard map (dense path)."""
    full = np.ascontiguousarray(full).view(np.uint16).ravel()
    sec, secp = _sections(sections)
    out = np.zeros(local_numel(rule, rows, cols, tp), dtype=np.uint16)
    rc = _load().orc_dense_shard(full.ctypes.data, rule, rows, cols, sec.size, secp, tp, d,
                                 out.ctypes.data)
    _check(rc, "dense_shard")
    return out


# ---------------------------------------------------------------------------------------------
# Transport objects (Sec. 4.2 "Asynchronous Weight Transfer": senders push fixed-size buckets to a
# relay, receivers pull what their metadata says they need).  A destination's entry stream is cut
# into objects that carry their own description, so each can be applied alone and in any order.
# The byte layout is this build's own (the paper fixes none); written out here by definition:
#   0   u32 magic 0x45534F52, u32 version 1, i32 shard, i32 n_tensors
#   16  i64 first_entry (position of the object's first entry in the shard's stream), i64 n_entries
#   32  zero up to 64
#   64  i64 seg_off[n_tensors + 1]: entries of tensor t are [seg_off[t], seg_off[t+1]) of THIS object
#   A   i32 idx[n_entries]   A = 64 + 8 (n_tensors + 1) rounded up to 16
#   B   u16 val[n_entries]   B = A + 4 n_entries rounded up to 16;  size = B + 2 n_entries rounded up to 16
# ---------------------------------------------------------------------------------------------
OBJECT_MAGIC = 0x45534F52


def _up16(x):
    return (x + 15) // 16 * 16


def object_bytes(n_tensors, n_entries):
    a = _up16(64 + 8 * (n_tensors + 1))
    return a + _up16(4 * n_entries) + _up16(2 * n_entries)


def pack_object(bucket, shard, first_entry, n_entries):
    """bucket: dict idx, val, seg_off (a whole destination stream) -> the object's bytes (uint8)."""
    seg = np.asarray(bucket["seg_off"], dtype=np.int64)
    nt = seg.size - 1
    total = int(seg[-1])
    if first_entry < 0 or n_entries < 0 or first_entry + n_entries > total:
        raise OracleError("object range outside the stream")
    out = np.zeros(object_bytes(nt, n_entries), dtype=np.uint8)
    out[0:8].view(np.uint32)[:] = (OBJECT_MAGIC, 1)
    out[8:16].view(np.int32)[:] = (shard, nt)
    out[16:32].view(np.int64)[:] = (first_entry, n_entries)
    local = np.clip(seg - first_entry, 0, n_entries)
    out[64:64 + 8 * (nt + 1)].view(np.int64)[:] = local
    a = _up16(64 + 8 * (nt + 1))
    b = a + _up16(4 * n_entries)
    out[a:a + 4 * n_entries].view(np.int32)[:] = np.asarray(bucket["idx"], dtype=np.int32)[first_entry:first_entry + n_entries]
    out[b:b + 2 * n_entries].view(np.uint16)[:] = np.asarray(bucket["val"], dtype=np.uint16)[first_entry:first_entry + n_entries]
    return out


def unpack_object(obj, n_tensors):
    """Object bytes -> dict shard, first_entry, idx, val, seg_off; raises on a malformed object."""
    obj = np.ascontiguousarray(obj, dtype=np.uint8)
    if obj.size < 64 + 8 * (n_tensors + 1):
        raise OracleError("object too short")
    magic, version = (int(x) for x in obj[0:8].view(np.uint32))
    shard, nt = (int(x) for x in obj[8:16].view(np.int32))
    first, n = (int(x) for x in obj[16:32].view(np.int64))
    if magic != OBJECT_MAGIC or version != 1 or nt != n_tensors or n < 0 or first < 0:
        raise OracleError("bad object header")
    if obj.size < object_bytes(nt, n):
        raise OracleError("object shorter than its header says")
    seg = obj[64:64 + 8 * (nt + 1)].view(np.int64).copy()
    if seg[0] != 0 or seg[-1] != n or (np.diff(seg) < 0).any():
        raise OracleError("bad segment table")
    a = _up16(64 + 8 * (nt + 1))
    b = a + _up16(4 * n)
    return {"shard": shard, "first_entry": first, "seg_off": seg,
            "idx": obj[a:a + 4 * n].view(np.int32).copy(), "val": obj[b:b + 2 * n].view(np.uint16).copy()}


def apply_object(obj, n_tensors, dsts):
    """Apply one object to the destination shard's tensors (list of uint16 arrays)."""
    apply_bucket(unpack_object(obj, n_tensors), dsts)

"""ctypes binding with the same names as the C ABI in include/th.h.

Only marshals arguments.  There is no fallback: if the shared library is
missing or fails to load, importing this module raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtensorhub_reshard.so")

TH_BF16, TH_F32 = 1, 2
TH_FLAG_HOST_ONLY, TH_FLAG_PTRS_ALIGNED16, TH_FLAG_CHECKSUM, TH_FLAG_NARROW_AT_UNPACK = 1, 2, 4, 8
TH_FLAG_PROGRESS = 16
TH_CFG_TILE_BYTES = 1
TH_CFG_TILE_BYTES_ANY = 2
TH_CFG_SPECIALIZE = 3
TH_CFG_TILE_BYTES_CHECKSUM = 4
TH_CFG_TILE_BYTES_NARROW = 5
TH_CFG_PLANNER_THREADS = 6
TH_CFG_TILE_BYTES_PROGRESS = 7
TH_CFG_SHORT_TILE_SLOTS = 8
TH_MODEL_DENSE, TH_MODEL_MOE = 1, 2
_DTYPE = {"bf16": TH_BF16, "f32": TH_F32}
_DTYPE_NAME = {TH_BF16: "bf16", TH_F32: "f32", 0: None}


def library_path():
    return _LIB_PATH


if not os.path.exists(_LIB_PATH):
    raise ImportError(
        "%s is missing: build it with `python -m paper_2604_09107_amd.build` "
        "(the reshard path has no non-HIP fallback)" % _LIB_PATH)
# PyTorch for ROCm ships its own copy of the HIP runtime, and a process must hold one runtime only
# (torch owns the buffers and streams that this library is handed).  Let torch load first when it
# is installed; the library then binds to the runtime that is already in the process.  Loading in
# the other order ends in "no ROCm-capable device" at the first plan.
try:
    import torch  # noqa: F401
except ImportError:
    pass
_lib = C.CDLL(_LIB_PATH)


class ThError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("th error %d: %s" % (code, msg))
        self.code = code


class _ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in (
        "kind", "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
        "tied_embeddings", "n_experts", "n_shared_experts", "expert_ffn", "weight_dtype", "norm_dtype")]


class _Layout(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("tp_size", "tp_rank", "ep_size", "ep_rank", "experts_stacked", "f32_store",
                                       "qkv_grouped", "padded_vocab")]


class _Segment(C.Structure):
    _fields_ = [("src_tensor", C.c_uint32), ("dst_tensor", C.c_uint32),
                ("src_elem_off", C.c_uint64), ("dst_elem_off", C.c_uint64),
                ("src_row_stride", C.c_uint64), ("dst_row_stride", C.c_uint64),
                ("nrows", C.c_uint64), ("row_len", C.c_uint64),
                ("src_dtype", C.c_uint8), ("dst_dtype", C.c_uint8), ("reserved", C.c_uint8 * 6)]


SEGMENT_NP = np.dtype([("src_tensor", "<u4"), ("dst_tensor", "<u4"), ("src_elem_off", "<u8"),
                       ("dst_elem_off", "<u8"), ("src_row_stride", "<u8"), ("dst_row_stride", "<u8"),
                       ("nrows", "<u8"), ("row_len", "<u8"), ("src_dtype", "u1"), ("dst_dtype", "u1"),
                       ("reserved", "u1", (6,))])
assert SEGMENT_NP.itemsize == C.sizeof(_Segment) == 64


class Run(C.Structure):
    _fields_ = [("src_tensor", C.c_uint32), ("dst_tensor", C.c_uint32), ("chunk", C.c_uint32),
                ("reserved", C.c_uint32),
                ("src_byte_off", C.c_uint64), ("src_byte_stride", C.c_uint64),
                ("dst_byte_off", C.c_uint64), ("dst_byte_stride", C.c_uint64),
                ("chunk_byte_off", C.c_uint64), ("wire_byte_stride", C.c_uint64),
                ("nrows", C.c_uint64), ("row_len", C.c_uint64),
                ("src_dtype", C.c_uint8), ("dst_dtype", C.c_uint8), ("pad_bytes", C.c_uint8),
                ("wire_dtype", C.c_uint8), ("reserved2", C.c_uint8 * 4)]


class TileInfo(C.Structure):
    _fields_ = [("src_buf", C.c_uint32), ("dst_buf", C.c_uint32),
                ("src_byte_off", C.c_uint64), ("src_byte_stride", C.c_uint64),
                ("dst_byte_off", C.c_uint64), ("dst_byte_stride", C.c_uint64),
                ("first_col", C.c_uint64), ("row_len", C.c_uint64), ("count", C.c_uint64),
                ("elem_bytes_src", C.c_uint8), ("elem_bytes_dst", C.c_uint8), ("kind", C.c_uint8),
                ("pad_bytes", C.c_uint8), ("reserved", C.c_uint8 * 4),
                ("src_tensor", C.c_uint32), ("reserved2", C.c_uint32), ("run_unit_base", C.c_uint64)]


def _sig(name, restype, *argtypes):
    f = getattr(_lib, name)
    f.restype = restype
    f.argtypes = list(argtypes)
    return f


_P = C.c_void_p
_plan_create = _sig("th_plan_create", C.c_int, C.POINTER(_ModelDesc), C.POINTER(_Layout), C.POINTER(_Layout),
                    C.c_size_t, C.c_uint, C.POINTER(_P))
_plan_create_seg = _sig("th_plan_create_from_segments", C.c_int, _P, C.c_size_t, _P, C.c_uint32, _P, C.c_uint32,
                        C.c_size_t, C.c_uint, C.POINTER(_P))
_pack = _sig("th_pack", C.c_int, _P, _P, C.c_uint32, _P, C.c_uint32, C.c_uint32, _P)
_pack_progress = _sig("th_pack_progress", C.c_int, _P, _P, C.c_uint32, _P, C.c_uint32, C.c_uint32, _P, _P)
_unpack_progress = _sig("th_unpack_progress", C.c_int, _P, _P, C.c_uint32, C.c_uint32, _P, C.c_uint32, _P, _P)
_pack_noalloc = _sig("th_pack_noalloc", C.c_int, _P, _P, C.c_uint32, _P, C.c_uint32, C.c_uint32, _P)
_unpack = _sig("th_unpack", C.c_int, _P, _P, C.c_uint32, C.c_uint32, _P, C.c_uint32, _P)
_pack_sum = _sig("th_pack_checksum", C.c_int, _P, _P, C.c_uint32, _P, C.c_uint32, C.c_uint32, _P, _P)
_unpack_sum = _sig("th_unpack_checksum", C.c_int, _P, _P, C.c_uint32, C.c_uint32, _P, C.c_uint32, _P, _P)
_reshard = _sig("th_reshard", C.c_int, _P, _P, C.c_uint32, _P, C.c_uint32, _P)
_destroy = _sig("th_plan_destroy", C.c_int, _P)
_num_chunks = _sig("th_plan_num_chunks", C.c_uint32, _P)
_chunk_bytes = _sig("th_plan_chunk_bytes", C.c_size_t, _P, C.c_uint32)
_wire_bytes = _sig("th_plan_wire_bytes", C.c_size_t, _P)
_payload_bytes = _sig("th_plan_payload_bytes", C.c_size_t, _P)
_src_read_bytes = _sig("th_plan_src_read_bytes", C.c_size_t, _P)
_num_tensors = _sig("th_plan_num_tensors", C.c_uint32, _P, C.c_int)
_tensor_info = _sig("th_plan_tensor_info", C.c_int, _P, C.c_int, C.c_uint32, C.c_char_p, C.c_size_t,
                    C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_int))
_num_runs = _sig("th_plan_num_runs", C.c_size_t, _P)
_get_run = _sig("th_plan_get_run", C.c_int, _P, C.c_size_t, C.POINTER(Run))
_num_tiles = _sig("th_plan_num_tiles", C.c_size_t, _P, C.c_int)
_get_tile = _sig("th_plan_get_tile", C.c_int, _P, C.c_int, C.c_size_t, C.POINTER(TileInfo))
_chunk_first_tile = _sig("th_plan_chunk_first_tile", C.c_size_t, _P, C.c_int, C.c_int, C.c_uint32)
_signal = _sig("th_signal", C.c_int, _P, C.c_uint64, _P)
_tensors_complete = _sig("th_plan_tensors_complete", C.c_uint32, _P, C.c_uint32)
_reference_copy = _sig("th_reference_copy", C.c_int, _P, _P, C.c_size_t, _P)
_config_set = _sig("th_config_set", C.c_int, C.c_int, C.c_uint64)
_config_get = _sig("th_config_get", C.c_uint64, C.c_int)
_last_error = _sig("th_last_error", C.c_char_p)
_version = _sig("th_version", C.c_char_p)


def th_last_error():
    return _last_error().decode()


def th_version():
    return _version().decode()


def _check(rc):
    if rc != 0:
        raise ThError(rc, th_last_error())


def _model_struct(m):
    return _ModelDesc(
        kind=TH_MODEL_MOE if m["kind"] == "moe" else TH_MODEL_DENSE,
        n_layers=m["n_layers"], hidden=m["hidden"], n_q_heads=m["n_q_heads"], n_kv_heads=m["n_kv_heads"],
        head_dim=m["head_dim"], ffn=m["ffn"], vocab=m["vocab"], tied_embeddings=int(m["tied_embeddings"]),
        n_experts=m["n_experts"], n_shared_experts=m["n_shared_experts"], expert_ffn=m["expert_ffn"],
        weight_dtype=_DTYPE[m["weight_dtype"]], norm_dtype=_DTYPE[m["norm_dtype"]])


def _layout_struct(l):
    return _Layout(tp_size=l["tp_size"], tp_rank=l["tp_rank"], ep_size=l["ep_size"], ep_rank=l["ep_rank"],
                   experts_stacked=int(l["experts_stacked"]), f32_store=_DTYPE[l["f32_store"]],
                   qkv_grouped=int(l.get("qkv_grouped", 0)), padded_vocab=int(l.get("padded_vocab", 0)))


class Plan:
    """Handle of a th_plan plus its read-only queries."""

    def __init__(self, handle):
        self._h = handle

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("plan was destroyed")
        return self._h

    num_chunks = property(lambda self: _num_chunks(self.handle))
    wire_bytes = property(lambda self: _wire_bytes(self.handle))
    payload_bytes = property(lambda self: _payload_bytes(self.handle))
    src_read_bytes = property(lambda self: _src_read_bytes(self.handle))
    num_runs = property(lambda self: _num_runs(self.handle))

    def chunk_bytes(self, c):
        return _chunk_bytes(self.handle, c)

    def num_tensors(self, side):
        return _num_tensors(self.handle, side)

    def tensor_info(self, side, i):
        name = C.create_string_buffer(256)
        rows, cols, dt = C.c_uint64(), C.c_uint64(), C.c_int()
        _check(_tensor_info(self.handle, side, i, name, 256, C.byref(rows), C.byref(cols), C.byref(dt)))
        return dict(name=name.value.decode(), rows=rows.value, cols=cols.value, dtype=_DTYPE_NAME[dt.value])

    def tensors(self, side):
        return [self.tensor_info(side, i) for i in range(self.num_tensors(side))]

    def run(self, i):
        r = Run()
        _check(_get_run(self.handle, i, C.byref(r)))
        return r

    def num_tiles(self, side):
        return _num_tiles(self.handle, side)

    def tile(self, side, i):
        t = TileInfo()
        _check(_get_tile(self.handle, side, i, C.byref(t)))
        return t

    def chunk_first_tile(self, side, path_class, chunk):
        return _chunk_first_tile(self.handle, side, path_class, chunk)

    def tensors_complete(self, n_chunks_done):
        return _tensors_complete(self.handle, n_chunks_done)

    def destroy(self):
        if self._h is not None:
            _check(_destroy(self._h))
            self._h = None


def th_plan_create(model, src_layout, dst_layout, chunk_bytes, flags=0):
    """model / layouts: dicts with the fields of th_model_desc / th_layout (dtypes as "bf16" / "f32")."""
    out = _P()
    m, s, d = _model_struct(model), _layout_struct(src_layout), _layout_struct(dst_layout)
    _check(_plan_create(C.byref(m), C.byref(s), C.byref(d), chunk_bytes, flags, C.byref(out)))
    return Plan(out.value)


def th_plan_create_from_segments(segments, src_tensor_elems, dst_tensor_elems, chunk_bytes, flags=0):
    """segments: numpy structured array of dtype SEGMENT_NP in wire order."""
    segs = np.ascontiguousarray(segments, dtype=SEGMENT_NP)
    se = np.ascontiguousarray(src_tensor_elems, dtype=np.uint64)
    de = np.ascontiguousarray(dst_tensor_elems, dtype=np.uint64)
    out = _P()
    _check(_plan_create_seg(segs.ctypes.data, len(segs), se.ctypes.data, len(se), de.ctypes.data, len(de),
                            chunk_bytes, flags, C.byref(out)))
    return Plan(out.value)


def _ptr_array(ptrs):
    return np.ascontiguousarray(ptrs, dtype=np.uint64)


def th_pack(plan, src_ptrs, wire_ptrs, chunk_first, chunk_count, stream=0):
    """src_ptrs / wire_ptrs: sequences (or uint64 arrays) of device addresses; stream: hipStream_t as int."""
    s, w = _ptr_array(src_ptrs), _ptr_array(wire_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_pack(plan.handle, s.ctypes.data, len(s), w.ctypes.data, chunk_first, chunk_count, stream))


def th_pack_progress(plan, src_ptrs, wire_ptrs, chunk_first, chunk_count, progress_ptr, stream=0):
    """progress_ptr: address of a uint64 in device memory or device-visible pinned host memory."""
    s, w = _ptr_array(src_ptrs), _ptr_array(wire_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_pack_progress(plan.handle, s.ctypes.data, len(s), w.ctypes.data, chunk_first, chunk_count, progress_ptr,
                          stream))


def th_unpack_progress(plan, wire_ptrs, chunk_first, chunk_count, dst_ptrs, progress_ptr, stream=0):
    w, d = _ptr_array(wire_ptrs), _ptr_array(dst_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_unpack_progress(plan.handle, w.ctypes.data, chunk_first, chunk_count, d.ctypes.data, len(d), progress_ptr,
                            stream))


def th_pack_noalloc(plan, src_ptrs, wire_ptrs, chunk_first, chunk_count, stream=0):
    """th_pack with its device pointer tables in a fixed array inside the library (allocates nothing)."""
    s, w = _ptr_array(src_ptrs), _ptr_array(wire_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_pack_noalloc(plan.handle, s.ctypes.data, len(s), w.ctypes.data, chunk_first, chunk_count, stream))


def th_unpack(plan, wire_ptrs, chunk_first, chunk_count, dst_ptrs, stream=0):
    w, d = _ptr_array(wire_ptrs), _ptr_array(dst_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_unpack(plan.handle, w.ctypes.data, chunk_first, chunk_count, d.ctypes.data, len(d), stream))


def th_pack_checksum(plan, src_ptrs, wire_ptrs, chunk_first, chunk_count, sums_ptr, stream=0):
    """sums_ptr: device address of 2 * plan.num_tensors(0) uint64, zeroed by the caller before a sweep."""
    s, w = _ptr_array(src_ptrs), _ptr_array(wire_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_pack_sum(plan.handle, s.ctypes.data, len(s), w.ctypes.data, chunk_first, chunk_count, sums_ptr, stream))


def th_unpack_checksum(plan, wire_ptrs, chunk_first, chunk_count, dst_ptrs, sums_ptr, stream=0):
    w, d = _ptr_array(wire_ptrs), _ptr_array(dst_ptrs)
    if len(w) != chunk_count:
        raise ValueError("need one wire pointer per chunk in the range")
    _check(_unpack_sum(plan.handle, w.ctypes.data, chunk_first, chunk_count, d.ctypes.data, len(d), sums_ptr, stream))


def th_reshard(plan, src_ptrs, dst_ptrs, stream=0):
    s, d = _ptr_array(src_ptrs), _ptr_array(dst_ptrs)
    _check(_reshard(plan.handle, s.ctypes.data, len(s), d.ctypes.data, len(d), stream))


def th_plan_destroy(plan):
    plan.destroy()


def th_signal(flag_ptr, value, stream=0):
    _check(_signal(flag_ptr, value, stream))


def th_reference_copy(dst_ptr, src_ptr, nbytes, stream=0):
    _check(_reference_copy(dst_ptr, src_ptr, nbytes, stream))


def th_config_set(key, value):
    _check(_config_set(key, value))


def th_config_get(key):
    return _config_get(key)

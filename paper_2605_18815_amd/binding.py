"""Thin ctypes binding of include/vps.h: argument marshalling only.

Every function of the C ABI appears here under the same name (without the ``vps_`` prefix)
as a method of :class:`Library`.  Device pointers are passed as integers (for example
``tensor.data_ptr()``), streams as the integer value of a ``hipStream_t``.  There is no CPU
fallback: if the HIP library is missing or a call fails, an exception is raised.
"""
import ctypes as C

import numpy as np

from . import build as _build

OK = 0
ERR_INVALID_ARG, ERR_INDIVISIBLE, ERR_RANK_RANGE, ERR_MODEL_MISMATCH = -1, -2, -3, -4
ERR_SCRATCH_TOO_SMALL, ERR_OOM, ERR_HIP = -5, -6, -7
NUM_BUFFERS = 8
NO_POS = (1 << 64) - 1
OPT_TILE_BYTES, OPT_SMALL_PLAN_BOXES, OPT_XPOSE_SHAPE, OPT_XCD_RUN, OPT_PAIR_ORDER_WORK = range(5)
PLAN_ROUTES_ONLY = 1
PLAN_THROUGH_BUFFERS = 2
COLL_NONE, COLL_P2P, COLL_BROADCAST, COLL_SCATTER, COLL_GATHER = range(5)

MODEL_FIELDS = ("family", "layers", "hidden", "q_heads", "kv_heads", "head_dim", "ffn", "vocab",
                "experts", "expert_ffn")
PARALLEL_FIELDS = ("tp", "pp", "dp", "ep", "zero_stage", "gpus_per_node", "qkv_layout",
                   "expert_layout", "flat_order", "ep_placement")


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in MODEL_FIELDS]


class ParallelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in PARALLEL_FIELDS]


class PlanStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("num_boxes", "num_retain_boxes", "num_send_boxes",
                                         "num_recv_boxes", "num_pack_tiles", "num_unpack_tiles",
                                         "num_retain_tiles", "num_peers_out", "num_peers_in")] + \
               [("plan_ms", C.c_double)]


PIECE_DTYPE = np.dtype([("tensor", "<i4"), ("rank", "<i4"), ("kind", "<i4"), ("buf", "<i4"),
                        ("lo", "<i4", (4,)), ("ext", "<i4", (4,)), ("off", "<i8"),
                        ("stride", "<i8", (4,))], align=True)
BOX_DTYPE = np.dtype([("tensor", "<i4"), ("kind", "<i4"), ("src_rank", "<i4"), ("dst_rank", "<i4"),
                      ("src_buf", "<i4"), ("dst_buf", "<i4"), ("lo", "<i4", (4,)),
                      ("ext", "<i4", (4,)), ("src_off", "<i8"), ("dst_off", "<i8"),
                      ("src_stride", "<i8", (4,)), ("dst_stride", "<i8", (4,)),
                      ("send_pos", "<u8"), ("recv_pos", "<u8")], align=True)
assert PIECE_DTYPE.itemsize == 88 and BOX_DTYPE.itemsize == 152


class VpsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"vps error {code}: {msg}")
        self.code = code


def model_desc(m):
    """The vps_model_desc of a dict of its fields (a struct made earlier passes through: callers
    that describe the same model again and again build it once)."""
    if isinstance(m, ModelDesc):
        return m
    return ModelDesc(**{k: int(m[k]) for k in MODEL_FIELDS})


def parallel_desc(p):
    """The vps_parallel_desc of a dict of its fields (`zero` is accepted for `zero_stage`); a
    struct made earlier passes through."""
    if isinstance(p, ParallelDesc):
        return p
    d = dict(p)
    if "zero" in d:
        d["zero_stage"] = d.pop("zero")
    d.setdefault("ep_placement", 0)
    return ParallelDesc(**{k: int(d[k]) for k in PARALLEL_FIELDS})


def _ptr_array(ptrs, n):
    if len(ptrs) != n:
        raise ValueError(f"expected {n} buffer pointers, got {len(ptrs)}")
    return (C.c_void_p * n)(*[int(p) if p else None for p in ptrs])


class Library:
    """The loaded C ABI.  ``prefix`` selects the exported symbol family (``vps_``)."""

    def __init__(self, path=None, prefix="vps_"):
        self.path = path or _build.library_path()
        self.prefix = prefix
        if prefix == "vps_":
            # PyTorch bundles its own HIP runtime under the same soname.  Loading torch first
            # makes this library bind to that copy, so that the process has one runtime and
            # torch-allocated memory and streams are valid in our calls.
            import torch  # noqa: F401
        self._dll = C.CDLL(self.path)
        vp, i32, i64, u64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_uint32
        P = C.POINTER
        sig = {
            "describe_config": [P(ModelDesc), P(ParallelDesc), i32, P(vp)],
            "plan_intersections": [vp, vp, i32, vp, P(vp)],
            "plan_intersections_ex": [vp, vp, i32, u32, vp, P(vp)],
            "pack": [vp, i32, P(vp), vp, vp],
            "unpack": [vp, i32, vp, P(vp), vp],
            "apply_transition": [vp, i32, P(vp), P(vp), vp, u64, vp],
            "config_world": [vp, P(i32)],
            "config_num_tensors": [vp, P(i32)],
            "config_num_buffers": [vp, i32, P(i32)],
            "config_buffer_bytes": [vp, i32, i32, P(u64)],
            "config_num_pieces": [vp, P(i64)],
            "config_get_pieces": [vp, vp, i64],
            "plan_pair_bytes": [vp, i32, i32, P(u64)],
            "plan_peer_bytes": [vp, i32, i32, P(u64), P(u64)],
            "plan_buffer_bytes": [vp, i32, P(u64), P(u64), P(u64), P(u64), P(u64)],
            "plan_peer_segment": [vp, i32, i32, P(u64), P(u64), P(u64)],
            "plan_num_boxes": [vp, P(i64)],
            "plan_get_boxes": [vp, vp, i64],
            "plan_stats": [vp, P(PlanStats)],
            "set_tile_bytes": [u32],
            "set_option": [i32, u32],
            "plain_copy": [vp, vp, u64, vp],
            "plain_read": [vp, u64, vp, vp],
            "plain_fill": [vp, u64, vp],
            "stage_exchange": [vp, u64, vp, P(vp)],
            "plan_classify_collectives": [vp, vp, vp, P(i32), i64],
            "stage_info": [vp, P(i32), P(i32), P(u64)],
            "stage_steps": [vp, P(i32), P(u64), i32],
            "apply_transition_staged": [vp, P(vp), P(vp), vp, u64, vp],
        }
        if prefix == "vps_":
            # product library only: the entry point that keeps its staging area in a device
            # array of the library image
            sig["apply_transition_static"] = [vp, P(vp), P(vp), vp]
        self._fn = {}
        for name, argtypes in sig.items():
            f = getattr(self._dll, prefix + name)
            f.argtypes = argtypes
            f.restype = C.c_int
            self._fn[name] = f
        for name in ("config_destroy", "plan_destroy", "stage_plan_destroy"):
            f = getattr(self._dll, prefix + name)
            f.argtypes = [vp]
            f.restype = None
            self._fn[name] = f
        f = getattr(self._dll, prefix + "last_error")
        f.argtypes = []
        f.restype = C.c_char_p
        self._fn["last_error"] = f
        if prefix == "vps_":
            f = getattr(self._dll, prefix + "static_scratch_bytes")
            f.argtypes = []
            f.restype = C.c_uint64
            self._fn["static_scratch_bytes"] = f

    EXPORTS = ("describe_config", "plan_intersections", "pack", "unpack", "apply_transition",
               "config_world", "config_num_tensors", "config_num_buffers", "config_buffer_bytes", "config_num_pieces",
               "config_get_pieces", "plan_pair_bytes", "plan_peer_bytes", "plan_buffer_bytes",
               "plan_peer_segment", "plan_num_boxes", "plan_get_boxes", "plan_stats",
               "set_tile_bytes", "plain_copy", "config_destroy", "plan_destroy", "last_error", "stage_exchange", "plan_intersections_ex", "plan_classify_collectives",
               "stage_info", "stage_steps", "apply_transition_staged", "stage_plan_destroy",
               "apply_transition_static", "static_scratch_bytes", "set_option", "plain_read", "plain_fill")

    def last_error(self):
        return self._fn["last_error"]().decode()

    def _check(self, rc):
        if rc != OK:
            raise VpsError(rc, self.last_error())

    # ---- the five calls
    def describe_config(self, model, par, rank=-1):
        out = C.c_void_p()
        m, p = model_desc(model), parallel_desc(par)
        self._check(self._fn["describe_config"](C.byref(m), C.byref(p), rank, C.byref(out)))
        return Config(self, out)

    def plan_intersections(self, src, dst, rank=-1, stream=0):
        out = C.c_void_p()
        self._check(self._fn["plan_intersections"](src._h, dst._h, rank, stream, C.byref(out)))
        return Plan(self, out)

    def plan_intersections_ex(self, src, dst, rank=-1, flags=0, stream=0):
        out = C.c_void_p()
        self._check(self._fn["plan_intersections_ex"](src._h, dst._h, rank, flags, stream, C.byref(out)))
        return Plan(self, out)

    def pack(self, plan, rank, src_bufs, send_buf, stream=0):
        self._check(self._fn["pack"](plan._h, rank, _ptr_array(src_bufs, NUM_BUFFERS), send_buf, stream))

    def unpack(self, plan, rank, recv_buf, dst_bufs, stream=0):
        self._check(self._fn["unpack"](plan._h, rank, recv_buf, _ptr_array(dst_bufs, NUM_BUFFERS), stream))

    def apply_transition(self, plan, rank, src_bufs, dst_bufs, scratch, scratch_bytes, stream=0):
        self._check(self._fn["apply_transition"](plan._h, rank, _ptr_array(src_bufs, len(src_bufs)),
                                                 _ptr_array(dst_bufs, len(dst_bufs)), scratch,
                                                 scratch_bytes, stream))

    def apply_transition_static(self, plan, src_bufs, dst_bufs, stream=0):
        self._check(self._fn["apply_transition_static"](plan._h, _ptr_array(src_bufs, len(src_bufs)),
                                                        _ptr_array(dst_bufs, len(dst_bufs)), stream))

    def static_scratch_bytes(self):
        return int(self._fn["static_scratch_bytes"]())

    def stage_exchange(self, plan, budget_bytes_per_rank, stream=0):
        out = C.c_void_p()
        self._check(self._fn["stage_exchange"](plan._h, budget_bytes_per_rank, stream, C.byref(out)))
        return StagePlan(self, out, plan)

    def apply_transition_staged(self, sp, src_bufs, dst_bufs, scratch, scratch_bytes, stream=0):
        self._check(self._fn["apply_transition_staged"](sp._h, _ptr_array(src_bufs, len(src_bufs)),
                                                        _ptr_array(dst_bufs, len(dst_bufs)), scratch,
                                                        scratch_bytes, stream))

    def plain_copy(self, dst, src, nbytes, stream=0):
        self._check(self._fn["plain_copy"](dst, src, nbytes, stream))

    def plain_read(self, src, nbytes, sink, stream=0):
        self._check(self._fn["plain_read"](src, nbytes, sink, stream))

    def plain_fill(self, dst, nbytes, stream=0):
        self._check(self._fn["plain_fill"](dst, nbytes, stream))

    def set_tile_bytes(self, n):
        self._check(self._fn["set_tile_bytes"](n))

    def set_option(self, option, value):
        self._check(self._fn["set_option"](option, value))


class Config:
    def __init__(self, lib, handle):
        self._lib, self._h = lib, handle

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib._fn["config_destroy"](self._h)
            self._h = None

    @property
    def world(self):
        v = C.c_int32()
        self._lib._check(self._lib._fn["config_world"](self._h, C.byref(v)))
        return v.value

    @property
    def num_tensors(self):
        v = C.c_int32()
        self._lib._check(self._lib._fn["config_num_tensors"](self._h, C.byref(v)))
        return v.value

    def num_buffers(self, rank):
        v = C.c_int32()
        self._lib._check(self._lib._fn["config_num_buffers"](self._h, rank, C.byref(v)))
        return v.value

    def buffer_bytes(self, rank, buf):
        v = C.c_uint64()
        self._lib._check(self._lib._fn["config_buffer_bytes"](self._h, rank, buf, C.byref(v)))
        return v.value

    @property
    def num_pieces(self):
        v = C.c_int64()
        self._lib._check(self._lib._fn["config_num_pieces"](self._h, C.byref(v)))
        return v.value

    def get_pieces(self):
        n = self.num_pieces
        out = np.zeros(n, dtype=PIECE_DTYPE)
        self._lib._check(self._lib._fn["config_get_pieces"](self._h, out.ctypes.data, n))
        return out


class Plan:
    def __init__(self, lib, handle):
        self._lib, self._h = lib, handle

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib._fn["plan_destroy"](self._h)
            self._h = None

    def pair_bytes(self, src_rank, dst_rank):
        v = C.c_uint64()
        self._lib._check(self._lib._fn["plan_pair_bytes"](self._h, src_rank, dst_rank, C.byref(v)))
        return v.value

    def peer_bytes(self, rank, peer):
        s, r = C.c_uint64(), C.c_uint64()
        self._lib._check(self._lib._fn["plan_peer_bytes"](self._h, rank, peer, C.byref(s), C.byref(r)))
        return s.value, r.value

    def buffer_bytes(self, rank):
        v = [C.c_uint64() for _ in range(5)]
        self._lib._check(self._lib._fn["plan_buffer_bytes"](self._h, rank, *[C.byref(x) for x in v]))
        return dict(zip(("send_total", "recv_total", "retain_total", "scratch_needed", "recv_offset"),
                        [x.value for x in v]))

    def peer_segment(self, src_rank, dst_rank):
        v = [C.c_uint64() for _ in range(3)]
        self._lib._check(self._lib._fn["plan_peer_segment"](self._h, src_rank, dst_rank, *[C.byref(x) for x in v]))
        return dict(zip(("send_off", "recv_off", "bytes"), [x.value for x in v]))

    @property
    def num_boxes(self):
        v = C.c_int64()
        self._lib._check(self._lib._fn["plan_num_boxes"](self._h, C.byref(v)))
        return v.value

    def get_boxes(self):
        n = self.num_boxes
        out = np.zeros(n, dtype=BOX_DTYPE)
        self._lib._check(self._lib._fn["plan_get_boxes"](self._h, out.ctypes.data, n))
        return out

    def classify_collectives(self, src_config, stream=0):
        """int32 array [num_tensors*4]: COLL code per (tensor, kind)."""
        n = src_config.num_tensors * 4
        out = np.zeros(n, dtype=np.int32)
        self._lib._check(self._lib._fn["plan_classify_collectives"](
            self._h, src_config._h, stream, out.ctypes.data_as(C.POINTER(C.c_int32)), n))
        return out

    def stats(self):
        st = PlanStats()
        self._lib._check(self._lib._fn["plan_stats"](self._h, C.byref(st)))
        return {n: getattr(st, n) for n, _ in PlanStats._fields_}


class StagePlan:
    def __init__(self, lib, handle, plan):
        self._lib, self._h, self._plan = lib, handle, plan   # keeps the plan alive

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib._fn["stage_plan_destroy"](self._h)
            self._h = None

    def info(self):
        a, b, c = C.c_int32(), C.c_int32(), C.c_uint64()
        self._lib._check(self._lib._fn["stage_info"](self._h, C.byref(a), C.byref(b), C.byref(c)))
        return dict(num_steps=a.value, num_stages=b.value, scratch_needed=c.value)

    def steps(self):
        n = self.info()["num_steps"] + 1
        st = (C.c_int32 * n)()
        cost = (C.c_uint64 * n)()
        self._lib._check(self._lib._fn["stage_steps"](self._h, st, cost, n))
        return list(st), list(cost)

"""ctypes front end of the CPU oracle (oracle/vps_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It never touches the HIP library.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

NBUF = 8
KIND_BYTES = (2, 4, 4, 4)


class _Model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("family", "layers", "hidden", "q_heads", "kv_heads",
                                         "head_dim", "ffn", "vocab", "experts", "expert_ffn")]


class _Parallel(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tp", "pp", "dp", "ep", "zero", "gpus_per_node",
                                         "qkv_layout", "expert_layout", "flat_order", "ep_placement")]


_lib = None


def lib():
    global _lib
    if _lib is not None:
        return _lib
    # ORACLE_LIB lets the mutation test of the pins load a deliberately broken build
    path = os.environ.get("ORACLE_LIB") or _build.build()
    L = C.CDLL(path)
    vp, i32, u64, u32, i64 = C.c_void_p, C.c_int32, C.c_uint64, C.c_uint32, C.c_int64
    pi32, pu64, pi64 = C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.POINTER(C.c_int64)
    L.orc_config_create.restype = vp
    L.orc_config_create.argtypes = [C.POINTER(_Model), C.POINTER(_Parallel), C.c_char_p, C.c_int]
    L.orc_config_destroy.argtypes = [vp]
    L.orc_world.restype = i32
    L.orc_world.argtypes = [vp]
    L.orc_num_tensors.restype = i32
    L.orc_num_tensors.argtypes = [vp]
    L.orc_tensor_info.argtypes = [vp, i32, pi32, pi32]
    L.orc_tensor_numel.restype = u64
    L.orc_tensor_numel.argtypes = [vp, i32]
    L.orc_total_params.restype = u64
    L.orc_total_params.argtypes = [vp]
    L.orc_rank_coords.argtypes = [vp, i32, pi32]
    L.orc_buffer_elems.restype = u64
    L.orc_buffer_elems.argtypes = [vp, i32, i32]
    L.orc_payload_elems.restype = u64
    L.orc_payload_elems.argtypes = [vp, i32, i32]
    L.orc_coord.restype = C.c_int
    L.orc_coord.argtypes = [vp, i32, i32, u64, pi32, pi32]
    L.orc_owners.restype = C.c_int
    L.orc_owners.argtypes = [vp, i32, i32, pi32, C.c_int, pi32, pi32, pu64]
    L.orc_linear.restype = u64
    L.orc_linear.argtypes = [vp, i32, pi32]
    L.orc_select_source.restype = C.c_int
    L.orc_select_source.argtypes = [vp, vp, i32, i32, i32, pi32, pi32, pi32, pu64]
    L.orc_fill.restype = C.c_int
    L.orc_fill.argtypes = [vp, i32, i32, u64, u64, u64, u64, vp, u32]
    L.orc_expected.restype = C.c_int
    L.orc_expected.argtypes = [vp, vp, i32, i32, u64, u64, u64, u64, vp, u32]
    L.orc_transition.restype = C.c_int
    L.orc_transition.argtypes = [vp, vp, i32, i32, C.POINTER(vp), u64, u64, vp]
    L.orc_route_bytes.restype = C.c_int
    L.orc_route_bytes.argtypes = [vp, vp, i32, u32, pu64]
    L.orc_send_bytes.restype = C.c_int
    L.orc_send_bytes.argtypes = [vp, vp, i32, u32, pu64]
    L.orc_check_boxes.restype = i64
    L.orc_check_boxes.argtypes = [vp, vp, pi32, pi64, i64, i32, pi64]
    L.orc_piece_key.restype = C.c_int
    L.orc_piece_key.argtypes = [vp, i32, i32, u64, pi64]
    L.orc_recv_payload.restype = i64
    L.orc_recv_payload.argtypes = [vp, vp, i32, C.c_int, u64, u64, C.c_uint8, vp, u64, pu64]
    L.orc_num_threads.restype = C.c_int
    L.orc_set_num_threads.argtypes = [C.c_int]
    L.orc_set_num_threads.restype = None
    _lib = L
    return L


def kind_dtype(buf):
    return np.uint16 if buf % 4 == 0 else np.uint32


class OracleError(ValueError):
    pass


class Config:
    """One parallel configuration of one model (the map F_P of Section 4.1)."""

    def __init__(self, model, parallel):
        self.model = dict(model)
        self.parallel = dict(parallel)
        m = _Model(**{k: int(v) for k, v in model.items()})
        p = _Parallel(**{k: int(v) for k, v in parallel.items()})
        err = C.create_string_buffer(256)
        self._h = lib().orc_config_create(C.byref(m), C.byref(p), err, 256)
        if not self._h:
            raise OracleError(err.value.decode())

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.orc_config_destroy(self._h)
            self._h = None

    # ---- scalars
    @property
    def world(self):
        return lib().orc_world(self._h)

    @property
    def num_tensors(self):
        return lib().orc_num_tensors(self._h)

    @property
    def total_params(self):
        return lib().orc_total_params(self._h)

    def tensor_info(self, t):
        shape = (C.c_int32 * 4)()
        info = (C.c_int32 * 4)()
        lib().orc_tensor_info(self._h, t, shape, info)
        return dict(shape=tuple(shape), tp_axis=info[0], group=info[1], layer=info[2], expert=info[3])

    def rank_coords(self, rank):
        o = (C.c_int32 * 6)()
        lib().orc_rank_coords(self._h, rank, o)
        return dict(tp=o[0], ddp=o[1], pp=o[2], ep=o[3], edp=o[4], etp=o[5])

    def buffer_elems(self, rank, buf):
        return lib().orc_buffer_elems(self._h, rank, buf)

    def payload_elems(self, rank, buf):
        return lib().orc_payload_elems(self._h, rank, buf)

    # ---- per-element maps
    def coord(self, rank, buf, off):
        t = C.c_int32()
        cd = (C.c_int32 * 4)()
        r = lib().orc_coord(self._h, rank, buf, off, C.byref(t), cd)
        if r < 0:
            raise IndexError("offset outside buffer")
        return (t.value, tuple(cd)) if r == 1 else None

    def owners(self, kind, tensor, coord, max_owners=4096):
        cd = (C.c_int32 * 4)(*coord)
        r = (C.c_int32 * max_owners)()
        b = (C.c_int32 * max_owners)()
        o = (C.c_uint64 * max_owners)()
        n = lib().orc_owners(self._h, kind, tensor, cd, max_owners, r, b, o)
        return [(r[k], b[k], o[k]) for k in range(n)]

    def piece_key(self, rank, buf, off):
        """(storage block, level, parent unit) of the piece that holds a stored element, None for padding."""
        o = (C.c_int64 * 3)()
        r = lib().orc_piece_key(self._h, rank, buf, off, o)
        if r < 0:
            raise IndexError("offset outside buffer or element without a piece")
        return tuple(o) if r == 1 else None

    def linear(self, tensor, coord):
        cd = (C.c_int32 * 4)(*coord)
        return lib().orc_linear(self._h, tensor, cd)

    # ---- bulk
    def fill(self, rank, buf, seed, rank_salt=0, off0=0, n=None, pad_word=0):
        if n is None:
            n = self.buffer_elems(rank, buf) - off0
        out = np.empty(int(n), dtype=kind_dtype(buf))
        rc = lib().orc_fill(self._h, rank, buf, seed, rank_salt, off0, n, out.ctypes.data, pad_word)
        if rc:
            raise IndexError("fill range outside buffer")
        return out


def select_source(a, b, j, kind, tensor, coord):
    cd = (C.c_int32 * 4)(*coord)
    r, bf, of = C.c_int32(), C.c_int32(), C.c_uint64()
    ok = lib().orc_select_source(a._h, b._h, j, kind, tensor, cd, C.byref(r), C.byref(bf), C.byref(of))
    if not ok:
        raise OracleError("no owner for element")
    return r.value, bf.value, of.value


def expected(a, b, j, buf, seed, rank_salt=0, off0=0, n=None, pad_word=0):
    if n is None:
        n = b.buffer_elems(j, buf) - off0
    out = np.empty(int(n), dtype=kind_dtype(buf))
    rc = lib().orc_expected(a._h, b._h, j, buf, seed, rank_salt, off0, n, out.ctypes.data, pad_word)
    if rc:
        raise OracleError("expected(): bad range or element without owner")
    return out


def transition(a, b, j, buf, src_bufs, dst, off0=0):
    """dst[k] = chosen source element for offsets off0+k.  src_bufs: dict (rank, buf) -> ndarray."""
    wa = a.world
    ptrs = (C.c_void_p * (wa * NBUF))()
    for (r, bf), arr in src_bufs.items():
        assert arr.dtype == kind_dtype(bf) and arr.flags.c_contiguous
        ptrs[r * NBUF + bf] = arr.ctypes.data
    assert dst.dtype == kind_dtype(buf) and dst.flags.c_contiguous
    rc = lib().orc_transition(a._h, b._h, j, buf, ptrs, off0, dst.size, dst.ctypes.data)
    if rc:
        raise OracleError("transition(): missing source buffer or bad range")
    return dst


def recv_payload(a, b, j, seed, rank_salt=0, through=False, pad_byte=0xA5):
    """The receive buffer of destination rank j as its sources must have packed it (uint8 array)
    and seg_off[world_A + 1]: segment of source i = bytes [seg_off[i], seg_off[i + 1])."""
    cap = sum(b.buffer_elems(j, buf) * KIND_BYTES[buf % 4] + 16 * 0 for buf in range(NBUF))
    cap = cap + 16 * (1 << 16)   # room for the alignment pad of up to 65536 boxes
    seg = np.zeros(a.world + 1, dtype=np.uint64)
    while True:
        out = np.empty(int(cap), dtype=np.uint8)
        n = lib().orc_recv_payload(a._h, b._h, j, int(bool(through)), seed, rank_salt, pad_byte, out.ctypes.data,
                                   cap, seg.ctypes.data_as(C.POINTER(C.c_uint64)))
        if n == -3:
            cap *= 2
            continue
        if n < 0:
            raise OracleError(f"recv_payload failed ({n})")
        return out[:n].copy(), seg


def route_bytes(a, b, j, buf_mask=0xFF):
    out = np.zeros(a.world, dtype=np.uint64)
    rc = lib().orc_route_bytes(a._h, b._h, j, buf_mask, out.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc:
        raise OracleError("route_bytes failed")
    return out


def send_bytes(a, b, i, buf_mask=0xFF):
    out = np.zeros(b.world, dtype=np.uint64)
    rc = lib().orc_send_bytes(a._h, b._h, i, buf_mask, out.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc:
        raise OracleError("send_bytes failed")
    return out


def check_boxes(a, b, ints, offs, samples=0):
    """ints: (n,16) int32, offs: (n,10) int64 (layout in vps_oracle.h). Returns (violations, first_bad)."""
    ints = np.ascontiguousarray(ints, dtype=np.int32)
    offs = np.ascontiguousarray(offs, dtype=np.int64)
    n = ints.shape[0]
    assert ints.shape == (n, 16) and offs.shape == (n, 10)
    first = C.c_int64(-1)
    bad = lib().orc_check_boxes(a._h, b._h, ints.ctypes.data_as(C.POINTER(C.c_int32)),
                                offs.ctypes.data_as(C.POINTER(C.c_int64)), n, samples, C.byref(first))
    return bad, first.value


def num_threads():
    return lib().orc_num_threads()


def set_num_threads(n):
    lib().orc_set_num_threads(int(n))

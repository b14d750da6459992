"""Shared parity procedures: drive the C ABI on seeded inputs and compare with the CPU oracle.

The same procedures run against the HIP library on device memory (``-m gpu`` tests) and
against the CPU build of the library's per-item code on host memory (tests/hostcheck).
Inputs always come from the oracle (``Config.fill``) or from the seeded pattern generator;
expected values always come from the oracle.
"""
import ctypes as C

import numpy as np

import oracle
from datagen import boxfill, pattern

SENTINEL = 0xA5
PLAN_THROUGH_BUFFERS = 2   # vps.h
SENT16, SENT32 = 0xA5A5, 0xA5A5A5A5


# ----------------------------------------------------------------------------- memory providers

class HostMem:
    """numpy-backed 'device' memory for the CPU build."""

    def __init__(self, lib=None):
        self.lib = lib
        self.live = []

    def alloc(self, nbytes, fill=SENTINEL):
        a = np.full(max(int(nbytes), 16) + 16, fill, dtype=np.uint8)
        off = (-a.ctypes.data) % 16
        v = a[off:off + max(int(nbytes), 0)]
        self.live.append((a, v))
        return v

    def ptr(self, v):
        return v.ctypes.data if v.size else 0

    def upload(self, v, host_bytes):
        v[:] = np.frombuffer(host_bytes, dtype=np.uint8) if not isinstance(host_bytes, np.ndarray) else host_bytes.view(np.uint8).ravel()

    def download(self, v):
        return v.copy()

    def copy(self, dst, doff, src, soff, n):
        dst[doff:doff + n] = src[soff:soff + n]

    def sync(self):
        pass

    def equal(self, x, y):
        return bool(np.array_equal(x, y))

    def all_bytes(self, x, value):
        return bool((x == value).all())

    def register_bounds(self):
        if self.lib is None:
            return
        arr = (C.c_void_p * (2 * len(self.live)))()
        for i, (_, v) in enumerate(self.live):
            arr[2 * i] = v.ctypes.data
            arr[2 * i + 1] = v.ctypes.data + v.size
        self.lib._dll.vpsh_set_bounds(arr, len(self.live))

    def violations(self):
        if self.lib is None:
            return 0
        self.lib._dll.vpsh_bounds_violations.restype = C.c_long
        return self.lib._dll.vpsh_bounds_violations()


class GpuMem:
    """torch-backed device memory (torch is only the allocator and the copy engine here).
    Every allocation sits between two guard zones; violations() counts guard bytes that a kernel
    overwrote (the CPU build checks every access instead)."""
    GUARD = 4096
    GUARD_BYTE = 0x5A

    def __init__(self):
        import torch
        self.torch = torch
        self.dev = torch.device("cuda:0")
        self.guards = []

    def alloc(self, nbytes, fill=SENTINEL):
        n = max(int(nbytes), 0)
        if n == 0:
            return self.torch.empty(0, dtype=self.torch.uint8, device=self.dev)
        whole = self.torch.empty(n + 2 * self.GUARD, dtype=self.torch.uint8, device=self.dev)
        whole[:self.GUARD].fill_(self.GUARD_BYTE)
        whole[self.GUARD + n:].fill_(self.GUARD_BYTE)
        t = whole[self.GUARD:self.GUARD + n]
        t.fill_(fill)
        self.guards.append((whole, n))
        return t

    def ptr(self, v):
        return v.data_ptr() if v.numel() else 0

    def upload(self, v, host):
        h = host.view(np.uint8).ravel() if isinstance(host, np.ndarray) else np.frombuffer(host, dtype=np.uint8)
        if h.size:
            v.copy_(self.torch.from_numpy(np.ascontiguousarray(h)))

    def download(self, v):
        return v.cpu().numpy()

    def copy(self, dst, doff, src, soff, n):
        if n:
            dst[doff:doff + n].copy_(src[soff:soff + n])

    def sync(self):
        self.torch.cuda.synchronize()

    def equal(self, x, y):
        return bool(self.torch.equal(x, y))

    def all_bytes(self, x, value):
        return bool((x == value).all()) if x.numel() else True

    def register_bounds(self):
        pass

    def violations(self):
        self.torch.cuda.synchronize()
        bad = 0
        for whole, n in self.guards:
            bad += int((whole[:self.GUARD] != self.GUARD_BYTE).sum()) + int((whole[self.GUARD + n:] != self.GUARD_BYTE).sum())
        return bad


# ----------------------------------------------------------------------------- helpers

def kind_dtype(buf):
    return np.uint16 if buf % 4 == 0 else np.uint32


def check_config_against_oracle(cfg, orc):
    assert cfg.world == orc.world
    assert cfg.num_tensors == orc.num_tensors
    for r in range(orc.world):
        for b in range(8):
            assert cfg.buffer_bytes(r, b) == orc.buffer_elems(r, b) * oracle.KIND_BYTES[b % 4], (r, b)


def boxes_to_oracle_arrays(boxes):
    n = boxes.shape[0]
    ints = np.zeros((n, 16), dtype=np.int32)
    offs = np.zeros((n, 10), dtype=np.int64)
    ints[:, 0] = boxes["kind"]; ints[:, 1] = boxes["tensor"]
    ints[:, 2] = boxes["src_rank"]; ints[:, 3] = boxes["dst_rank"]
    ints[:, 4] = boxes["src_buf"]; ints[:, 5] = boxes["dst_buf"]
    ints[:, 6:10] = boxes["lo"]; ints[:, 10:14] = boxes["ext"]
    offs[:, 0] = boxes["src_off"]; offs[:, 1] = boxes["dst_off"]
    offs[:, 2:6] = boxes["src_stride"]; offs[:, 6:10] = boxes["dst_stride"]
    return ints, offs


def box_volume(b):
    return int(np.prod(b["ext"].astype(np.int64)))


def box_linear_indices(b, shape):
    """Global row-major linear indices of the elements of a box, in the box's row-major order."""
    lo, ext = b["lo"].astype(np.int64), b["ext"].astype(np.int64)
    idx = np.zeros(tuple(ext), dtype=np.int64)
    mult = 1
    for ax in (3, 2, 1, 0):
        shp = [1, 1, 1, 1]
        shp[ax] = int(ext[ax])
        idx = idx + (np.arange(lo[ax], lo[ax] + ext[ax], dtype=np.int64) * mult).reshape(shp)
        mult *= int(shape[ax])
    return idx.ravel()


def gather_box(buf_words, off, strides, ext):
    """Elements of a strided box of a local buffer (numpy words), row-major in global axes."""
    ext = [int(e) for e in ext]
    strides = [int(s) for s in strides]
    idx = np.full((1, 1, 1, 1), int(off), dtype=np.int64)
    for ax in range(4):
        shp = [1, 1, 1, 1]
        shp[ax] = ext[ax]
        idx = idx + (np.arange(ext[ax], dtype=np.int64) * strides[ax]).reshape(shp)
    return buf_words[idx.ravel()]


def check_stats(plan, boxes, planned_rank, through=False):
    """The plan's box counts against their definitions over the box list: a box is retained when
    its source rank is its destination rank (unless everything goes through the buffers); any
    other box counts as sent when its source rank is resident on this GPU (the planned rank, or
    every rank of an all-ranks plan) and as received when its destination rank is."""
    st = plan.stats()
    same = boxes["src_rank"] == boxes["dst_rank"]
    retained = same & (not through)
    src_res = np.ones(len(boxes), bool) if planned_rank < 0 else boxes["src_rank"] == planned_rank
    dst_res = np.ones(len(boxes), bool) if planned_rank < 0 else boxes["dst_rank"] == planned_rank
    want = dict(num_boxes=len(boxes), num_retain_boxes=int(retained.sum()), num_send_boxes=int((~retained & src_res).sum()),
                num_recv_boxes=int((~retained & dst_res).sum()))
    got = {k: int(st[k]) for k in want}
    assert got == want, f"plan statistics {got}, the boxes give {want}"


def validate_boxes(a, b, boxes, planned_rank, samples=0, through=False, plan=None):
    """Per-element validation of the plan by the oracle, plus exact coverage counts (and the
    plan's statistics when the plan is given)."""
    if plan is not None:
        check_stats(plan, boxes, planned_rank, through)
    ints, offs = boxes_to_oracle_arrays(boxes)
    bad, first = oracle.check_boxes(a, b, ints, offs, samples=samples)
    assert bad == 0, f"{bad} element violations, first bad box {first}: {boxes[first] if first >= 0 else None}"
    vols = np.prod(boxes["ext"].astype(np.int64), axis=1)
    es = np.where(boxes["kind"] == 0, 2, 4)
    ranks = range(b.world) if planned_rank < 0 else [planned_rank] if planned_rank < b.world else []
    for j in ranks:
        sel = boxes["dst_rank"] == j
        got = int((vols[sel] * es[sel]).sum())
        want = sum(b.payload_elems(j, buf) * oracle.KIND_BYTES[buf % 4] for buf in range(8))
        assert got == want, f"dst rank {j}: boxes cover {got} bytes, payload is {want}"
    # inside a peer buffer boxes are 16-byte aligned, disjoint and dense in their order
    for key, pos_key in (("src_rank", "send_pos"), ("dst_rank", "recv_pos")):
        travels = (boxes["src_rank"] != boxes["dst_rank"]) | through
        if not through:
            stay = boxes[boxes["src_rank"] == boxes["dst_rank"]]
            assert (stay[pos_key] == np.uint64(2**64 - 1)).all(), "a retained box has a buffer position"
        moving = boxes[travels & (boxes[pos_key] != np.uint64(2**64 - 1))]
        for r in np.unique(moving[key]):
            bx = moving[moving[key] == r]
            order = np.argsort(bx[pos_key], kind="stable")
            pos = bx[pos_key][order].astype(np.int64)
            size = ((np.prod(bx["ext"].astype(np.int64), axis=1) * np.where(bx["kind"] == 0, 2, 4))[order] + 15) // 16 * 16
            assert (pos % 16 == 0).all()
            assert pos[0] == 0 and (pos[1:] == pos[:-1] + size[:-1]).all()
            peer = bx["dst_rank" if key == "src_rank" else "src_rank"][order]
            assert (np.diff(peer) >= 0).all(), "peer segments must ascend"
            # the documented order inside a segment: kinds 1, 2, 3, 0; tensor id; lo corner row-major
            lin = np.zeros(len(bx), dtype=np.int64)
            for i, o in enumerate(order):
                shp = a.tensor_info(int(bx["tensor"][o]))["shape"]
                lo = [int(v) for v in bx["lo"][o]]
                lin[i] = ((lo[0] * shp[1] + lo[1]) * shp[2] + lo[2]) * shp[3] + lo[3]
            keys = list(zip(peer.tolist(), ((bx["kind"][order] + 3) & 3).tolist(), bx["tensor"][order].tolist(), lin.tolist()))
            assert keys == sorted(keys), "boxes of a peer segment are not in the documented order"


# ----------------------------------------------------------------------------- all ranks resident

def run_all_ranks(lib, mem, model, pa, pb, seed, rank_salt=0x9E37, check_send_payload=True, through=False):
    """Every virtual rank resident: apply_transition(rank=-1), then per-rank pack / exchange /
    unpack; dst buffers, per-pair byte counts and send payloads against the oracle."""
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    check_config_against_oracle(ca, a)
    check_config_against_oracle(cb, b)
    plan = lib.plan_intersections_ex(ca, cb, -1, PLAN_THROUGH_BUFFERS) if through else lib.plan_intersections(ca, cb, -1)
    boxes = plan.get_boxes()
    validate_boxes(a, b, boxes, -1, through=through, plan=plan)
    travels = (boxes["src_rank"] != boxes["dst_rank"]) | through

    src_host = {(r, buf): a.fill(r, buf, seed, rank_salt, pad_word=0x3C3C3C3C) for r in range(a.world) for buf in range(8)}
    src = {k: mem.alloc(v.nbytes) for k, v in src_host.items()}
    for k, v in src_host.items():
        mem.upload(src[k], v)
    want = {(j, buf): oracle.expected(a, b, j, buf, seed, rank_salt, pad_word=SENT32) for j in range(b.world) for buf in range(8)}

    # byte counts
    for j in range(b.world):
        rb = oracle.route_bytes(a, b, j)
        for i in range(a.world):
            assert plan.pair_bytes(i, j) == rb[i], (i, j)

    def fresh_dst():
        return {k: mem.alloc(v.nbytes) for k, v in want.items()}

    def compare(dst, tag):
        for k, v in want.items():
            got = mem.download(dst[k]).view(v.dtype)
            if not np.array_equal(got, v):
                bad = np.nonzero(got != v)[0]
                raise AssertionError(f"{tag}: dst {k} differs at {bad.size} of {v.size} elements, first offsets {bad[:5]}")

    # (1) one call for everything
    info = plan.buffer_bytes(-1)
    kept = sum(plan.pair_bytes(q, q) for q in range(min(a.world, b.world)))    # checked against the oracle above
    assert info["retain_total"] == (0 if through else kept)
    if through:
        assert info["retain_total"] == 0
        assert info["send_total"] >= sum(b.payload_elems(j, buf) * oracle.KIND_BYTES[buf % 4]
                                         for j in range(b.world) for buf in range(8))
    scratch = mem.alloc(info["scratch_needed"])
    dst = fresh_dst()
    mem.register_bounds()
    lib.apply_transition(plan, -1, [mem.ptr(src[(r, buf)]) for r in range(a.world) for buf in range(8)],
                         [mem.ptr(dst[(j, buf)]) for j in range(b.world) for buf in range(8)],
                         mem.ptr(scratch), info["scratch_needed"])
    mem.sync()
    assert mem.violations() == 0
    compare(dst, "apply_transition(all)")

    # (1b) and back again: the destination state just verified is the source of the reverse
    # transition; expected values from the oracle's element-by-element copy of that state
    rplan = lib.plan_intersections_ex(cb, ca, -1, PLAN_THROUGH_BUFFERS) if through else lib.plan_intersections(cb, ca, -1)
    rinfo = rplan.buffer_bytes(-1)
    rscratch = mem.alloc(rinfo["scratch_needed"])
    back = {k: mem.alloc(v.nbytes) for k, v in src_host.items()}
    mem.register_bounds()
    lib.apply_transition(rplan, -1, [mem.ptr(dst[(j, buf)]) for j in range(b.world) for buf in range(8)],
                         [mem.ptr(back[(r, buf)]) for r in range(a.world) for buf in range(8)],
                         mem.ptr(rscratch), rinfo["scratch_needed"])
    mem.sync()
    assert mem.violations() == 0
    for (r, buf), h in src_host.items():
        exp = np.full(h.size, SENT16 if buf % 4 == 0 else SENT32, dtype=h.dtype)
        oracle.transition(b, a, r, buf, want, exp)
        got = mem.download(back[(r, buf)]).view(h.dtype)
        assert np.array_equal(got, exp), ("reverse transition", r, buf)
    del back, rscratch, rplan

    # (2) per rank: pack, exchange segment by segment, unpack
    sends = {}
    for i in range(a.world):
        bi = plan.buffer_bytes(i)
        sends[i] = mem.alloc(bi["send_total"])
    recvs = {j: mem.alloc(plan.buffer_bytes(j)["recv_total"]) for j in range(b.world)}
    dst2 = fresh_dst()
    mem.register_bounds()
    for i in range(a.world):
        lib.pack(plan, i, [mem.ptr(src[(i, buf)]) for buf in range(8)], mem.ptr(sends[i]))
    mem.sync()
    moved = 0
    for i in range(a.world):
        for j in range(b.world):
            seg = plan.peer_segment(i, j)
            if seg["bytes"]:
                mem.copy(recvs[j], seg["recv_off"], sends[i], seg["send_off"], seg["bytes"])
                moved += seg["bytes"]
    for j in range(b.world):
        lib.unpack(plan, j, mem.ptr(recvs[j]), [mem.ptr(dst2[(j, buf)]) for buf in range(8)])
    mem.sync()
    assert mem.violations() == 0
    # retained data does not travel: dst2 is complete only after the retain copies, which
    # pack/unpack do not perform; compare the received part box by box instead
    for j in range(b.world):
        got = {buf: mem.download(dst2[(j, buf)]).view(kind_dtype(buf)) for buf in range(8)}
        for bx in boxes[(boxes["dst_rank"] == j) & travels]:
            buf = int(bx["dst_buf"])
            g = gather_box(got[buf], bx["dst_off"], bx["dst_stride"], bx["ext"])
            w = gather_box(want[(j, buf)], bx["dst_off"], bx["dst_stride"], bx["ext"])
            assert np.array_equal(g, w), ("unpack", j, bx)
        for bx in boxes[(boxes["dst_rank"] == j) & ~travels]:
            buf = int(bx["dst_buf"])
            g = gather_box(got[buf], bx["dst_off"], bx["dst_stride"], bx["ext"])
            assert (g == (SENT16 if buf % 4 == 0 else SENT32)).all(), "unpack wrote a retained box"

    # (3) per-peer buffers against the oracle (Algorithm 1, PackData): every receive buffer as a
    # whole (unwritten pad bytes still hold the fill byte, which is the oracle's pad byte), every
    # segment of every send buffer, and the segment table
    if check_send_payload:
        send_host = {i: mem.download(sends[i]) for i in range(a.world)}
        for j in range(b.world):
            want_recv, seg = oracle.recv_payload(a, b, j, seed, rank_salt, through=through, pad_byte=SENTINEL)
            got_recv = mem.download(recvs[j])
            assert got_recv.size == want_recv.size, ("receive buffer size", j, got_recv.size, want_recv.size)
            assert np.array_equal(got_recv, want_recv), ("receive buffer", j)
            for i in range(a.world):
                lo, hi = int(seg[i]), int(seg[i + 1])
                sg = plan.peer_segment(i, j)
                assert sg["bytes"] == hi - lo, ("segment size", i, j)
                if hi > lo:
                    assert sg["recv_off"] == lo
                    assert np.array_equal(send_host[i][sg["send_off"]:sg["send_off"] + hi - lo], want_recv[lo:hi]), ("send segment", i, j)
    return dict(boxes=len(boxes), moved=moved, stats=plan.stats())


# ----------------------------------------------------------------------------- one rank resident

def synth_recv_buffer(a, boxes, rank, nbytes, seed, rank_salt):
    """What the peers would have packed for `rank`: for every incoming box the pattern words of
    its elements (row-major in global axes) at the box's position in the receive buffer."""
    out = np.full(int(nbytes), SENTINEL, dtype=np.uint8)
    for bx in boxes[(boxes["dst_rank"] == rank) & (boxes["src_rank"] != rank)]:
        t, kind = int(bx["tensor"]), int(bx["kind"])
        sd = pattern.seed_for_rank(seed, rank_salt, int(bx["src_rank"]))
        pos, n = int(bx["recv_pos"]), box_volume(bx)
        w = out[pos:pos + n * (2 if kind == 0 else 4)].view(np.uint16 if kind == 0 else np.uint32)
        boxfill.fill_box(sd, kind, t, a.tensor_info(t)["shape"], bx["lo"], bx["ext"], w)
    return out


def run_single_rank(lib, mem, model, pa, pb, rank, seed, rank_salt=0x9E37, box_samples=0,
                    full_compare=True, chunk=1 << 24, check_bytes=True, through=False, send_payload_ranks=None):
    """One rank's share: retain + pack + unpack in one apply_transition call, peers' buffers
    synthesized from the seeded pattern."""
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    plan = lib.plan_intersections_ex(ca, cb, rank, PLAN_THROUGH_BUFFERS) if through else lib.plan_intersections(ca, cb, rank)
    boxes = plan.get_boxes()
    validate_boxes(a, b, boxes, rank, samples=box_samples, through=through, plan=plan)
    info = plan.buffer_bytes(rank)
    if through:
        assert info["retain_total"] == 0 and plan.stats()["num_retain_tiles"] == 0

    in_a, in_b = rank < a.world, rank < b.world
    src_host, src, dst = {}, {}, {}
    for buf in range(8):
        n = a.buffer_elems(rank, buf) if in_a else 0
        src_host[buf] = a.fill(rank, buf, seed, rank_salt, pad_word=0x3C3C3C3C) if n else np.zeros(0, kind_dtype(buf))
        src[buf] = mem.alloc(src_host[buf].nbytes)
        mem.upload(src[buf], src_host[buf])
        dst[buf] = mem.alloc((b.buffer_elems(rank, buf) if in_b else 0) * oracle.KIND_BYTES[buf % 4])
    scratch = mem.alloc(info["scratch_needed"])
    # what the peers would have packed for this rank: from the oracle, not from the plan
    if in_b:
        recv, recv_seg = oracle.recv_payload(a, b, rank, seed, rank_salt, through=through, pad_byte=SENTINEL)
    else:
        recv, recv_seg = np.zeros(0, np.uint8), np.zeros(a.world + 1, np.uint64)
    assert recv.size == info["recv_total"], ("receive buffer size", recv.size, info["recv_total"])
    if through and rank < a.world:
        # the rank's own segment is read out of the send region, where its pack launch writes it
        lo, hi = int(recv_seg[rank]), int(recv_seg[rank + 1])
        recv = recv.copy()
        recv[lo:hi] = SENTINEL
    if recv.size:
        mem.upload(scratch[info["recv_offset"]:info["recv_offset"] + recv.size], recv)
    mem.register_bounds()
    lib.apply_transition(plan, rank, [mem.ptr(src[buf]) for buf in range(8)],
                         [mem.ptr(dst[buf]) for buf in range(8)], mem.ptr(scratch), info["scratch_needed"])
    mem.sync()
    assert mem.violations() == 0

    # destination buffers against the oracle
    if in_b:
        for buf in range(8):
            n = b.buffer_elems(rank, buf)
            got = mem.download(dst[buf]).view(kind_dtype(buf))
            for o in range(0, n, chunk):
                m = min(chunk, n - o)
                want = oracle.expected(a, b, rank, buf, seed, rank_salt, off0=o, n=m, pad_word=SENT32)
                if not np.array_equal(got[o:o + m], want):
                    bad = np.nonzero(got[o:o + m] != want)[0]
                    raise AssertionError(f"dst buf {buf}: {bad.size} wrong elements from offset {o + bad[0]}")
    # byte counts seen from this rank (quadratic in the number of replicas: skipped for huge worlds)
    if not check_bytes:
        in_a = in_b = False
    nb = len(boxes)
    if in_b:
        rb = oracle.route_bytes(a, b, rank)
        for i in range(a.world):
            assert plan.pair_bytes(i, rank) == rb[i], (i, rank)
        own = int(rb[rank]) if rank < a.world else 0
        assert info["retain_total"] == (0 if through else own)
        incoming = int(rb.sum()) - (0 if through else own)
        assert incoming <= info["recv_total"] <= incoming + 16 * nb      # payload plus alignment pad
    if in_a:
        sbytes = oracle.send_bytes(a, b, rank)
        for j in range(b.world):
            assert plan.pair_bytes(rank, j) == sbytes[j], (rank, j)
        outgoing = int(sbytes.sum()) - (0 if through or rank >= b.world else int(sbytes[rank]))
        assert outgoing <= info["send_total"] <= outgoing + 16 * nb
    # send buffer against the oracle: the segment of every destination, in ascending order
    sb = mem.download(scratch)[:info["send_total"]]
    if rank < a.world and send_payload_ranks != 0:
        pos = 0
        dsts = range(b.world) if send_payload_ranks is None else send_payload_ranks
        for j in dsts:
            sg = plan.peer_segment(rank, j)
            if send_payload_ranks is None:
                assert sg["bytes"] == 0 or sg["send_off"] == pos, ("send segments must be dense and ascending", j)
                pos += sg["bytes"]
            if not sg["bytes"]:
                continue
            want, seg = oracle.recv_payload(a, b, j, seed, rank_salt, through=through, pad_byte=SENTINEL)
            lo, hi = int(seg[rank]), int(seg[rank + 1])
            assert sg["bytes"] == hi - lo, ("segment size", rank, j)
            assert np.array_equal(sb[sg["send_off"]:sg["send_off"] + hi - lo], want[lo:hi]), ("send segment", rank, j)
        if send_payload_ranks is None:
            assert pos == info["send_total"]
    return dict(boxes=len(boxes), info=info, stats=plan.stats())


# ----------------------------------------------------------------------------- full size

def check_send_buffer_on_device(mem, a, out_boxes, src, scratch, seed, pattern_budget):
    """Every element of every outgoing box against the send buffer, on the device: (1) the box as
    a strided view of the source buffer (which the oracle filled, element by element) must equal
    the bytes at the box's position in the send buffer; (2) those bytes must also be the pattern
    words of the box's global coordinates (generated on the host, box by box, up to
    pattern_budget bytes), which ties the source addressing of a box to the coordinates it claims."""
    torch = mem.torch
    dts = {2: torch.int16, 4: torch.int32}
    gathered = patterned = 0
    spent = 0
    for bx in out_boxes:
        kind, buf = int(bx["kind"]), int(bx["src_buf"])
        es = 2 if kind == 0 else 4
        ext = [int(e) for e in bx["ext"]]
        vol = ext[0] * ext[1] * ext[2] * ext[3]
        pos = int(bx["send_pos"])
        words = src[buf].view(dts[es])
        got = scratch[pos:pos + vol * es].view(dts[es])
        step = max(1, (1 << 28) // max(1, ext[1] * ext[2] * ext[3]))     # slabs of the outer axis, 256 Mi elements at most
        for o in range(0, ext[0], step):
            m = min(step, ext[0] - o)
            view = torch.as_strided(words, (m, ext[1], ext[2], ext[3]), tuple(int(v) for v in bx["src_stride"]),
                                    words.storage_offset() + int(bx["src_off"]) + o * int(bx["src_stride"][0]))
            inner = ext[1] * ext[2] * ext[3]
            assert torch.equal(view.reshape(-1), got[o * inner:(o + m) * inner]), ("send payload differs from the source box", bx, o)
        gathered += vol
        if spent + vol * es <= pattern_budget:
            want = np.empty(vol, dtype=np.uint16 if kind == 0 else np.uint32)
            t = int(bx["tensor"])
            boxfill.fill_box(seed, kind, t, a.tensor_info(t)["shape"], bx["lo"], bx["ext"], want)
            dev = torch.from_numpy(want.view(np.int16 if kind == 0 else np.int32)).to(got.device)
            assert torch.equal(dev, got), ("send payload is not the pattern of the box's coordinates", bx)
            patterned += vol
            spent += vol * es
            del dev, want
    return gathered, patterned


def check_cross_plan_segments(lib, model, pa, pb, pairs):
    """Two ranks plan on their own (single-rank plans): for every pair (i, j) the sender's plan and
    the receiver's plan must list the same boxes for the segment i -> j, at the same offsets
    inside the segment, and agree on its size: what i packs is what j expects to unpack."""
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    plans = {}

    def plan_of(r):
        if r not in plans:
            p = lib.plan_intersections(ca, cb, r)
            plans[r] = (p, p.get_boxes())
        return plans[r]

    checked = 0
    for i, j in pairs:
        if i == j:
            continue
        (pi, bi), (pj, bj) = plan_of(i), plan_of(j)
        si, sj = pi.peer_segment(i, j), pj.peer_segment(i, j)
        assert si["bytes"] == sj["bytes"], ("segment size seen by sender and receiver", i, j, si, sj)
        mine = bi[(bi["src_rank"] == i) & (bi["dst_rank"] == j)]
        theirs = bj[(bj["src_rank"] == i) & (bj["dst_rank"] == j)]
        assert len(mine) == len(theirs)
        if not len(mine):
            assert si["bytes"] == 0
            continue
        key = ["tensor", "kind", "lo", "ext", "src_buf", "dst_buf", "src_off", "dst_off"]
        om = np.argsort(mine["send_pos"], kind="stable")
        ot = np.argsort(theirs["recv_pos"], kind="stable")
        for k in key:
            assert np.array_equal(mine[k][om], theirs[k][ot]), ("box lists of the segment differ in " + k, i, j)
        assert np.array_equal(mine["send_pos"][om] - np.uint64(si["send_off"]), theirs["recv_pos"][ot] - np.uint64(sj["recv_off"])), \
            ("offsets inside the segment differ between sender and receiver", i, j)
        checked += len(mine)
    return checked


def _sample_chunks(n, chunk, fraction, edges, rng):
    """Chunk indices to verify: every chunk that holds a box edge, the first and last chunk, and
    a random fraction of the rest."""
    nchunks = -(-n // chunk)
    pick = set([0, nchunks - 1])
    for e in edges:
        if 0 <= e < n:
            pick.add(int(e) // chunk)
    pick.update(np.nonzero(rng.random(nchunks) < fraction)[0].tolist())
    return sorted(pick)


def run_single_rank_fullsize(lib, mem, model, pa, pb, rank, seed, fraction=0.05, chunk=1 << 20,
                             box_samples=32, pattern_budget=8 << 30, log=print, through=False):
    """One rank's share at full size, in the launch configuration the benchmark times.

    The source buffers are filled by the oracle (every element), the receive buffer with the
    pattern of the incoming boxes.  After one vps_apply_transition the destination buffers are
    compared with the oracle on 1 Mi-element chunks (all of them when fraction = 1: every chunk
    holding a box edge plus a random fraction otherwise), the padding must be untouched, every box
    is validated by the oracle on its corners and random interior points, and every element of
    every outgoing box is compared with the send buffer (see check_send_buffer_on_device).
    through = True plans with VPS_PLAN_THROUGH_BUFFERS: the whole share is packed and unpacked."""
    import time
    t0 = time.time()
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    plan = lib.plan_intersections_ex(ca, cb, rank, PLAN_THROUGH_BUFFERS) if through else lib.plan_intersections(ca, cb, rank)
    boxes = plan.get_boxes()
    validate_boxes(a, b, boxes, rank, samples=box_samples, through=through, plan=plan)
    info = plan.buffer_bytes(rank)
    log(f"  plan: {len(boxes)} boxes, send {info['send_total'] >> 20} MiB, recv {info['recv_total'] >> 20} MiB, "
        f"retain {info['retain_total'] >> 20} MiB ({time.time() - t0:.1f}s)")

    src_host, src, dst = {}, {}, {}
    for buf in range(8):
        n = a.buffer_elems(rank, buf) if rank < a.world else 0
        src_host[buf] = a.fill(rank, buf, seed, 0, pad_word=0x3C3C3C3C) if n else np.zeros(0, kind_dtype(buf))
        src[buf] = mem.alloc(src_host[buf].nbytes, fill=0)
        mem.upload(src[buf], src_host[buf])
        dst[buf] = mem.alloc((b.buffer_elems(rank, buf) if rank < b.world else 0) * oracle.KIND_BYTES[buf % 4])
    log(f"  source filled by the oracle and uploaded ({time.time() - t0:.1f}s)")
    scratch = mem.alloc(info["scratch_needed"])
    recv = synth_recv_buffer(a, boxes, rank, info["recv_total"], seed, 0)
    if recv.size:
        mem.upload(scratch[info["recv_offset"]:info["recv_offset"] + recv.size], recv)
    del recv
    log(f"  receive buffer synthesized ({time.time() - t0:.1f}s)")
    lib.apply_transition(plan, rank, [mem.ptr(src[buf]) for buf in range(8)],
                         [mem.ptr(dst[buf]) for buf in range(8)], mem.ptr(scratch), info["scratch_needed"])
    mem.sync()
    log(f"  transition done ({time.time() - t0:.1f}s)")

    rng = np.random.default_rng(seed & 0xFFFF)
    checked = 0
    for buf in range(8):
        n = b.buffer_elems(rank, buf) if rank < b.world else 0
        if not n:
            continue
        got = mem.download(dst[buf]).view(kind_dtype(buf))
        mine = boxes[(boxes["dst_rank"] == rank) & (boxes["dst_buf"] == buf)]
        edges = np.concatenate([mine["dst_off"], mine["dst_off"] - 1]) if len(mine) else np.zeros(0, np.int64)
        for c in _sample_chunks(n, chunk, fraction, edges, rng):
            o, m = c * chunk, min(chunk, n - c * chunk)
            want = b.fill(rank, buf, seed, 0, off0=o, n=m, pad_word=SENT32)
            if not np.array_equal(got[o:o + m], want):
                bad = np.nonzero(got[o:o + m] != want)[0]
                raise AssertionError(f"dst buf {buf}: {bad.size} wrong elements in chunk at {o}, first {o + bad[0]}")
            checked += m
        pay = b.payload_elems(rank, buf)
        sent = SENT16 if buf % 4 == 0 else SENT32
        assert (got[pay:] == sent).all(), f"padding of dst buf {buf} was written"
        del got
    log(f"  {checked} destination elements compared with the oracle ({time.time() - t0:.1f}s)")

    out_boxes = boxes[(boxes["src_rank"] == rank) & ((boxes["dst_rank"] != rank) | through)]
    n_gathered, n_pattern = check_send_buffer_on_device(mem, a, out_boxes, src, scratch, seed, pattern_budget)
    log(f"  send buffer: {n_gathered} elements of {len(out_boxes)} outgoing boxes equal the source data they name, "
        f"{n_pattern} of them also the pattern of their global coordinates ({time.time() - t0:.1f}s)")
    assert mem.violations() == 0, "a kernel wrote outside its buffers"
    return dict(boxes=len(boxes), info=info, checked=checked, stats=plan.stats())


def run_all_ranks_fullsize(lib, mem, model, pa, pb, seed, fraction=1.0, chunk=1 << 22, box_samples=16, log=print,
                           round_trip=True, staged_budget=None):
    """Every virtual rank resident at full size: one vps_apply_transition(rank=-1) call, all
    destination buffers against the oracle (layout-B fill of the same coordinate hash).  With
    staged_budget the transition then runs once more through vps_stage_exchange and
    vps_apply_transition_staged under that per-rank budget, into fresh destination buffers that
    must equal the ones just compared with the oracle byte for byte."""
    import time
    t0 = time.time()
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    check_config_against_oracle(ca, a)
    check_config_against_oracle(cb, b)
    plan = lib.plan_intersections(ca, cb, -1)
    boxes = plan.get_boxes()
    validate_boxes(a, b, boxes, -1, samples=box_samples, plan=plan)
    info = plan.buffer_bytes(-1)
    log(f"  plan: {len(boxes)} boxes, exchanged {info['send_total'] >> 20} MiB, retained {info['retain_total'] >> 20} MiB ({time.time() - t0:.1f}s)")
    src, dst = {}, {}
    for r in range(a.world):
        for buf in range(8):
            h = a.fill(r, buf, seed, 0, pad_word=0x3C3C3C3C) if a.buffer_elems(r, buf) else np.zeros(0, kind_dtype(buf))
            src[(r, buf)] = mem.alloc(h.nbytes, fill=0)
            mem.upload(src[(r, buf)], h)
    for j in range(b.world):
        for buf in range(8):
            dst[(j, buf)] = mem.alloc(b.buffer_elems(j, buf) * oracle.KIND_BYTES[buf % 4])
    scratch = mem.alloc(info["scratch_needed"])
    log(f"  sources filled by the oracle and uploaded ({time.time() - t0:.1f}s)")
    lib.apply_transition(plan, -1, [mem.ptr(src[(r, buf)]) for r in range(a.world) for buf in range(8)],
                         [mem.ptr(dst[(j, buf)]) for j in range(b.world) for buf in range(8)],
                         mem.ptr(scratch), info["scratch_needed"])
    mem.sync()
    log(f"  transition done ({time.time() - t0:.1f}s)")
    rng = np.random.default_rng(seed & 0xFFFF)
    checked = 0
    for j in range(b.world):
        for buf in range(8):
            n = b.buffer_elems(j, buf)
            if not n:
                continue
            got = mem.download(dst[(j, buf)]).view(kind_dtype(buf))
            mine = boxes[(boxes["dst_rank"] == j) & (boxes["dst_buf"] == buf)]
            edges = np.concatenate([mine["dst_off"], mine["dst_off"] - 1]) if len(mine) else np.zeros(0, np.int64)
            for c in _sample_chunks(n, chunk, fraction, edges, rng):
                o, m = c * chunk, min(chunk, n - c * chunk)
                want = b.fill(j, buf, seed, 0, off0=o, n=m, pad_word=SENT32)
                if not np.array_equal(got[o:o + m], want):
                    bad = np.nonzero(got[o:o + m] != want)[0]
                    raise AssertionError(f"dst ({j},{buf}): {bad.size} wrong elements in chunk at {o}, first {o + bad[0]}")
                checked += m
    log(f"  {checked} destination elements compared with the oracle ({time.time() - t0:.1f}s)")
    if staged_budget is not None:
        sp = lib.stage_exchange(plan, staged_budget)
        sinfo = sp.info()
        assert sinfo["scratch_needed"] <= info["scratch_needed"]
        sscratch = mem.alloc(sinfo["scratch_needed"])
        again = {k: mem.alloc(len(v)) for k, v in dst.items()}
        lib.apply_transition_staged(sp, [mem.ptr(src[(r, buf)]) for r in range(a.world) for buf in range(8)],
                                    [mem.ptr(again[(j, buf)]) for j in range(b.world) for buf in range(8)],
                                    mem.ptr(sscratch), sinfo["scratch_needed"])
        mem.sync()
        for k, v in dst.items():
            assert mem.equal(again[k], v), f"staged exchange differs from the one-shot result in buffer {k}"
        log(f"  staged: {sinfo['num_stages']} stages over {sinfo['num_steps']} steps, scratch {sinfo['scratch_needed'] >> 20} MiB "
            f"(one shot {info['scratch_needed'] >> 20} MiB), same bytes as the one-shot transition ({time.time() - t0:.1f}s)")
        del sscratch, again, sp
    if round_trip:
        # A -> B -> A gives back every payload element of every source buffer (replicas hold the
        # same bits under the seeded pattern, so the choice of source does not show)
        del scratch
        rplan = lib.plan_intersections(cb, ca, -1)
        rinfo = rplan.buffer_bytes(-1)
        rscratch = mem.alloc(rinfo["scratch_needed"])
        back = {k: mem.alloc(len(v)) for k, v in src.items()}
        lib.apply_transition(rplan, -1, [mem.ptr(dst[(j, buf)]) for j in range(b.world) for buf in range(8)],
                             [mem.ptr(back[(r, buf)]) for r in range(a.world) for buf in range(8)],
                             mem.ptr(rscratch), rinfo["scratch_needed"])
        mem.sync()
        same = 0
        for (r, buf), t in src.items():
            n = a.payload_elems(r, buf) * oracle.KIND_BYTES[buf % 4]
            assert mem.equal(back[(r, buf)][:n], t[:n]), f"round trip changed source buffer ({r},{buf})"
            assert mem.all_bytes(back[(r, buf)][n:], SENTINEL), f"round trip wrote the padding of ({r},{buf})"
            same += n
        log(f"  round trip: {same} bytes identical to the source state ({time.time() - t0:.1f}s)")
    assert mem.violations() == 0, "a kernel wrote outside its buffers"
    return dict(boxes=len(boxes), info=info, checked=checked, stats=plan.stats())


class DryRun:
    """CPU build only: made-up buffer addresses for a walk of the tile table without memory.
    Sources, destinations and scratch live in three separate address windows; the copy step
    checks every access against the registered extents, records every write and moves nothing."""
    SRC, DST, SCRATCH, END = 1 << 44, 1 << 45, 1 << 46, 1 << 47

    def __init__(self, hlib):
        self.dll = hlib._dll
        self.ranges = []
        self.next = {self.SRC: self.SRC, self.DST: self.DST, self.SCRATCH: self.SCRATCH}
        self.dll.vpsh_dry_run_written.restype = C.c_uint64
        self.dll.vpsh_dry_run_written.argtypes = [C.c_uint64, C.c_uint64, C.POINTER(C.c_int64)]
        self.dll.vpsh_bounds_violations.restype = C.c_long

    def buffer(self, window, nbytes, extent=None):
        """Address of a buffer of nbytes in `window`; accesses are legal in its first `extent` bytes."""
        if not nbytes:
            return 0
        p = self.next[window]
        self.next[window] = p + (int(nbytes) + 4095) // 4096 * 4096 + 4096
        self.ranges.append((p, p + int(nbytes if extent is None else extent)))
        return p

    TILE_KINDS = ("full_run", "partial_run", "few_runs", "many_runs", "transpose", "elementwise", "empty")

    def __enter__(self):
        skip = (C.c_uint64 * 7)()
        self.dll.vpsh_tile_histogram(skip, skip)    # reset
        self.dll.vpsh_unaligned_run_tiles()
        arr = (C.c_void_p * (2 * len(self.ranges)))()
        for i, (lo, hi) in enumerate(self.ranges):
            arr[2 * i], arr[2 * i + 1] = lo, hi
        self.dll.vpsh_set_bounds(arr, len(self.ranges))
        self.dll.vpsh_set_dry_run(1)
        return self

    def __exit__(self, *exc):
        self.violations = self.dll.vpsh_bounds_violations()
        ov = C.c_int64(0)
        self.dst_written = self.dll.vpsh_dry_run_written(self.DST, self.SCRATCH, C.byref(ov))
        self.dst_overlaps = ov.value
        self.scratch_written = self.dll.vpsh_dry_run_written(self.SCRATCH, self.END, C.byref(ov))
        self.scratch_overlaps = ov.value
        self.dll.vpsh_set_dry_run(0)
        n, by = (C.c_uint64 * 7)(), (C.c_uint64 * 7)()
        self.dll.vpsh_tile_histogram(n, by)
        self.tiles = {k: (int(n[i]), int(by[i])) for i, k in enumerate(self.TILE_KINDS)}   # kind -> (count, bytes)
        self.dll.vpsh_unaligned_run_tiles.restype = C.c_uint64
        self.unaligned_run_tiles = int(self.dll.vpsh_unaligned_run_tiles())
        return False


def dry_run_single_rank(hlib, model, pa, pb, rank, box_samples=16, through=False):
    """CPU build only: walk the tile table of one rank's apply_transition at full size without
    memory behind it (see DryRun; destination extents end at the padding).  The writes must be
    disjoint and add up to the whole destination payload and the outgoing payload: every
    destination byte and every byte of the send buffer's boxes is written exactly once."""
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = hlib.describe_config(model, pa), hlib.describe_config(model, pb)
    plan = hlib.plan_intersections_ex(ca, cb, rank, PLAN_THROUGH_BUFFERS) if through else hlib.plan_intersections(ca, cb, rank)
    boxes = plan.get_boxes()
    validate_boxes(a, b, boxes, rank, samples=box_samples, through=through, plan=plan)
    info = plan.buffer_bytes(rank)
    dry = DryRun(hlib)
    es = oracle.KIND_BYTES
    src = [dry.buffer(dry.SRC, a.buffer_elems(rank, k) * es[k % 4] if rank < a.world else 0) for k in range(8)]
    dst = [dry.buffer(dry.DST, b.buffer_elems(rank, k) * es[k % 4] if rank < b.world else 0,
                      b.payload_elems(rank, k) * es[k % 4] if rank < b.world else 0) for k in range(8)]
    dst_payload = sum(b.payload_elems(rank, k) * es[k % 4] for k in range(8)) if rank < b.world else 0
    scratch = dry.buffer(dry.SCRATCH, info["scratch_needed"])
    with dry:
        hlib.apply_transition(plan, rank, src, dst, scratch, info["scratch_needed"])
    out = boxes[(boxes["src_rank"] == rank) & ((boxes["dst_rank"] != rank) | through)]
    sent = int((np.prod(out["ext"].astype(np.int64), axis=1) * np.where(out["kind"] == 0, 2, 4)).sum())
    assert dry.violations == 0, f"{dry.violations} accesses outside the buffers"
    assert dry.dst_overlaps == 0 and dry.scratch_overlaps == 0, "a byte is written twice"
    assert dry.dst_written == dst_payload and dry.scratch_written == sent, (dry.dst_written, dst_payload, dry.scratch_written, sent)
    return dict(written=dry.dst_written + dry.scratch_written, dst_payload=dst_payload, sent=sent, stats=plan.stats(), info=info,
                tiles=dry.tiles, unaligned_run_tiles=dry.unaligned_run_tiles)


def dry_run_all_ranks(hlib, model, pa, pb, staged_budget=None, box_samples=4):
    """CPU build only: every virtual rank resident, at full size without memory: the one-shot
    apply_transition(rank=-1), or the staged exchange under a per-rank budget (its scratch regions
    are reused from stage to stage, so only the destination writes must be disjoint)."""
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = hlib.describe_config(model, pa), hlib.describe_config(model, pb)
    plan = hlib.plan_intersections(ca, cb, -1)
    boxes = plan.get_boxes()
    validate_boxes(a, b, boxes, -1, samples=box_samples, plan=plan)
    es = oracle.KIND_BYTES
    dry = DryRun(hlib)
    src = [dry.buffer(dry.SRC, a.buffer_elems(r, k) * es[k % 4]) for r in range(a.world) for k in range(8)]
    dst = [dry.buffer(dry.DST, b.buffer_elems(j, k) * es[k % 4], b.payload_elems(j, k) * es[k % 4])
           for j in range(b.world) for k in range(8)]
    dst_payload = sum(b.payload_elems(j, k) * es[k % 4] for j in range(b.world) for k in range(8))
    moving = boxes[boxes["src_rank"] != boxes["dst_rank"]]
    sent = int((np.prod(moving["ext"].astype(np.int64), axis=1) * np.where(moving["kind"] == 0, 2, 4)).sum())
    if staged_budget is None:
        need = plan.buffer_bytes(-1)["scratch_needed"]
        scratch = dry.buffer(dry.SCRATCH, need)
        with dry:
            hlib.apply_transition(plan, -1, src, dst, scratch, need)
        assert dry.scratch_overlaps == 0 and dry.scratch_written == sent, (dry.scratch_written, sent)
        stages = 0
    else:
        sp = hlib.stage_exchange(plan, staged_budget)
        sinfo = sp.info()
        need, stages = sinfo["scratch_needed"], sinfo["num_stages"]
        scratch = dry.buffer(dry.SCRATCH, need)
        with dry:
            hlib.apply_transition_staged(sp, src, dst, scratch, need)
        assert dry.scratch_written == 2 * sent, (dry.scratch_written, sent)   # packed once, exchanged once
    assert dry.violations == 0, f"{dry.violations} accesses outside the buffers"
    assert dry.dst_overlaps == 0, "a destination byte is written twice"
    assert dry.dst_written == dst_payload, (dry.dst_written, dst_payload)
    return dict(written=dry.dst_written, sent=sent, scratch=need, stages=stages)


# ----------------------------------------------------------------------------- staged exchange

def check_stage_assignment(cost, budget, stage_of_step):
    """Algorithm 1, MemoryAwareChunk, as the properties that define its result (with the two
    declared readings: steps without traffic belong to no stage, no stage is empty).  The stages
    are consecutive groups of the busy steps, in step order; a stage fits the budget unless it is
    a single step; and no stage could have taken the first step of the next one.  These fix the
    partition.  Returns the stages as lists of steps."""
    busy = [s for s in range(1, len(cost)) if cost[s] > 0]
    assert all(stage_of_step[s] == -1 for s in range(1, len(cost)) if cost[s] == 0), "a step without traffic has a stage"
    ids = [stage_of_step[s] for s in busy]
    assert all(g >= 0 for g in ids)
    assert ids == sorted(ids) and (not ids or (ids[0] == 0 and set(ids) == set(range(ids[-1] + 1)))), "stages are not consecutive groups"
    stages = [[s for s in busy if stage_of_step[s] == g] for g in range(ids[-1] + 1)] if ids else []
    load = [sum(cost[s] for s in st) for st in stages]
    for g, st in enumerate(stages):
        assert load[g] <= budget or len(st) == 1, ("a stage of several steps exceeds the budget", g)
        if g + 1 < len(stages):
            assert load[g] + cost[stages[g + 1][0]] > budget, ("a stage was closed although the next step still fitted", g)
    return stages


def run_staged(lib, mem, model, pa, pb, seed, budget, rank_salt=0x9E37):
    """All ranks resident, exchange in XOR step order under a per-rank buffer budget."""
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    plan = lib.plan_intersections(ca, cb, -1)
    sp = lib.stage_exchange(plan, budget)
    info = sp.info()
    stage_of_step, step_cost = sp.steps()
    W = max(a.world, b.world)
    assert info["num_steps"] == (1 << max(W - 1, 0).bit_length()) - 1

    # the schedule against the properties that define Algorithm 1's stages
    seg = np.zeros((W, W), dtype=np.int64)
    for i in range(a.world):
        rb = None
        for j in range(b.world):
            if i != j:
                seg[i, j] = plan.peer_segment(i, j)["bytes"]
    cost = [0] * (info["num_steps"] + 1)
    for s in range(1, info["num_steps"] + 1):
        cost[s] = max(int(seg[r, r ^ s] if (r ^ s) < W else 0) + int(seg[r ^ s, r] if (r ^ s) < W else 0) for r in range(W))
    assert cost == [int(c) for c in step_cost]
    stages = check_stage_assignment(cost, budget, stage_of_step)
    assert len(stages) == info["num_stages"]
    # XOR pairing: an involution, and every pair with traffic is met in exactly one step
    for i in range(W):
        for j in range(W):
            if i != j and seg[i, j]:
                s = i ^ j
                assert 1 <= s <= info["num_steps"] and (j ^ s) == i and stage_of_step[s] >= 0
    # payload never exceeds the aligned segments, and the budget holds when it can
    for j in range(b.world):
        rb = oracle.route_bytes(a, b, j)
        for i in range(a.world):
            if i != j:
                assert rb[i] <= seg[i, j] <= rb[i] + 16 * plan.num_boxes
    if budget >= max(cost):
        for steps in stages:
            assert sum(cost[s] for s in steps) <= budget

    src_host = {(r, buf): a.fill(r, buf, seed, rank_salt, pad_word=0x3C3C3C3C) for r in range(a.world) for buf in range(8)}
    src = {k: mem.alloc(v.nbytes) for k, v in src_host.items()}
    for k, v in src_host.items():
        mem.upload(src[k], v)
    dst = {(j, buf): mem.alloc(b.buffer_elems(j, buf) * oracle.KIND_BYTES[buf % 4]) for j in range(b.world) for buf in range(8)}
    scratch = mem.alloc(info["scratch_needed"])
    mem.register_bounds()
    lib.apply_transition_staged(sp, [mem.ptr(src[(r, buf)]) for r in range(a.world) for buf in range(8)],
                                [mem.ptr(dst[(j, buf)]) for j in range(b.world) for buf in range(8)],
                                mem.ptr(scratch), info["scratch_needed"])
    mem.sync()
    assert mem.violations() == 0
    for (j, buf), d in dst.items():
        want = oracle.expected(a, b, j, buf, seed, rank_salt, pad_word=SENT32)
        got = mem.download(d).view(want.dtype)
        assert np.array_equal(got, want), ("staged", j, buf)
    one_shot = plan.buffer_bytes(-1)["scratch_needed"]
    return dict(stages=info["num_stages"], steps=info["num_steps"], scratch=info["scratch_needed"], one_shot=one_shot,
                max_cost=max(cost), costs=cost)


# ----------------------------------------------------------------------------- collective intent

def classify_bruteforce(boxes, shapes):
    """Algorithm 1, OptimizePrimitives, from its definitions over plain index sets: per logical
    tensor and kind, the slices that leave their rank as sets of positions in the flattened
    tensor.  Identical = all the same set; a tiling = every slice an interval, the slices disjoint
    and their union an interval again.  One source and several destinations make a broadcast
    (identical slices) or a scatter (tiling), several sources and one destination with a tiling a
    gather, anything else stays point-to-point.  Returns {(tensor, kind): code} as in vps.h."""
    P2P, BROADCAST, SCATTER, GATHER = 1, 2, 3, 4
    groups = {}
    for bx in boxes:
        if bx["src_rank"] != bx["dst_rank"]:
            cells = np.ix_(*[np.arange(int(l), int(l) + int(e)) for l, e in zip(bx["lo"], bx["ext"])])
            where = frozenset(np.ravel_multi_index(cells, shapes[int(bx["tensor"])]).ravel().tolist())
            g = groups.setdefault((int(bx["tensor"]), int(bx["kind"])), dict(src=set(), dst=set(), slices=[]))
            g["src"].add(int(bx["src_rank"]))
            g["dst"].add(int(bx["dst_rank"]))
            g["slices"].append(where)
    interval = lambda cells: max(cells) - min(cells) + 1 == len(cells)
    out = {}
    for key, g in groups.items():
        union = frozenset().union(*g["slices"])
        identical = len(set(g["slices"])) == 1
        tiling = all(interval(c) for c in g["slices"]) and sum(len(c) for c in g["slices"]) == len(union) and interval(union)
        fan_out, fan_in = len(g["src"]) == 1 and len(g["dst"]) > 1, len(g["src"]) > 1 and len(g["dst"]) == 1
        out[key] = BROADCAST if fan_out and identical else SCATTER if fan_out and tiling else GATHER if fan_in and tiling else P2P
    return out


def run_classify(lib, model, pa, pb):
    a = oracle.Config(model, pa)
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    plan = lib.plan_intersections_ex(ca, cb, -1, flags=1)
    got = plan.classify_collectives(ca)
    shapes = [a.tensor_info(t)["shape"] for t in range(a.num_tensors)]
    want = classify_bruteforce(plan.get_boxes(), shapes)
    for t in range(a.num_tensors):
        for kind in range(4):
            assert got[t * 4 + kind] == want.get((t, kind), 0), (t, kind, got[t * 4 + kind], want.get((t, kind), 0))
    return np.bincount(got, minlength=5)

"""Textbook resharding with numpy slicing: a second, independent formulation of the layouts.

Used only to pin the CPU oracle (tests/test_oracle_*.py).  Where the oracle computes one
element at a time from index arithmetic, this module builds every logical tensor as an array of
addresses, cuts it with np.split / np.transpose / np.concatenate the way a training framework
would shard it, and flattens the result into the rank-local buffers.  The two share no code.

Layout conventions restated here (declared readings, the paper leaves them open):
rank = tp + TP*(ddp + DDP*pp); the expert group sees position q = rank mod (TP*DDP) of a stage
as q = etp + ETP*(ep + EP*edp), with (ETP, EDP, DDP) = (TP, DP, DP*EP) when EP and expert-DP form
a grid beside TP and (1, TP*DP/EP, DP) when EP is carved out of the TP x DP ranks; stage p owns
layers [p*L//PP, (p+1)*L//PP); flat buffers are per (rank, group), tail padded to 8*D elements.
"""
import numpy as np

GPT, GQA, MOE = 0, 1, 2


def inventory(m):
    """[(natural shape, tp axis or None, group, layer, expert, role)] in forward order."""
    h, d, g, L = m["hidden"], m["head_dim"], m["kv_heads"], m["layers"]
    s = m["q_heads"] // m["kv_heads"] + 2
    qd = m["q_heads"] * d
    inv = [((m["vocab"], h), 0, 0, -1, -1, "")]
    for l in range(L):
        if m["family"] == GPT:
            inv += [((h,), None, 0, l, -1, ""), ((h,), None, 0, l, -1, ""),
                    ((g, s, d, h), 0, 0, l, -1, "qkv"), ((g, s, d), 0, 0, l, -1, "qkv"),
                    ((h, qd), 1, 0, l, -1, ""), ((h,), None, 0, l, -1, ""),
                    ((h,), None, 0, l, -1, ""), ((h,), None, 0, l, -1, ""),
                    ((m["ffn"], h), 0, 0, l, -1, ""), ((m["ffn"],), 0, 0, l, -1, ""),
                    ((h, m["ffn"]), 1, 0, l, -1, ""), ((h,), None, 0, l, -1, "")]
        else:
            inv += [((h,), None, 0, l, -1, ""), ((g, s, d, h), 0, 0, l, -1, "qkv")]
            if m["family"] == MOE:
                inv += [((d,), None, 0, l, -1, ""), ((d,), None, 0, l, -1, "")]
            inv += [((h, qd), 1, 0, l, -1, ""), ((h,), None, 0, l, -1, "")]
            if m["family"] == GQA:
                inv += [((2, m["ffn"], h), 1, 0, l, -1, ""), ((h, m["ffn"]), 1, 0, l, -1, "")]
            else:
                inv += [((m["experts"], h), None, 0, l, -1, "")]
                for e in range(m["experts"]):
                    inv += [((2, m["expert_ffn"], h), 1, 1, l, e, "gate_up"),
                            ((h, m["expert_ffn"]), 1, 1, l, e, "down")]
    inv += [((h,), None, 0, L, -1, "")] * (2 if m["family"] == GPT else 1)
    inv += [((m["vocab"], h), 0, 0, L, -1, "")]
    return inv


def _stage(layer, L, PP):
    if layer < 0:
        return 0
    if layer >= L:
        return PP - 1
    return [p for p in range(PP) if (p * L) // PP <= layer < ((p + 1) * L) // PP][0]


def _stored_blocks(addr, tp_axis, tp, TP, role, p, q_per_g):
    """Shard `addr` (array of linear indices in natural shape) the way a rank stores it: a list of
    arrays (storage blocks), each to be flattened row-major, one after the other."""
    x = addr
    if tp_axis is not None:
        x = np.split(x, TP, axis=tp_axis)[tp]
    if role == "qkv" and p["qkv_layout"] == 1:
        return [x[:, :q_per_g], x[:, q_per_g:q_per_g + 1], x[:, q_per_g + 1:]]
    if role == "gate_up" and p["expert_layout"] == 1:
        return [np.transpose(x, (2, 0, 1))]
    if role == "down" and p["expert_layout"] == 1:
        return [np.transpose(x, (1, 0))]
    return [x]


def degrees(p):
    """(TP, PP, dense DP, EP, expert TP, expert DP, world) of a parallel description."""
    TP, PP, DP, EP = p["tp"], p["pp"], p["dp"], p["ep"]
    if p.get("ep_placement", 0) == 0:
        return TP, PP, DP * EP, EP, TP, DP, TP * PP * DP * EP
    return TP, PP, DP, EP, 1, TP * DP // EP, TP * PP * DP


def rank_position(p, rank):
    """tp, dense dp index, pipeline stage, expert tp, ep, expert dp index of a rank."""
    TP, PP, DDP, EP, ETP, EDP, world = degrees(p)
    tp, ddp, pp = rank % TP, (rank // TP) % DDP, rank // (TP * DDP)
    q = rank % (TP * DDP)
    return tp, ddp, pp, q % ETP, (q // ETP) % EP, q // (ETP * EP)


def rank_blocks(m, p, rank, group):
    """The storage blocks of (rank, group) in flat order: [(tensor, block array of addresses)],
    the data-parallel group size and the rank's index in it."""
    inv = inventory(m)
    TP, PP, DDP, EP, ETP, EDP, world = degrees(p)
    tp, ddp, pp, etp, ep, edp = rank_position(p, rank)
    L = m["layers"]
    q_per_g = m["q_heads"] // m["kv_heads"]
    T, t_idx, D, didx = (TP, tp, DDP, ddp) if group == 0 else (ETP, etp, EDP, edp)
    order = range(len(inv))
    if p["flat_order"] == 1:
        order = reversed(order)
    blocks = []
    for t in order:
        shape, tp_axis, grp, layer, expert, role = inv[t]
        if grp != group or _stage(layer, L, PP) != pp:
            continue
        if group == 1 and expert // (m["experts"] // EP) != ep:
            continue
        addr = np.arange(int(np.prod(shape)), dtype=np.int64).reshape(shape)
        for blk in _stored_blocks(addr, tp_axis, t_idx, T, role, p, q_per_g):
            blocks.append((t, blk))
    return blocks, D, didx


def address_layout(m, p):
    """{(rank, buf): (tensor ids int32, linear indices int64)}; padding slots have tensor -1."""
    world = degrees(p)[6]
    out = {}
    for rank in range(world):
        for group in (0, 1):
            blocks, D, didx = rank_blocks(m, p, rank, group)
            tid = np.concatenate([np.zeros(0, np.int32)] + [np.full(b.size, t, np.int32) for t, b in blocks])
            lin = np.concatenate([np.zeros(0, np.int64)] + [b.ravel() for t, b in blocks])
            padn = (-tid.size) % (8 * D)
            tid = np.concatenate([tid, np.full(padn, -1, np.int32)])
            lin = np.concatenate([lin, np.full(padn, -1, np.int64)])
            for kind in range(4):
                if kind != 0 and p["zero"] == 1:
                    out[(rank, group * 4 + kind)] = (np.split(tid, D)[didx], np.split(lin, D)[didx])
                else:
                    out[(rank, group * 4 + kind)] = (tid, lin)
    return out


def range_boxes(shape, v0, v1):
    """The linear range [v0, v1) of a row-major array of `shape` as the fewest boxes (tuples of
    slices): whole slabs along the leading axis form one box, a partial first or last slab is cut
    the same way one axis further in."""
    if not shape:
        return [()]
    inner = int(np.prod(shape[1:], dtype=np.int64))
    first, last = v0 // inner, (v1 - 1) // inner
    if v0 == first * inner and v1 == (last + 1) * inner:
        return [(slice(first, last + 1),) + tuple(slice(0, n) for n in shape[1:])]
    if first == last:
        return [(slice(first, first + 1),) + b for b in range_boxes(shape[1:], v0 - first * inner, v1 - first * inner)]
    out, k0, k1 = [], first, last + 1
    if v0 != first * inner:
        out += [(slice(first, first + 1),) + b for b in range_boxes(shape[1:], v0 - first * inner, inner)]
        k0 = first + 1
    tail = []
    if v1 != (last + 1) * inner:
        tail = [(slice(last, last + 1),) + b for b in range_boxes(shape[1:], 0, v1 - last * inner)]
        k1 = last
    if k0 < k1:
        out.append((slice(k0, k1),) + tuple(slice(0, n) for n in shape[1:]))
    return out + tail


def pieces(m, p):
    """{(rank, buf): [(tensor, buffer offsets int64, addresses int64)]}: every rank's stored data cut
    into boxes: per storage block the rank's flat range, split by range_boxes.  Offsets and
    addresses (linear indices in the unsharded tensor) are in the box's storage order."""
    world = degrees(p)[6]
    out = {}
    for rank in range(world):
        for group in (0, 1):
            blocks, D, didx = rank_blocks(m, p, rank, group)
            total = sum(b.size for _, b in blocks)
            padded = total + (-total) % (8 * D)
            for kind in range(4):
                sharded = kind != 0 and p["zero"] == 1
                r0, r1 = (padded // D * didx, padded // D * (didx + 1)) if sharded else (0, padded)
                lst, start = [], 0
                for t, blk in blocks:
                    v0, v1 = max(r0, start) - start, min(r1, start + blk.size) - start
                    if v0 < v1:
                        where = np.arange(blk.size, dtype=np.int64).reshape(blk.shape)
                        for box in range_boxes(blk.shape, v0, v1):
                            lst.append((t, where[box].ravel() + (start - r0), blk[box].ravel()))
                    start += blk.size
                out[(rank, group * 4 + kind)] = lst
    return out


def scatter(full, layout, dtype_of_buf, pad_word=0):
    """Local buffers from full logical tensors: full[(kind, tensor)] = flat ndarray."""
    bufs = {}
    for (rank, buf), (tid, lin) in layout.items():
        kind = buf % 4
        out = np.full(tid.size, pad_word, dtype=dtype_of_buf(buf))
        for t in np.unique(tid[tid >= 0]):
            sel = tid == t
            out[sel] = full[(kind, int(t))][lin[sel]]
        bufs[(rank, buf)] = out
    return bufs


def assemble(bufs, layout, inv):
    """Full logical tensors from local buffers; asserts that every replica agrees."""
    full, seen = {}, {}
    for (rank, buf), (tid, lin) in layout.items():
        kind = buf % 4
        for t in np.unique(tid[tid >= 0]):
            key = (kind, int(t))
            n = int(np.prod(inv[int(t)][0]))
            if key not in full:
                full[key] = np.zeros(n, dtype=bufs[(rank, buf)].dtype)
                seen[key] = np.zeros(n, dtype=bool)
            sel = tid == t
            vals, idx = bufs[(rank, buf)][sel], lin[sel]
            again = seen[key][idx]
            assert np.array_equal(full[key][idx[again]], vals[again]), "replicas disagree"
            full[key][idx] = vals
            seen[key][idx] = True
    for key, s in seen.items():
        assert s.all(), f"tensor {key} not fully covered"
    return full

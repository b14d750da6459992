"""Textbook resharding with numpy slicing: a second, independent formulation of the layouts.

Used only to pin the CPU oracle (tests/test_oracle_*.py).  Where the oracle computes one
element at a time from index arithmetic, this module builds every logical tensor as an array of
addresses, cuts it with np.split / np.transpose / np.concatenate the way a training framework
would shard it, and flattens the result into the rank-local buffers.  The two share no code.

Layout conventions restated here (declared readings, the paper leaves them open):
rank = tp + TP*(ddp + DDP*pp), ddp = ep + EP*edp; stage p owns layers
[p*L//PP, (p+1)*L//PP); flat buffers are per (rank, group), tail padded to 8*D elements.
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


def _stored(addr, tp_axis, tp, TP, role, p, q_per_g):
    """Shard `addr` (array of linear indices in natural shape) and flatten in storage order."""
    x = addr
    if tp_axis is not None:
        x = np.split(x, TP, axis=tp_axis)[tp]
    if role == "qkv" and p["qkv_layout"] == 1:
        parts = [x[:, :q_per_g], x[:, q_per_g:q_per_g + 1], x[:, q_per_g + 1:]]
        return np.concatenate([q.ravel() for q in parts])
    if role == "gate_up" and p["expert_layout"] == 1:
        return np.transpose(x, (2, 0, 1)).ravel()
    if role == "down" and p["expert_layout"] == 1:
        return np.transpose(x, (1, 0)).ravel()
    return x.ravel()


def address_layout(m, p):
    """{(rank, buf): (tensor ids int32, linear indices int64)}; padding slots have tensor -1."""
    inv = inventory(m)
    TP, PP, DP, EP = p["tp"], p["pp"], p["dp"], p["ep"]
    DDP = DP * EP
    L = m["layers"]
    q_per_g = m["q_heads"] // m["kv_heads"]
    out = {}
    for pp in range(PP):
        for ddp in range(DDP):
            ep, edp = ddp % EP, ddp // EP
            for tp in range(TP):
                rank = tp + TP * (ddp + DDP * pp)
                for group in (0, 1):
                    D, didx = (DDP, ddp) if group == 0 else (DP, edp)
                    tids, lins = [np.zeros(0, np.int32)], [np.zeros(0, np.int64)]
                    order = range(len(inv))
                    if p["flat_order"] == 1:
                        order = reversed(order)
                    for t in order:
                        shape, tp_axis, grp, layer, expert, role = inv[t]
                        if grp != group or _stage(layer, L, PP) != pp:
                            continue
                        if group == 1 and expert // (m["experts"] // EP) != ep:
                            continue
                        addr = np.arange(int(np.prod(shape)), dtype=np.int64).reshape(shape)
                        flat = _stored(addr, tp_axis, tp, TP, role, p, q_per_g)
                        lins.append(flat)
                        tids.append(np.full(flat.size, t, np.int32))
                    tid, lin = np.concatenate(tids), np.concatenate(lins)
                    quantum = 8 * D
                    padn = (-tid.size) % quantum
                    tid = np.concatenate([tid, np.full(padn, -1, np.int32)])
                    lin = np.concatenate([lin, np.full(padn, -1, np.int64)])
                    for kind in range(4):
                        if kind != 0 and p["zero"] == 1:
                            out[(rank, group * 4 + kind)] = (np.split(tid, D)[didx], np.split(lin, D)[didx])
                        else:
                            out[(rank, group * 4 + kind)] = (tid, lin)
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

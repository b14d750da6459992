"""Pins for the CPU oracle: it is checked against things other than itself.

* an independent numpy-slicing formulation of every layout (tests/textbook.py),
* brute force over every element of tiny models (inverse maps, replica counts),
* closed forms (parameter counts, pure-TP / pure-DP byte counts),
* invariants (identity, round trip, region algebra of Section 4.2.1),
* the worked example of Figure 4 (rank 3, (TP,PP) = (2,2) -> (4,1)).
"""
import itertools

import numpy as np
import pytest

import oracle
import textbook
from datagen import configs as cf
from datagen import pattern

P = cf.parallel

LAYOUT_CASES = [
    ("gpt-tp2dp2z1", cf.TINY_GPT, P(tp=2, dp=2, zero=1)),
    ("gpt-tp1dp4z0", cf.TINY_GPT, P(tp=1, dp=4, zero=0)),
    ("gpt-tp4pp2dp1", cf.TINY_GPT, P(tp=4, pp=2, dp=1, zero=1)),
    ("gpt-tp2pp4dp3-blocked-rev", cf.TINY_GPT, P(tp=2, pp=4, dp=3, zero=1, qkv_layout=1, flat_order=1)),
    ("gpt-odd-tp3pp3dp2", cf.ODD_GPT, P(tp=3, pp=3, dp=2, zero=1)),
    ("gpt-odd-tp2dp5-blocked", cf.ODD_GPT, P(tp=2, pp=2, dp=5, zero=1, qkv_layout=1)),
    ("gqa-tp4pp2dp2", cf.TINY_GQA, P(tp=4, pp=2, dp=2, zero=1)),
    ("gqa-tp2pp1dp3-blocked", cf.TINY_GQA, P(tp=2, pp=1, dp=3, zero=1, qkv_layout=1)),
    ("moe-ep4dp2pp2", cf.TINY_MOE, P(tp=1, pp=2, dp=2, ep=4, zero=1)),
    ("moe-ep8dp1pp4-transposed", cf.TINY_MOE, P(tp=1, pp=4, dp=1, ep=8, zero=1, expert_layout=1)),
    ("moe-tp2ep2dp2-transposed-rev", cf.TINY_MOE, P(tp=2, pp=1, dp=2, ep=2, zero=1, expert_layout=1, flat_order=1)),
    ("moe-odd-ep3dp2pp2z0", cf.ODD_MOE, P(tp=1, pp=2, dp=2, ep=3, zero=0)),
    ("moe-odd-tp2ep2dp3-blocked-transposed", cf.ODD_MOE, P(tp=2, pp=3, dp=3, ep=2, zero=1, qkv_layout=1, expert_layout=1)),
]

# EP carved out of the TP x DP ranks of a stage (the form of the paper's MoE strategy tuples)
LAYOUT_CASES += [
    ("moe-carved-tp2dp2ep4", cf.TINY_MOE, P(tp=2, pp=2, dp=2, ep=4, zero=1, ep_placement=1)),
    ("moe-carved-tp4dp1ep2-transposed", cf.TINY_MOE, P(tp=4, pp=1, dp=1, ep=2, zero=1, expert_layout=1, ep_placement=1)),
    ("moe-odd-carved-tp2dp3ep3-z0", cf.ODD_MOE, P(tp=2, pp=1, dp=3, ep=3, zero=0, ep_placement=1)),
    ("moe-odd-carved-tp1dp6ep2-blocked-rev", cf.ODD_MOE, P(tp=1, pp=5, dp=6, ep=2, zero=1, qkv_layout=1, flat_order=1, ep_placement=1)),
]

TRANSITIONS = [
    ("gpt-zero-to-replicated", cf.TINY_GPT, P(tp=2, dp=2, zero=1), P(tp=1, dp=4, zero=0)),
    ("gpt-tp-pp", cf.TINY_GPT, P(tp=4, pp=2, dp=1), P(tp=2, pp=4, dp=1)),
    ("gpt-blocked-rev", cf.TINY_GPT, P(tp=2, pp=2, dp=2), P(tp=4, pp=1, dp=2, qkv_layout=1, flat_order=1)),
    ("gpt-odd", cf.ODD_GPT, P(tp=3, pp=1, dp=2), P(tp=2, pp=3, dp=1, qkv_layout=1)),
    ("gpt-world-grows", cf.TINY_GPT, P(tp=2, pp=2, dp=2), P(tp=4, pp=4, dp=1)),
    ("gqa", cf.TINY_GQA, P(tp=4, pp=1, dp=2), P(tp=2, pp=2, dp=2, qkv_layout=1)),
    ("moe-ep", cf.TINY_MOE, P(tp=1, pp=4, dp=2, ep=2), P(tp=1, pp=2, dp=2, ep=4)),
    ("moe-transposed", cf.TINY_MOE, P(tp=2, pp=2, dp=1, ep=2), P(tp=1, pp=2, dp=2, ep=2, expert_layout=1)),
    ("moe-odd", cf.ODD_MOE, P(tp=1, pp=2, dp=2, ep=3), P(tp=2, pp=1, dp=3, ep=2, expert_layout=1, flat_order=1)),
]


# Transitions between configurations with EP carved out of TP x DP (and to / from the grid form)
TRANSITIONS_CARVED = [
    ("moe-carved-ep-shrinks", cf.TINY_MOE, P(tp=4, pp=2, dp=1, ep=4, ep_placement=1), P(tp=2, pp=1, dp=4, ep=2, ep_placement=1)),
    ("moe-carved-ep-grows", cf.TINY_MOE, P(tp=2, pp=2, dp=2, ep=2, ep_placement=1), P(tp=4, pp=4, dp=1, ep=4, ep_placement=1, expert_layout=1)),
    ("moe-grid-to-carved", cf.TINY_MOE, P(tp=2, pp=2, dp=1, ep=2), P(tp=2, pp=1, dp=4, ep=8, ep_placement=1)),
    ("moe-odd-carved", cf.ODD_MOE, P(tp=2, pp=1, dp=3, ep=3, ep_placement=1), P(tp=1, pp=5, dp=2, ep=2, ep_placement=1, flat_order=1)),
]
ALL_TRANSITIONS = TRANSITIONS + TRANSITIONS_CARVED


def _golden():
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [x.strip() for x in line.split("=")]
            vals[k] = float(v)
    return vals


GOLD = _golden()


# ----------------------------------------------------------------------------- inventory

def _closed_form_params(m):
    h, d, q, kv, L, V = m["hidden"], m["head_dim"], m["q_heads"], m["kv_heads"], m["layers"], m["vocab"]
    qkv = (q + 2 * kv) * d * h
    if m["family"] == cf.FAMILY_GPT:
        per = 2 * h + qkv + (q + 2 * kv) * d + h * q * d + h + 2 * h + 2 * m["ffn"] * h + m["ffn"] + h
        return L * per + 2 * V * h + 2 * h
    if m["family"] == cf.FAMILY_GQA:
        return L * (2 * h + qkv + h * q * d + 3 * m["ffn"] * h) + 2 * V * h + h
    E, ef = m["experts"], m["expert_ffn"]
    return L * (2 * h + qkv + 2 * d + h * q * d + E * h + E * 3 * ef * h) + 2 * V * h + h


@pytest.mark.parametrize("name,tensors,params", [
    ("toy", 28, 2_104_320), ("gpt1p3b", 292, 1_414_647_808), ("gqa8b", 195, 8_030_261_248),
    ("gqa70b", 483, 70_553_706_496), ("moe235b", 24_725, 235_093_634_560)])
def test_inventory_matches_architecture_closed_form(name, tensors, params):
    w = cf.WORKLOADS[name]
    c = oracle.Config(w["model"], w["src"])
    assert c.num_tensors == tensors
    assert c.total_params == params == _closed_form_params(w["model"])
    assert c.world == cf.world(w["src"])
    assert oracle.Config(w["model"], w["dst"]).world == cf.world(w["dst"])


def test_70b_replica_state_is_about_1p26_tb():
    # Section 2.3 (C3): one DP replica of a 70B model in bf16-fp32 training holds about 1.26 TB
    # (2 B param + 4 B grad + 4 B master + 4 B m + 4 B v per parameter).
    w = cf.WORKLOADS["gqa70b"]
    n = oracle.Config(w["model"], w["src"]).total_params
    assert abs(n * GOLD["replica_state_bytes_per_param"] / (GOLD["replica_state_70b_tb"] * 1e12) - 1) < 0.01
    # Without gradients (collected before a switch) the migrated state is 14 B per parameter:
    a = oracle.Config(w["model"], w["src"])
    tot = 0
    for pp in range(8):
        for tp in range(8):
            r = tp + 8 * (0 + 2 * pp)
            tot += 2 * a.payload_elems(r, 0)
            for dp in range(2):
                rr = tp + 8 * (dp + 2 * pp)
                tot += sum(4 * a.payload_elems(rr, k) for k in (1, 2, 3))
    # norms are replicated over TP, so the sum is slightly above 14 B/param
    assert tot == 14 * (n + 7 * 161 * 8192)  # 161 norm vectors, 7 extra TP copies each


@pytest.mark.parametrize("bad", [P(tp=3), P(tp=16), P(pp=5), P(ep=2)])
def test_indivisible_degrees_are_rejected(bad):
    with pytest.raises(oracle.OracleError):
        oracle.Config(cf.TINY_GPT, bad)
    with pytest.raises(oracle.OracleError):
        oracle.Config(cf.TINY_MOE, P(ep=3))


# ----------------------------------------------------------------------------- layouts

@pytest.mark.parametrize("name,m,p", LAYOUT_CASES, ids=[c[0] for c in LAYOUT_CASES])
def test_fill_equals_textbook_layout(name, m, p):
    """coord_P against numpy slicing, every slot of every rank and buffer."""
    c = oracle.Config(m, p)
    layout = textbook.address_layout(m, p)
    assert c.world == cf.world(p) == textbook.degrees(p)[6]
    seed = 0xABCDEF
    for rank in range(c.world):
        for buf in range(8):
            tid, lin = layout[(rank, buf)]
            assert c.buffer_elems(rank, buf) == tid.size
            assert c.payload_elems(rank, buf) == int((tid >= 0).sum())
            got = c.fill(rank, buf, seed, pad_word=0xA5A5A5A5)
            want = np.full(tid.size, 0xA5A5A5A5 & (0xFFFF if buf % 4 == 0 else 0xFFFFFFFF), dtype=got.dtype)
            for t in np.unique(tid[tid >= 0]):
                sel = tid == t
                want[sel] = pattern.word(seed, buf % 4, int(t), lin[sel].astype(np.uint64))
            assert np.array_equal(got, want), (rank, buf)
            with pytest.raises(IndexError):
                c.coord(rank, buf, tid.size)


@pytest.mark.parametrize("name,m,p", LAYOUT_CASES, ids=[c[0] for c in LAYOUT_CASES])
def test_owners_is_inverse_of_coord_bruteforce(name, m, p):
    """owners_P against the set of slots that the textbook layout gives; replica counts."""
    c = oracle.Config(m, p)
    layout = textbook.address_layout(m, p)
    slots = {}
    for (rank, buf), (tid, lin) in layout.items():
        for pos in np.nonzero(tid >= 0)[0]:
            slots.setdefault((buf % 4, int(tid[pos]), int(lin[pos])), []).append((rank, buf, int(pos)))
    TP, PP, DDP, EP, ETP, EDP, world = textbook.degrees(p)
    assert c.world == world
    total = 0
    for t in range(c.num_tensors):
        info = c.tensor_info(t)
        shape = info["shape"]
        for kind in range(4):
            D = DDP if info["group"] == 0 else EDP
            T = TP if info["group"] == 0 else ETP
            replicas = (T if (info["tp_axis"] < 0 or T == 1) else 1) * (1 if (kind and p["zero"]) else D)
            step = 1 if kind in (0, 1) else 7  # kinds 2, 3 behave like kind 1: sample them
            for lin_idx in range(0, int(np.prod(shape)), step):
                cd = np.unravel_index(lin_idx, shape)
                own = c.owners(kind, t, [int(x) for x in cd], max_owners=256)
                assert c.linear(t, [int(x) for x in cd]) == lin_idx
                assert len(own) == replicas
                assert sorted(own) == sorted(slots[(kind, t, lin_idx)])
                assert [o[0] for o in own] == sorted(o[0] for o in own)
                for (r, b, o) in own[:2]:
                    assert c.coord(r, b, o) == (t, tuple(int(x) for x in cd))
                total += len(own)
    assert total > 0


# ----------------------------------------------------------------------------- transitions

def _random_full(m, rng):
    inv = textbook.inventory(m)
    full = {}
    for t, (shape, *_rest) in enumerate(inv):
        n = int(np.prod(shape))
        full[(0, t)] = rng.integers(0, 1 << 16, n, dtype=np.uint16)
        for k in (1, 2, 3):
            full[(k, t)] = rng.integers(0, 1 << 32, n, dtype=np.uint32)
    return inv, full


def _oracle_transition_all(a, b, src):
    out = {}
    for j in range(b.world):
        for buf in range(8):
            n = b.buffer_elems(j, buf)
            dst = np.full(n, 0xA5A5, dtype=oracle.kind_dtype(buf))
            if n:
                oracle.transition(a, b, j, buf, src, dst)
            out[(j, buf)] = dst
    return out


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_transition_equals_assemble_then_slice(name, m, pa, pb):
    """The per-element transition against the textbook reshard: gather every logical tensor
    from the source shards, cut it again for the destination configuration."""
    rng = np.random.default_rng(7)
    inv, full = _random_full(m, rng)
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    la, lb = textbook.address_layout(m, pa), textbook.address_layout(m, pb)
    src = textbook.scatter(full, la, oracle.kind_dtype, pad_word=0x5A5A)
    again = textbook.assemble(src, la, inv)
    for key in full:
        assert np.array_equal(again[key], full[key])
    want = textbook.scatter(full, lb, oracle.kind_dtype, pad_word=0xA5A5)
    got = _oracle_transition_all(a, b, src)
    for key in want:
        assert np.array_equal(got[key], want[key]), key


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_expected_is_layout_b_fill_and_roundtrip(name, m, pa, pb):
    """With coordinate-hash payloads: A->B gives the layout-B fill; A->B->A is the identity."""
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    seed = 99
    srcA = {(r, buf): a.fill(r, buf, seed, pad_word=0x1111) for r in range(a.world) for buf in range(8)}
    mid = _oracle_transition_all(a, b, srcA)
    for j in range(b.world):
        for buf in range(8):
            fillB = b.fill(j, buf, seed, pad_word=0xA5A5)
            assert np.array_equal(mid[(j, buf)], fillB)
            assert np.array_equal(oracle.expected(a, b, j, buf, seed, pad_word=0xA5A5), fillB)
    back = _oracle_transition_all(b, a, mid)
    for r in range(a.world):
        for buf in range(8):
            pay = a.payload_elems(r, buf)
            # payload identical, padding untouched by the transition
            tid_ok = np.array([a.coord(r, buf, o) is not None for o in range(a.buffer_elems(r, buf))], dtype=bool)
            assert int(tid_ok.sum()) == pay
            assert np.array_equal(back[(r, buf)][tid_ok], srcA[(r, buf)][tid_ok])
            assert (back[(r, buf)][~tid_ok] == 0xA5A5).all()


@pytest.mark.parametrize("name,m,p", LAYOUT_CASES[:6] + LAYOUT_CASES[8:10], ids=[c[0] for c in LAYOUT_CASES[:6] + LAYOUT_CASES[8:10]])
def test_identity_transition_moves_nothing(name, m, p):
    """Only shards affected by the change move (Section 6.2): A->A retains everything."""
    a = oracle.Config(m, p)
    for j in range(a.world):
        rb = oracle.route_bytes(a, a, j)
        pay = sum(a.payload_elems(j, buf) * oracle.KIND_BYTES[buf % 4] for buf in range(8))
        assert rb[j] == pay and rb.sum() == pay
        sb = oracle.send_bytes(a, a, j)
        assert sb[j] == pay and sb.sum() == pay


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_send_and_receive_byte_counts_agree(name, m, pa, pb):
    """Buffer byte counts match on both sides: what i sends to j is what j takes from i, the
    received plus retained volume is the destination payload."""
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    recv = np.stack([oracle.route_bytes(a, b, j) for j in range(b.world)])      # [j, i]
    send = np.stack([oracle.send_bytes(a, b, i) for i in range(a.world)])       # [i, j]
    assert np.array_equal(recv, send.T)
    for j in range(b.world):
        pay = sum(b.payload_elems(j, buf) * oracle.KIND_BYTES[buf % 4] for buf in range(8))
        assert recv[j].sum() == pay


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_region_algebra_and_selection_rule(name, m, pa, pb):
    """Section 4.2.1: per rank, T_retain = R_src & R_dst is exactly what is copied locally,
    T_recv = R_dst - R_src is exactly what arrives from peers, T_send = R_src - R_dst never
    stays.  The chosen source is always an owner; a same-node owner wins over a remote one."""
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    la, lb = textbook.address_layout(m, pa), textbook.address_layout(m, pb)

    def region(layout, rank):
        s = set()
        for buf in range(8):
            if (rank, buf) not in layout:
                continue
            tid, lin = layout[(rank, buf)]
            ok = tid >= 0
            s.update(zip(itertools.repeat(buf % 4), tid[ok].tolist(), lin[ok].tolist()))
        return s

    node = pa["gpus_per_node"]
    for j in range(b.world):
        r_dst = region(lb, j)
        r_src = region(la, j) if j < a.world else set()
        retained, received = set(), set()
        for buf in range(8):
            tid, lin = lb[(j, buf)]
            for pos in np.nonzero(tid >= 0)[0][::3]:
                t = int(tid[pos])
                cd = [int(x) for x in np.unravel_index(int(lin[pos]), b.tensor_info(t)["shape"])]
                own = a.owners(buf % 4, t, cd, max_owners=256)
                r, sb, so = oracle.select_source(a, b, j, buf % 4, t, cd)
                assert (r, sb, so) in own
                owner_ranks = [o[0] for o in own]
                if j in owner_ranks:
                    assert r == j
                elif any(o // node == j // node for o in owner_ranks):
                    assert r // node == j // node
                (retained if r == j else received).add((buf % 4, t, int(lin[pos])))
        assert retained <= (r_src & r_dst)
        assert received <= (r_dst - r_src)
        assert not (retained & received)
        assert (r_src - r_dst).isdisjoint(r_dst)


# ----------------------------------------------------------------------------- closed forms

def test_pure_tp_change_closed_form():
    """TP 2 -> 4 on one pipeline stage, no DP: a column- or row-parallel tensor is cut into 4
    pieces of numel/4; destination tp rank j takes its quarter from source tp rank j//2.
    Replicated tensors come from the rule's pick among both source ranks."""
    m = cf.TINY_GPT
    a, b = oracle.Config(m, P(tp=2, zero=0)), oracle.Config(m, P(tp=4, zero=0))
    sharded = sum(a.tensor_info(t)["tp_axis"] >= 0 and int(np.prod(a.tensor_info(t)["shape"])) for t in range(a.num_tensors))
    repl = sum(a.tensor_info(t)["tp_axis"] < 0 and int(np.prod(a.tensor_info(t)["shape"])) for t in range(a.num_tensors))
    per_elem = 2 + 3 * 4
    for j in range(4):
        rb = oracle.route_bytes(a, b, j)
        want = np.zeros(2, dtype=np.uint64)
        want[j // 2] += sharded // 4 * per_elem
        # replicated: j in {0,1} owns them already; j in {2,3} has dp index 0 -> first owner
        want[j if j < 2 else 0] += repl * per_elem
        assert np.array_equal(rb, want)


def test_pure_dp_change_with_zero_closed_form():
    """DP 2 -> 4 with sharded fp32 state: volumes are overlaps of the even flat ranges."""
    m = cf.TINY_GPT
    a, b = oracle.Config(m, P(dp=2, zero=1)), oracle.Config(m, P(dp=4, zero=1))
    L = a.total_params
    la, lb = a.buffer_elems(0, 0), b.buffer_elems(0, 0)
    assert la == -(-L // 16) * 16 and lb == -(-L // 32) * 32
    for j in range(4):
        rb = oracle.route_bytes(a, b, j, buf_mask=0b1110)
        for i in range(2):
            lo = max(i * la // 2, j * lb // 4)
            hi = min((i + 1) * la // 2, (j + 1) * lb // 4, L)
            assert rb[i] == 3 * 4 * max(0, hi - lo)
        rb0 = oracle.route_bytes(a, b, j, buf_mask=0b0001)
        src = j if j < 2 else j % 2  # owner itself, else owners[dp index mod 2]
        assert rb0[src] == 2 * L and rb0.sum() == 2 * L


def test_pure_pp_change_moves_whole_tensors():
    m = cf.TINY_GPT
    a, b = oracle.Config(m, P(pp=2, zero=0)), oracle.Config(m, P(pp=4, zero=0))
    per = 2 + 12
    sizes = [int(np.prod(a.tensor_info(t)["shape"])) for t in range(a.num_tensors)]
    layer = [a.tensor_info(t)["layer"] for t in range(a.num_tensors)]
    for j in range(4):
        rb = oracle.route_bytes(a, b, j)
        want = np.zeros(2, dtype=np.uint64)
        for t, n in enumerate(sizes):
            sa = 0 if layer[t] < 2 else 1          # 4 layers over 2 stages; embedding first, head last
            sb = min(max(layer[t], 0), 3)
            if sb == j:
                want[sa] += n * per
        assert np.array_equal(rb, want)


# ----------------------------------------------------------------------------- worked examples

def _peers(a, b, rank, tensor_filter):
    """(sources rank receives from, destinations rank sends to) restricted to some tensors."""
    srcs, dsts = set(), set()
    for j in range(b.world):
        for buf in range(8):
            for off in range(b.buffer_elems(j, buf)):
                e = b.coord(j, buf, off)
                if e is None or not tensor_filter(e[0]):
                    continue
                r, _, _ = oracle.select_source(a, b, j, buf % 4, e[0], list(e[1]))
                if j == rank:
                    srcs.add(r)
                if r == rank:
                    dsts.add(j)
    return srcs, dsts


def test_figure4_worked_example_rank3():
    """Figure 4: rank 3 switching (TP,PP) = (2,2) -> (4,1) has a non-empty send, retain and
    receive set.  With TP as the fastest rank digit it holds the upper half of the stage-1
    layers; afterwards the last quarter of every layer.  It therefore keeps the last quarter
    of stage 1, sends the third quarter of stage 1 to rank 2 and receives the last quarter of
    stage 0 from rank 1."""
    m = cf.model(cf.FAMILY_GPT, 4, 8, 4, 4, 2, 16, 16)
    g = {k[8:]: int(v) for k, v in GOLD.items() if k.startswith("figure4_")}
    a = oracle.Config(m, P(tp=g["src_tp"], pp=g["src_pp"], zero=0))
    b = oracle.Config(m, P(tp=g["dst_tp"], pp=g["dst_pp"], zero=0))
    assert g["rank"] == 3
    sharded = lambda t: a.tensor_info(t)["tp_axis"] >= 0
    srcs, dsts = _peers(a, b, g["rank"], sharded)
    assert srcs == {g["receives_from"], g["rank"]} and dsts == {g["sends_to"], g["rank"]}
    rb = oracle.route_bytes(a, b, 3)
    assert rb[3] > 0 and rb[1] > 0 and oracle.send_bytes(a, b, 3)[2] > 0
    # the retained sharded part is exactly the stage-1 share of rank 3's new quarter
    stage1 = sum(int(np.prod(a.tensor_info(t)["shape"])) // 4 for t in range(a.num_tensors)
                 if sharded(t) and a.tensor_info(t)["layer"] >= 2)
    stage0 = sum(int(np.prod(a.tensor_info(t)["shape"])) // 4 for t in range(a.num_tensors)
                 if sharded(t) and a.tensor_info(t)["layer"] < 2)
    repl1 = sum(int(np.prod(a.tensor_info(t)["shape"])) for t in range(a.num_tensors)
                if not sharded(t) and a.tensor_info(t)["layer"] >= 2)
    assert rb[3] == (stage1 + repl1) * 14
    assert rb[1] == stage0 * 14


def test_figure6_sharded_optimizer_same_transition():
    """Figure 6: the same switch with two DP ranks and sharded optimizer state.  Both DP ranks
    of a TP/PP position hold the same bf16 shard but disjoint halves of the fp32 flat buffer;
    every half is routed to whichever rank owns those flat offsets afterwards."""
    m = cf.model(cf.FAMILY_GPT, 4, 8, 4, 4, 2, 16, 16)
    a = oracle.Config(m, P(tp=2, pp=2, dp=2, zero=1))
    b = oracle.Config(m, P(tp=4, pp=1, dp=2, zero=1))
    for tp in range(2):
        for pp in range(2):
            r0, r1 = tp + 2 * (0 + 2 * pp), tp + 2 * (1 + 2 * pp)
            assert np.array_equal(a.fill(r0, 0, 5), a.fill(r1, 0, 5))            # same params
            n = a.buffer_elems(r0, 1)
            e0 = {a.coord(r0, 1, o) for o in range(n)} - {None}
            e1 = {a.coord(r1, 1, o) for o in range(n)} - {None}
            assert e0 and e1 and not (e0 & e1)                                   # slices 1 and 2
    # every fp32 element has exactly one source and one destination; bytes are conserved
    recv = np.stack([oracle.route_bytes(a, b, j, buf_mask=0b1110) for j in range(8)])
    send = np.stack([oracle.send_bytes(a, b, i, buf_mask=0b1110) for i in range(8)])
    assert np.array_equal(recv, send.T)
    tp_repl = sum(int(np.prod(a.tensor_info(t)["shape"])) for t in range(a.num_tensors) if a.tensor_info(t)["tp_axis"] < 0)
    assert recv.sum() == 12 * (a.total_params + 3 * tp_repl)   # TP-replicated tensors: 4 copies
    # a flat half crosses tensor edges: some rank receives fp32 data from more than one peer
    assert max(int((recv[j] > 0).sum()) for j in range(8)) >= 2


def test_70b_mid_pipeline_rank_keeps_all_fp32_state():
    """Special case of the 70B switch (TP8,PP8,DP2) -> (TP8,PP4,DP4): for a rank away from the
    first and last stage the fp32 flat range covers the same five layers before and after,
    so every fp32 element is retained.  Checked on sampled offsets."""
    w = cf.WORKLOADS["gqa70b"]
    a, b = oracle.Config(w["model"], w["src"]), oracle.Config(w["model"], w["dst"])
    rng = np.random.default_rng(3)
    j = 43
    n = b.buffer_elems(j, 1)
    assert n == a.buffer_elems(j, 1)
    offs = np.concatenate([[0, 1, n - 2, n - 1], rng.integers(0, n, 3000)])
    for off in offs:
        e = b.coord(j, 1, int(off))
        assert e is not None
        r, sb, so = oracle.select_source(a, b, j, 1, e[0], list(e[1]))
        assert (r, sb, so) == (j, 1, int(off))
    # a first-stage rank is different: the embedding shifts its flat range off layer edges
    j = 11
    moved = 0
    for off in rng.integers(0, b.buffer_elems(j, 1), 500):
        e = b.coord(j, 1, int(off))
        if e is not None and oracle.select_source(a, b, j, 1, e[0], list(e[1]))[0] != j:
            moved += 1
    assert moved > 0


def test_boxfill_generator_matches_numpy_pattern():
    """The C box generator (inputs only) against the numpy twin of the pattern."""
    from datagen import boxfill
    rng = np.random.default_rng(11)
    for kind in (0, 1, 3):
        shape = [int(x) for x in rng.integers(2, 9, 4)]
        lo = [int(rng.integers(0, s)) for s in shape]
        ext = [int(rng.integers(1, s - l + 1)) for s, l in zip(shape, lo)]
        out = np.zeros(int(np.prod(ext)), dtype=np.uint16 if kind == 0 else np.uint32)
        boxfill.fill_box(1234, kind, 17, shape, lo, ext, out)
        idx = np.arange(int(np.prod(shape)), dtype=np.uint64).reshape(shape)
        idx = idx[lo[0]:lo[0] + ext[0], lo[1]:lo[1] + ext[1], lo[2]:lo[2] + ext[2], lo[3]:lo[3] + ext[3]]
        assert np.array_equal(out, pattern.word(1234, kind, 17, idx.ravel()))


# ----------------------------------------------------------------------------- declared readings, worked out by hand

def _declared():
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "declared_readings.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [x.strip() for x in line.split("=")]
            vals[k] = [int(x) for x in v.split(",")]
    return vals


@pytest.mark.parametrize("layers,pp", [(94, 8), (94, 4), (80, 8), (80, 4), (5, 3), (4, 4)])
def test_pipeline_split_matches_the_hand_table(layers, pp):
    """Layers per pipeline stage when the layer count is not a multiple of PP (a declared
    reading: the paper does not say): read off from where the oracle puts every layer's first
    tensor, against the table in tests/golden/declared_readings.txt."""
    want = _declared()[f"stage_sizes_{layers}_layers_pp{pp}"]
    assert len(want) == pp and sum(want) == layers
    m = cf.model(cf.FAMILY_GQA, layers, 8, 2, 2, 4, 16, 16)
    c = oracle.Config(m, P(pp=pp, zero=0))
    got = [0] * pp
    for l in range(layers):
        t = 1 + 6 * l                       # embedding, then six tensors per layer
        assert c.tensor_info(t)["layer"] == l and c.tensor_info(t - 1)["layer"] == l - 1
        (rank, _, _), = c.owners(0, t, (0, 0, 0, 0))
        got[c.rank_coords(rank)["pp"]] += 1
    assert got == want
    # embedding on the first stage, final norm and output layer on the last
    assert c.rank_coords(c.owners(0, 0, (0, 0, 0, 0))[0][0])["pp"] == 0
    for t in (c.num_tensors - 2, c.num_tensors - 1):
        assert c.rank_coords(c.owners(0, t, (0, 0, 0, 0))[0][0])["pp"] == pp - 1


@pytest.mark.parametrize("experts,ep", [(128, 8), (128, 16), (8, 4), (6, 3)])
def test_expert_blocks_match_the_hand_table(experts, ep):
    """Experts are cut over EP in contiguous blocks (declared reading): first expert of every
    block against the table, both for the grid placement and for EP carved out of TP x DP."""
    first = _declared()[f"first_expert_of_block_{experts}_experts_ep{ep}"]
    assert len(first) == ep
    m = cf.model(cf.FAMILY_MOE, 1, 8, 2, 2, 4, 0, 16, experts=experts, expert_ffn=4)
    for par in (P(ep=ep, zero=0), P(tp=1, dp=ep, ep=ep, zero=0, ep_placement=1)):
        c = oracle.Config(m, par)
        got = {}
        for e in range(experts):
            t = 1 + 7 + 2 * e                # embedding, seven dense tensors of layer 0, two tensors per expert
            assert c.tensor_info(t)["expert"] == e
            (rank, _, _), = c.owners(0, t, (0, 0, 0, 0))
            got.setdefault(c.rank_coords(rank)["ep"], []).append(e)
        assert [min(got[k]) for k in range(ep)] == first
        assert all(got[k] == list(range(first[k], first[k] + experts // ep)) for k in range(ep))


def test_carved_expert_ranks_follow_the_hand_example():
    """EP carved out of TP x DP, (TP, PP, DP, EP) = (2, 1, 4, 2) on 8 ranks: position q = tp + 2*dp
    inside the stage, ep = q mod 2, expert data-parallel index = q div 2 (table in
    tests/golden/declared_readings.txt)."""
    d = _declared()
    m = cf.model(cf.FAMILY_MOE, 1, 8, 2, 2, 4, 0, 16, experts=4, expert_ffn=4)
    c = oracle.Config(m, P(tp=2, pp=1, dp=4, ep=2, ep_placement=1))
    assert c.world == 8
    assert [c.rank_coords(r)["ep"] for r in range(8)] == d["carved_tp2_dp4_ep2_ep_of_rank"]
    assert [c.rank_coords(r)["edp"] for r in range(8)] == d["carved_tp2_dp4_ep2_edp_of_rank"]
    assert [c.rank_coords(r)["tp"] for r in range(8)] == d["carved_tp2_dp4_ep2_tp_of_rank"]
    assert [c.rank_coords(r)["ddp"] for r in range(8)] == d["carved_tp2_dp4_ep2_dp_of_rank"]


def test_source_rule_follows_the_hand_examples():
    """The choice among replicas (itself, else its node's owners, else all; index = destination
    data-parallel index modulo count) on the three examples evaluated by hand in
    tests/golden/declared_readings.txt."""
    d = _declared()
    m = cf.TINY_GPT                       # 4 layers, hidden 16, ffn 32; fc1.w of layer 0 is tensor 9: (32, 16), TP on rows
    fc1 = 1 + 0 * 12 + 8
    assert list(oracle.Config(m, P(tp=1)).tensor_info(fc1)["shape"][2:]) == [m["ffn"], m["hidden"]]
    for gpn in (2, 8):
        a = oracle.Config(m, P(tp=2, pp=1, dp=2, zero=0, gpus_per_node=gpn))
        b = oracle.Config(m, P(tp=1, pp=1, dp=4, zero=0, gpus_per_node=gpn))
        for half, row in (("first", 3), ("second", 20)):
            got = [oracle.select_source(a, b, j, 0, fc1, (0, 0, row, 5))[0] for j in range(4)]
            assert got == d[f"select_tp2dp2_to_dp4_gpn{gpn}_{half}_half"], (gpn, half, got)
    a = oracle.Config(m, P(tp=1, pp=2, dp=4, zero=0, gpus_per_node=4))
    b = oracle.Config(m, P(tp=1, pp=1, dp=8, zero=0, gpus_per_node=4))
    for layer in (0, 3):
        t = 1 + layer * 12 + 8
        got = [oracle.select_source(a, b, j, 1, t, (0, 0, 7, 2))[0] for j in range(8)]
        assert got == d[f"select_pp2dp4_to_dp8_gpn4_layer{layer}"], (layer, got)
    a = oracle.Config(m, P(tp=1, pp=1, dp=2, zero=0, gpus_per_node=8))
    b = oracle.Config(m, P(tp=2, pp=1, dp=2, zero=0, gpus_per_node=8))
    ln1 = 1                               # ln1.w of layer 0: a vector of `hidden` elements, replicated over TP
    got = [oracle.select_source(a, b, j, 0, ln1, (0, 0, 0, 9))[0] for j in range(4)]
    assert got == d["select_dp2_to_tp2dp2_gpn8_replicated"], got


# ----------------------------------------------------------------------------- per-peer buffers

@pytest.mark.parametrize("name,m,p", LAYOUT_CASES, ids=[c[0] for c in LAYOUT_CASES])
def test_pieces_match_the_box_decomposition(name, m, p):
    """The oracle's per-element piece rule (coarsest aligned storage unit inside the rank's flat
    range) against the numpy decomposition of every storage block's range into the fewest boxes:
    the same partition of every buffer."""
    c = oracle.Config(m, p)
    pcs = textbook.pieces(m, p)
    for rank in range(c.world):
        for buf in range(8):
            n = c.buffer_elems(rank, buf)
            groups = {}
            for off in range(n):
                key = c.piece_key(rank, buf, off)
                if key is not None:
                    groups.setdefault((c.coord(rank, buf, off)[0],) + key, []).append(off)
            got = sorted(tuple(v) for v in groups.values())
            want = sorted(tuple(sorted(offs.tolist())) for _, offs, _ in pcs[(rank, buf)])
            assert got == want, (rank, buf)
            # and each piece is an axis-aligned box of its tensor
            for t, offs, addr in pcs[(rank, buf)]:
                shape = c.tensor_info(t)["shape"]
                cd = np.stack(np.unravel_index(addr, shape))
                assert int(np.prod(cd.max(axis=1) - cd.min(axis=1) + 1)) == addr.size


def _box_based_recv_buffer(a, b, m, pa, pb, j, seed, salt, through, pad_byte=0xA5):
    """The receive buffer of rank j built from boxes: every (source piece x destination piece)
    intersection whose selected source is that source rank, ordered by (source, kind 1 2 3 0,
    tensor, lo corner), serialised row-major, 16-byte aligned."""
    pcs_a, pcs_b = textbook.pieces(m, pa), textbook.pieces(m, pb)
    by_tensor = {}
    for (i, buf), lst in pcs_a.items():
        for t, _, addr in lst:
            by_tensor.setdefault((buf % 4, t), []).append((i, np.sort(addr)))
    routed = []
    for buf in range(8):
        kind = buf % 4
        for t, _, addr_b in pcs_b[(j, buf)]:
            shape = a.tensor_info(t)["shape"]
            for i, addr_a in by_tensor.get((kind, t), []):
                x = np.intersect1d(addr_a, addr_b, assume_unique=True)
                if not x.size:
                    continue
                picks = {oracle.select_source(a, b, j, kind, t, [int(v) for v in np.unravel_index(int(e), shape)])[0]
                         for e in (x[0], x[-1], x[x.size // 2])}
                assert len(picks) == 1
                if picks != {i} or (i == j and not through):
                    continue
                routed.append((i, (kind + 3) & 3, t, int(x[0]), kind, x))
    routed.sort(key=lambda r: r[:4])
    out, seg = [], np.zeros(a.world + 1, dtype=np.uint64)
    pos = 0
    for i, _, t, _, kind, x in routed:
        words = pattern.word(pattern.seed_for_rank(seed, salt, i), kind, t, x.astype(np.uint64))
        raw = words.astype(np.uint16 if kind == 0 else np.uint32).tobytes()
        raw += bytes([pad_byte]) * ((-len(raw)) % 16)
        out.append(raw)
        pos += len(raw)
        seg[i + 1:] = pos
    return np.frombuffer(b"".join(out), dtype=np.uint8), seg


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_recv_payload_equals_the_box_based_formulation(name, m, pa, pb):
    """Algorithm 1, PackData: the per-element construction of a receive buffer against the
    box-based one; the order inside a buffer is a convention of this repository, stated twice."""
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    for through in (False, True):
        for j in range(b.world):
            got, seg = oracle.recv_payload(a, b, j, seed=31, rank_salt=0x77, through=through)
            want, wseg = _box_based_recv_buffer(a, b, m, pa, pb, j, 31, 0x77, through)
            assert np.array_equal(seg, wseg), (j, through)
            assert np.array_equal(got, want), (j, through)
            if not through:
                rb = oracle.route_bytes(a, b, j)
                for i in range(a.world):
                    nbytes = int(seg[i + 1] - seg[i])
                    assert nbytes % 16 == 0
                    if i != j:
                        assert int(rb[i]) <= nbytes
                        assert (nbytes == 0) == (rb[i] == 0)


def test_recv_payload_of_a_pipeline_merge_written_out_by_hand():
    """A case in which order A13 can be written down without any box logic: (TP, PP, DP) = (1, 2, 1)
    -> (1, 1, 1) without ZeRO.  Rank 0 keeps stage 0 and receives every tensor of stage 1 whole
    from rank 1: the buffer is, for the kinds in the order 1, 2, 3, 0 and the tensors of stage 1 in
    ascending id order, the tensor's words in row-major order, each tensor padded to 16 bytes."""
    m = cf.TINY_GPT
    a, b = oracle.Config(m, P(tp=1, pp=2, dp=1, zero=0)), oracle.Config(m, P(tp=1, pp=1, dp=1, zero=0))
    got, seg = oracle.recv_payload(a, b, 0, seed=77, rank_salt=0x33, pad_byte=0xEE)
    first = 1 + (m["layers"] // 2) * 12                      # first tensor of stage 1 (12 tensors per GPT layer)
    want = []
    for kind in (1, 2, 3, 0):
        for t in range(first, a.num_tensors):
            n = int(np.prod(a.tensor_info(t)["shape"]))
            words = pattern.word(pattern.seed_for_rank(77, 0x33, 1), kind, t, np.arange(n, dtype=np.uint64))
            raw = words.astype(np.uint16 if kind == 0 else np.uint32).tobytes()
            want.append(raw + bytes([0xEE]) * ((-len(raw)) % 16))
    want = np.frombuffer(b"".join(want), dtype=np.uint8)
    assert list(seg) == [0, 0, len(want)]
    assert np.array_equal(got, want)


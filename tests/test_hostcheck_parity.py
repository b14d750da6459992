"""CPU build of the library's mapper / planner / tile-geometry code against the oracle.

The product runs this code only inside HIP kernels.  Here the same per-item functions are
compiled for the host (tests/hostcheck) with bounds checks and UBSan, so that index errors are
found on a machine without a GPU.  The GPU parity tests (test_gpu_parity.py) run the identical
procedures through the real library.
"""
import ctypes as C

import numpy as np
import pytest

import parity
from datagen import configs as cf
from hostcheck import build as hc_build
from paper_2605_18815_amd.binding import Library, VpsError
from test_oracle_pins import ALL_TRANSITIONS, TRANSITIONS

P = cf.parallel


@pytest.fixture(scope="module")
def hlib():
    import os
    # VPSH_LIB lets the mutation test of the parity suite load a deliberately broken CPU build
    return Library(os.environ.get("VPSH_LIB") or hc_build.build(), prefix="vpsh_")


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_all_ranks_resident(hlib, name, m, pa, pb):
    mem = parity.HostMem(hlib)
    out = parity.run_all_ranks(hlib, mem, m, pa, pb, seed=0x5EED + len(name))
    assert out["boxes"] > 0


MEDIUM = [
    ("mid-moe-to-transposed", cf.MID_MOE, P(tp=2, pp=1, dp=1, ep=2), P(tp=1, pp=2, dp=2, ep=1, expert_layout=1)),
    ("mid-moe-from-transposed", cf.MID_MOE, P(tp=1, pp=2, dp=1, ep=4, expert_layout=1), P(tp=2, pp=1, dp=2, ep=2)),
    ("mid-moe-both-transposed", cf.MID_MOE, P(tp=2, pp=1, dp=2, ep=1, expert_layout=1), P(tp=1, pp=1, dp=2, ep=2, expert_layout=1, flat_order=1)),
    ("mid-gpt-tp-blocked", cf.MID_GPT, P(tp=3, pp=1, dp=2), P(tp=2, pp=2, dp=1, qkv_layout=1)),
]


@pytest.mark.parametrize("name,m,pa,pb", MEDIUM, ids=[c[0] for c in MEDIUM])
def test_medium_shapes_all_ranks(hlib, name, m, pa, pb):
    out = parity.run_all_ranks(hlib, parity.HostMem(hlib), m, pa, pb, seed=0xC0FFEE)
    assert out["boxes"] > 0


STAGED = [("gpt-zero-to-replicated", 0), ("gpt-blocked-rev", 1), ("gpt-world-grows", 2), ("moe-transposed", 3), ("moe-odd", 4)]


@pytest.mark.parametrize("name,budget_kind", [(n, k) for n, _ in STAGED for k in ("tiny", "mid", "exact", "huge")],
                         ids=[f"{n}-{k}" for n, _ in STAGED for k in ("tiny", "mid", "exact", "huge")])
def test_staged_xor_exchange(hlib, name, budget_kind):
    """Memory-aware stages and the XOR step order (Algorithm 1) give the same final state."""
    _, m, pa, pb = [t for t in TRANSITIONS if t[0] == name][0]
    probe = parity.run_staged(hlib, parity.HostMem(hlib), m, pa, pb, seed=5, budget=1 << 60)
    assert probe["stages"] == 1
    busy = [c for c in probe["costs"][1:] if c]
    # "exact": the first two steps with traffic fill the budget to the byte and must share a stage
    budget = {"tiny": 1, "mid": max(probe["max_cost"] * 2, 1), "exact": sum(busy[:2]) or 1, "huge": 1 << 60}[budget_kind]
    out = parity.run_staged(hlib, parity.HostMem(hlib), m, pa, pb, seed=6, budget=budget)
    if budget_kind == "tiny":
        assert out["stages"] >= 2 and out["scratch"] < out["one_shot"] * 2
    if budget_kind == "mid":
        assert 1 <= out["stages"] <= probe["steps"]


COLLECTIVE_CASES = [
    ("broadcast-dp-grows", cf.TINY_GPT, P(dp=1, zero=0), P(dp=4, zero=0), 2),
    ("scatter-tp-grows", cf.TINY_GPT, P(tp=1, zero=0), P(tp=4, zero=0), 3),
    ("scatter-zero-on", cf.TINY_GPT, P(dp=1, zero=0), P(dp=4, zero=1), 3),
    ("gather-tp-shrinks", cf.TINY_GPT, P(tp=4, zero=0), P(tp=1, zero=0), 4),
    ("p2p-tp-pp", cf.TINY_GPT, P(tp=4, pp=2, dp=1), P(tp=2, pp=4, dp=1), 1),
]


@pytest.mark.parametrize("name,m,pa,pb,expect", COLLECTIVE_CASES, ids=[c[0] for c in COLLECTIVE_CASES])
def test_collective_intent_cases(hlib, name, m, pa, pb, expect):
    """Algorithm 1, OptimizePrimitives: the device classification against plain Python sets."""
    counts = parity.run_classify(hlib, m, pa, pb)
    assert counts[expect] > 0, counts


@pytest.mark.parametrize("name,m,pa,pb", TRANSITIONS, ids=[c[0] for c in TRANSITIONS])
def test_collective_intent_matches_bruteforce(hlib, name, m, pa, pb):
    counts = parity.run_classify(hlib, m, pa, pb)
    assert counts.sum() == 4 * len(__import__("textbook").inventory(m))


def test_parity_subset_under_address_sanitizer():
    """The CPU build again with AddressSanitizer, in a child process that preloads its runtime:
    heap bounds of every table the mapper, the planner, the stage plan and the classification
    touch, and the lifetime of what the handles own (a backend that goes out of scope takes along
    whatever it was not told to hand over)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    select = ("error_codes or staged_xor_exchange or beyond_the_counting_limit or single_rank_share or routes_only "
              "or (all_ranks_resident and (odd or carved)) or collective_intent_cases or piece_queries")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(root, "tests", "test_hostcheck_parity.py"), "-x", "-q",
                          "-k", select, "-p", "no:cacheprovider"], env=hc_build.asan_env(), cwd=root, capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]


@pytest.mark.parametrize("m", [cf.TINY_GPT, cf.TINY_GQA, cf.TINY_MOE, cf.ODD_MOE, cf.MID_MOE], ids=["gpt", "gqa", "moe", "odd-moe", "mid-moe"])
def test_tensor_ids_by_group(hlib, m):
    """The planner of all-ranks transitions enumerates the dense and the expert tensors separately,
    from the layout of the inventory; the ids must be those whose pieces live in the group's
    buffers, ascending."""
    import ctypes as C
    from paper_2605_18815_amd import binding as B
    par = P(tp=2, dp=2, ep=2 if m["family"] == cf.FAMILY_MOE else 1)
    pieces = hlib.describe_config(m, par).get_pieces()
    nt = int(pieces["tensor"].max()) + 1
    for group in (0, 1):
        want = sorted(set(int(t) for t in pieces["tensor"][pieces["buf"] // 4 == group]))
        out = (C.c_int32 * nt)()
        n = hlib._dll.vpsh_group_tensors(C.byref(B.model_desc(m)), C.byref(B.parallel_desc(par)), group, out, nt)
        assert n == len(want) and list(out[:n]) == want
    assert sorted(set(int(t) for t in pieces["tensor"])) == list(range(nt))


def test_piece_queries_then_planning(hlib):
    """Regression: the piece table is built on the first piece query, by a backend that lives only
    for that call; it has to hand the table over to the configuration (once, a second query reuses
    it), and the tables of later plans must not land in the same memory."""
    ca, cb = hlib.describe_config(cf.TINY_MOE, P(tp=1, pp=4, dp=2, ep=2)), hlib.describe_config(cf.TINY_MOE, P(tp=1, pp=2, dp=2, ep=4))
    n = ca.num_pieces
    first = ca.get_pieces()
    plans = [hlib.plan_intersections(ca, cb, r) for r in (-1, 0, 5)]
    assert ca.num_pieces == n and np.array_equal(ca.get_pieces(), first)
    assert cb.num_pieces > 0 and all(p.num_boxes > 0 for p in plans)
    parity.run_all_ranks(hlib, parity.HostMem(hlib), cf.TINY_MOE, P(tp=1, pp=4, dp=2, ep=2), P(tp=1, pp=2, dp=2, ep=4), seed=12)
    assert np.array_equal(ca.get_pieces(), first)


def test_routes_only_plan_refuses_copies(hlib):
    from paper_2605_18815_amd import binding as B
    ca = hlib.describe_config(cf.TINY_GPT, P(tp=2, dp=2))
    cb = hlib.describe_config(cf.TINY_GPT, P(tp=1, dp=4, zero=0))
    plan = hlib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_ROUTES_ONLY)
    full = hlib.plan_intersections(ca, cb, -1)
    assert plan.num_boxes == full.num_boxes and np.array_equal(plan.get_boxes(), full.get_boxes())
    assert plan.stats()["num_pack_tiles"] == 0
    mem = parity.HostMem(hlib)
    bufs = [mem.ptr(mem.alloc(max(ca.buffer_bytes(r % 4, b), cb.buffer_bytes(r % 4, b)))) for r in range(4) for b in range(8)]
    with pytest.raises(VpsError) as e:
        hlib.apply_transition(plan, -1, bufs, bufs, mem.ptr(mem.alloc(1 << 20)), 1 << 20)
    assert e.value.code == B.ERR_INVALID_ARG
    with pytest.raises(VpsError):
        hlib.plan_intersections_ex(ca, cb, -1, flags=8)
    own_peer = hlib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_THROUGH_BUFFERS)
    with pytest.raises(VpsError) as e:
        hlib.stage_exchange(own_peer, 1 << 20)
    assert e.value.code == B.ERR_INVALID_ARG


SINGLE = [
    ("gpt-zero-to-replicated", 0), ("gpt-zero-to-replicated", 3), ("gpt-tp-pp", 5), ("gpt-blocked-rev", 2),
    ("gpt-odd", 1), ("gpt-world-grows", 11), ("gpt-world-grows", 3), ("gqa", 6), ("moe-ep", 9),
    ("moe-transposed", 3), ("moe-odd", 7), ("moe-carved-ep-shrinks", 5), ("moe-carved-ep-grows", 13), ("moe-grid-to-carved", 3),
    ("moe-odd-carved", 4),
]


@pytest.mark.parametrize("name,rank", SINGLE, ids=[f"{n}-r{r}" for n, r in SINGLE])
def test_single_rank_share(hlib, name, rank):
    _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == name][0]
    mem = parity.HostMem(hlib)
    parity.run_single_rank(hlib, mem, m, pa, pb, rank, seed=0xBEEF + rank)


THROUGH = [("gpt-zero-to-replicated", 3), ("gpt-tp-pp", 5), ("gpt-world-grows", 3), ("moe-transposed", 3), ("moe-odd", -1),
           ("gpt-blocked-rev", -1), ("moe-carved-ep-shrinks", -1), ("moe-grid-to-carved", 6)]


@pytest.mark.parametrize("name,rank", THROUGH, ids=[f"{n}-r{r}" for n, r in THROUGH])
def test_rank_as_its_own_peer(hlib, name, rank):
    """VPS_PLAN_THROUGH_BUFFERS: retained data travels through the rank's own segment; the
    destination bits and the payload in the send buffer stay those of the oracle."""
    _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == name][0]
    mem = parity.HostMem(hlib)
    if rank < 0:
        parity.run_all_ranks(hlib, mem, m, pa, pb, seed=0xD00D, through=True)
    else:
        parity.run_single_rank(hlib, mem, m, pa, pb, rank, seed=0xD00D + rank, through=True)


def run_staged_long_runs(lib, mem_factory):
    """Regression: runs longer than a tile whose pack descriptors the staged exchange moves to other
    places of the scratch area (here to offset 0, below the phase their cuts were made for) keep
    their cuts and their number of tiles."""
    pa = P(tp=3, pp=2, dp=2, zero=1, gpus_per_node=8, qkv_layout=1, flat_order=1)
    pb = P(tp=3, pp=1, dp=3, zero=1, gpus_per_node=4)
    for tile, budget in ((4096, 1), (8192, 1 << 14), (8192, 1 << 18)):
        lib.set_tile_bytes(tile)
        try:
            out = parity.run_staged(lib, mem_factory(), cf.MID_GPT, pa, pb, seed=42000993, budget=budget)
        finally:
            lib.set_tile_bytes(8192)
        assert out["stages"] > 1


def test_staged_exchange_moves_long_runs(hlib):
    run_staged_long_runs(hlib, lambda: parity.HostMem(hlib))


# (limit of the counting path, log2 of the work bound of the pair-by-pair ordering: 32 = the
# default, 0 = all-ranks plans always take the radix sort, 1 = they start pair by pair, find the
# bound exceeded and plan again with the sort)
BEYOND = [(1, 32), (7, 32), (64, 32), (1, 0), (7, 1)]


def run_plans_beyond_the_counting_limit(lib, mem_factory, limit, pair_work):
    from paper_2605_18815_amd import binding as B
    lib.set_option(B.OPT_SMALL_PLAN_BOXES, limit)
    lib.set_option(B.OPT_PAIR_ORDER_WORK, pair_work)
    try:
        for name, rank in (("gpt-zero-to-replicated", -1), ("gpt-blocked-rev", -1), ("moe-odd", -1), ("moe-carved-ep-grows", -1),
                           ("gpt-world-grows", -1), ("gpt-tp-pp", 5), ("moe-transposed", 3), ("gpt-world-grows", 11)):
            _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == name][0]
            if rank < 0:
                # twice: the second plan of a transition knows its size beforehand, and a large
                # all-ranks plan then counts its boxes per pair while it emits them
                for again in range(2):
                    parity.run_all_ranks(lib, mem_factory(), m, pa, pb, seed=0x1A46E + limit + again, through=(limit == 7))
            else:
                parity.run_single_rank(lib, mem_factory(), m, pa, pb, rank, seed=0x1A46E + rank, through=(limit == 7))
        _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == "moe-ep"][0]
        parity.run_staged(lib, mem_factory(), m, pa, pb, seed=3, budget=1 << 12)
        parity.run_classify(lib, m, pa, pb)
    finally:
        lib.set_option(B.OPT_SMALL_PLAN_BOXES, 8192)
        lib.set_option(B.OPT_PAIR_ORDER_WORK, 32)


@pytest.mark.parametrize("limit,pair_work", BEYOND, ids=[f"{a}-{['sort', 'bound-exceeded'][b] if b < 2 else 'pairs'}" for a, b in BEYOND])
def test_plans_beyond_the_counting_limit(hlib, limit, pair_work):
    """Plans with more boxes than the counting path takes: all-ranks plans are ordered pair by pair
    (or by the radix sort), single-rank plans by the radix sort, positions by sums and scans: same
    boxes, same buffers.  The limit is lowered so that tiny models reach those paths (and, at 64,
    so that some plans take one path and some the other)."""
    run_plans_beyond_the_counting_limit(hlib, lambda: parity.HostMem(hlib), limit, pair_work)


@pytest.mark.parametrize("name", ["gpt-zero-to-replicated", "gpt-world-grows", "moe-odd", "moe-carved-ep-grows"])
def test_sender_and_receiver_agree_on_segments(hlib, name):
    """Single-rank plans of the two ends of every segment list the same boxes at the same offsets."""
    import oracle
    _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == name][0]
    wa, wb = oracle.Config(m, pa).world, oracle.Config(m, pb).world
    assert parity.check_cross_plan_segments(hlib, m, pa, pb, [(i, j) for i in range(wa) for j in range(wb)]) > 0


def test_toy_workload_all_ranks(hlib):
    w = cf.WORKLOADS["toy"]
    mem = parity.HostMem(hlib)
    out = parity.run_all_ranks(hlib, mem, w["model"], w["src"], w["dst"], seed=cf.seed_of("toy"))
    assert out["moved"] > 0


@pytest.mark.parametrize("tile", [4096, 65536])
def test_tile_size_does_not_change_results(hlib, tile):
    hlib.set_tile_bytes(tile)
    try:
        _, m, pa, pb = TRANSITIONS[3]
        parity.run_all_ranks(hlib, parity.HostMem(hlib), m, pa, pb, seed=77)
        w = cf.WORKLOADS["toy"]
        parity.run_single_rank(hlib, parity.HostMem(hlib), w["model"], w["src"], w["dst"], 1, seed=78)
    finally:
        hlib.set_tile_bytes(8192)


def test_split_linear_range_properties(hlib):
    """A linear range over a k-D row-major array splits into at most 2k-1 boxes whose volumes
    sum to the range length and which tile it in order (Section 4.2.2: flat ranges cut across
    tensor boundaries)."""
    rng = np.random.default_rng(5)
    f = hlib._dll.vpsh_split_linear_range
    f.restype = C.c_int
    f.argtypes = [C.POINTER(C.c_int64), C.c_uint64, C.c_uint64, C.POINTER(C.c_int64), C.c_int]
    for _ in range(3000):
        dims = [int(x) for x in rng.integers(1, 7, 4)]
        total = int(np.prod(dims))
        v0 = int(rng.integers(0, total))
        v1 = int(rng.integers(v0 + 1, total + 1))
        out = (C.c_int64 * 60)()
        n = f((C.c_int64 * 4)(*dims), v0, v1, out, 20)
        k = sum(1 for d in dims if d > 1) or 1
        assert 1 <= n <= 2 * k - 1 or (n <= 7 and k == 4), (dims, v0, v1, n)
        assert n <= max(1, 2 * k - 1)
        st = [dims[1] * dims[2] * dims[3], dims[2] * dims[3], dims[3], 1]
        cur = v0
        for i in range(n):
            start, axis, cnt = out[3 * i], out[3 * i + 1], out[3 * i + 2]
            assert start == cur and cnt >= 1
            assert start % st[axis] == 0                       # aligned to the unit it spans
            assert (start // st[axis]) % dims[axis] + cnt <= dims[axis]  # stays inside the axis
            cur += cnt * st[axis]
        assert cur == v1


def test_library_exports_every_declared_symbol():
    """The C ABI library loads without a GPU and exports every function include/vps.h declares."""
    import os
    import re
    import ctypes
    from paper_2605_18815_amd import build as lib_build
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "vps.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(vps_[a-z_]+)\s*\(", header))
    assert {"vps_describe_config", "vps_plan_intersections", "vps_pack", "vps_unpack", "vps_apply_transition"} <= names
    dll = ctypes.CDLL(lib_build.library_path())
    for n in sorted(names):
        assert hasattr(dll, n), f"{n} is declared in include/vps.h but not exported"
    # and the binding wraps all of them
    from paper_2605_18815_amd.binding import Library
    assert {"vps_" + e for e in Library.EXPORTS} == names


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/vps.h compiles as strict C99, the struct sizes are those the binding assumes, and a
    C program linked against the library can call it (argument errors only: no GPU needed)."""
    import os
    import subprocess
    from paper_2605_18815_amd import build as lib_build
    from paper_2605_18815_amd.binding import BOX_DTYPE, PIECE_DTYPE
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib = lib_build.library_path()
    src = tmp_path / "use_vps.c"
    src.write_text('''
#include <stdio.h>
#include <string.h>
#include "vps.h"
int main(void)
{
    vps_model_desc m;
    vps_parallel_desc p;
    vps_config* c = 0;
    memset(&m, 0, sizeof m);
    memset(&p, 0, sizeof p);
    printf("%d %d ", (int)sizeof(vps_piece), (int)sizeof(vps_box));
    printf("%d ", vps_describe_config(&m, &p, -1, &c));      /* all-zero descriptors: invalid argument */
    printf("%d ", vps_describe_config(0, &p, -1, &c));
    printf("%d ", vps_set_tile_bytes(1000));
    printf("%d\\n", vps_last_error()[0] != 0);
    return 0;
}
''')
    exe = tmp_path / "use_vps"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe), lib, "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()
    assert [int(v) for v in out] == [PIECE_DTYPE.itemsize, BOX_DTYPE.itemsize, -1, -1, -1, 1]


def test_product_calls_fail_loudly_without_a_gpu(gpu_available):
    """No CPU fallback: on a machine without a GPU every compute entry point reports VPS_ERR_HIP."""
    if gpu_available:
        pytest.skip("a GPU is present")
    import paper_2605_18815_amd as vps
    from paper_2605_18815_amd import binding as B
    lib = vps.load()
    with pytest.raises(VpsError) as e:
        lib.describe_config(cf.TINY_GPT, P(tp=2))
    assert e.value.code == B.ERR_HIP
    with pytest.raises(VpsError) as e:   # argument errors are still reported first
        lib.describe_config(cf.TINY_GPT, P(tp=3))
    assert e.value.code == B.ERR_INDIVISIBLE


EDGE_TRANSITIONS = [
    ("identity", cf.TINY_GPT, P(tp=2, pp=2, dp=2), P(tp=2, pp=2, dp=2)),
    ("world-shrinks", cf.TINY_GPT, P(tp=4, pp=2, dp=2), P(tp=2, pp=1, dp=2)),
    ("zero-off-to-on", cf.TINY_GQA, P(tp=2, dp=3, zero=0), P(tp=2, dp=3, zero=1)),
    ("single-rank-worlds", cf.TINY_GPT, P(), P(zero=0)),
    ("moe-dense-only-change", cf.TINY_MOE, P(tp=1, pp=2, dp=2, ep=2), P(tp=1, pp=2, dp=1, ep=4)),
]


@pytest.mark.parametrize("name,m,pa,pb", EDGE_TRANSITIONS, ids=[c[0] for c in EDGE_TRANSITIONS])
def test_edge_transitions(hlib, name, m, pa, pb):
    """Degenerate cases: nothing moves, ranks that exist on one side only, empty peer buffers."""
    out = parity.run_all_ranks(hlib, parity.HostMem(hlib), m, pa, pb, seed=3)
    if name == "identity":
        assert out["moved"] == 0 and out["stats"]["num_send_boxes"] == 0
    import oracle
    wa, wb = oracle.Config(m, pa).world, oracle.Config(m, pb).world
    for r in sorted({0, wa - 1, wb - 1, max(wa, wb) - 1}):
        parity.run_single_rank(hlib, parity.HostMem(hlib), m, pa, pb, r, seed=4)


def test_tensors_beyond_32_bit_sizes(hlib):
    """A 162 B-parameter model whose embedding has 6.5e10 elements and whose rank shares reach
    100 GB: offsets, strides and tile counts beyond 32 bits (the CPU build runs under UBSan).
    Planning only; every box is validated by the oracle on corners and random interior points."""
    import oracle
    from paper_2605_18815_amd import binding as B
    m = cf.model(cf.FAMILY_GQA, 2, 32768, 256, 32, 128, 131072, 2_000_000)
    pa, pb = P(tp=8, pp=1, dp=4), P(tp=4, pp=2, dp=4, qkv_layout=1)
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    assert a.total_params > 1.6e11
    ca, cb = hlib.describe_config(m, pa), hlib.describe_config(m, pb)
    routes = hlib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_ROUTES_ONLY)
    parity.validate_boxes(a, b, routes.get_boxes(), -1, samples=16, plan=routes)
    # rank 0 with copy descriptors and the tile table: its embedding shard is one contiguous
    # stretch of 8.2e9 elements, more than a 32-bit extent holds
    out = parity.dry_run_single_rank(hlib, m, pa, pb, 0)
    assert out["info"]["retain_total"] > 8e10 and out["sent"] > 2e10


# (workload, rank, layout fields changed on both sides, plan through the buffers, tile bytes)
FULL_SIZE_SHARES = [("gqa8b", 5, {}, False, 8192), ("gqa70b", 11, {}, False, 8192), ("gqa70b", 43, {}, False, 8192),
                    ("gqa70b", 11, {"flat_order": 1}, False, 8192), ("moe235b", 37, {}, False, 8192),
                    ("gpt1p3b", 29, {}, False, 8192), ("gqa70b", 11, {}, True, 8192), ("moe235b", 37, {}, True, 8192),
                    ("gqa70b", 11, {}, False, 4096), ("gqa8b", 5, {"qkv_layout": 1}, False, 1 << 20),
                    ("gqa70b-odd", 11, {}, False, 8192)]


@pytest.mark.parametrize("name,rank,over,through,tile", FULL_SIZE_SHARES,
                         ids=[f"{n}-r{r}{'-var' if o else ''}{'-through' if t else ''}-{tb}" for n, r, o, t, tb in FULL_SIZE_SHARES])
def test_full_size_shares_dry_run(hlib, name, rank, over, through, tile):
    """The benchmark's rank shares at full size on the CPU build: the whole tile table is walked
    without memory behind it; accesses stay inside the buffers and the writes cover every
    destination payload byte and every outgoing byte exactly once."""
    w = cf.workload(name)
    pa, pb = dict(w["src"]), dict(w["dst"])
    pa.update(over)
    pb.update(over)
    hlib.set_tile_bytes(tile)
    try:
        out = parity.dry_run_single_rank(hlib, w["model"], pa, pb, rank, box_samples=4, through=through)
    finally:
        hlib.set_tile_bytes(8192)
    assert out["written"] > 0
    # tile quality: no workgroup without work, and the bulk of the bytes in tiles of at least half
    # the tile size (small tiles cost a workgroup launch each)
    tiles = out["tiles"]
    assert tiles["empty"][0] == 0 and tiles["elementwise"][0] == 0
    total = sum(b for _, b in tiles.values())
    assert total == out["written"]
    big = tiles["full_run"][1] + tiles["few_runs"][1] + tiles["many_runs"][1]
    assert big >= 0.95 * total, tiles
    # long runs are cut at 256-byte boundaries of the destination buffer, wherever the run starts:
    # only the first piece of a run may begin elsewhere (these shares have one run per box)
    if name.startswith("gqa"):
        assert out["unaligned_run_tiles"] <= 2 * out["stats"]["num_boxes"], out["unaligned_run_tiles"]


@pytest.mark.parametrize("name,budget", [("toy", None), ("toy", 1), ("toy", 1 << 60), ("gpt1p3b", None), ("gpt1p3b", 64 << 20)],
                         ids=["toy-oneshot", "toy-tiny-budget", "toy-one-stage", "gpt1p3b-oneshot", "gpt1p3b-64MiB-stages"])
def test_all_ranks_full_size_dry_run(hlib, name, budget):
    """All virtual ranks resident at full size on the CPU build, one-shot and staged in XOR step
    order: accesses inside the buffers, every destination payload byte written exactly once."""
    w = cf.WORKLOADS[name]
    out = parity.dry_run_all_ranks(hlib, w["model"], w["src"], w["dst"], staged_budget=budget)
    assert out["written"] > 0 and (budget is None or out["stages"] >= 1)
    if name == "gpt1p3b" and budget:
        assert out["stages"] > 1 and out["scratch"] < out["sent"]


@pytest.mark.parametrize("name", sorted(cf.PAPER_TRANSITIONS))
@pytest.mark.parametrize("reverse", [False, True], ids=["forward", "back"])
def test_paper_table_transitions_at_model_scale(hlib, name, reverse):
    """The world-size-changing (TP, PP, DP) transitions of the paper's hybrid reconfiguration table
    (dense rows), the pair of its ablation study and the table's two MoE pairs (EP carved out of
    the TP x DP ranks), both directions, on the full model shapes: routes of every rank validated
    by the oracle, and the copy tables of the last rank walked in a dry run."""
    import oracle
    from paper_2605_18815_amd import binding as B
    w = cf.PAPER_TRANSITIONS[name]
    pa, pb = (w["dst"], w["src"]) if reverse else (w["src"], w["dst"])
    a, b = oracle.Config(w["model"], pa), oracle.Config(w["model"], pb)
    assert (a.world != b.world) == ("-to-" in name)
    ca, cb = hlib.describe_config(w["model"], pa), hlib.describe_config(w["model"], pb)
    routes = hlib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_ROUTES_ONLY)
    parity.validate_boxes(a, b, routes.get_boxes(), -1, samples=2, plan=routes)
    if not reverse:
        # ordered by the radix sort instead of pair by pair: the same table
        hlib.set_option(B.OPT_PAIR_ORDER_WORK, 0)
        try:
            again = hlib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_ROUTES_ONLY).get_boxes()
        finally:
            hlib.set_option(B.OPT_PAIR_ORDER_WORK, 32)
        assert again.tobytes() == routes.get_boxes().tobytes()
    for rank in {max(a.world, b.world) - 1, min(a.world, b.world) - 1}:
        parity.dry_run_single_rank(hlib, w["model"], pa, pb, rank, box_samples=2)


def test_random_transitions(hlib):
    import random_cases
    ran = sum(random_cases.run_case(hlib, lambda: parity.HostMem(hlib), c) for c in random_cases.cases(20260000, 150))
    assert ran >= 40   # the rest drew a degree that does not divide the model


def test_largest_world(hlib):
    """32768 ranks on each side (the limit of the 16-bit rank fields in the sort keys)."""
    m = cf.model(cf.FAMILY_GPT, 8, 32, 8, 8, 4, 64, 64)
    pa, pb = P(tp=4, pp=8, dp=1024, zero=1), P(tp=8, pp=8, dp=512, zero=1)
    for rank in (32767, 12345):
        parity.run_single_rank(hlib, parity.HostMem(hlib), m, pa, pb, rank, seed=9, box_samples=4, check_bytes=False,
                               send_payload_ranks=0)
    with pytest.raises(VpsError):
        hlib.describe_config(m, P(tp=4, pp=8, dp=2048))


def test_box_checker_detects_planted_mistakes(hlib):
    """The oracle's per-element check of a box list must notice a shifted source offset, a
    shifted destination offset, a wrong stride, a box moved in the coordinate space, and a source
    rank that holds the data but is not the one the selection rule names."""
    import oracle
    _, m, pa, pb = [t for t in TRANSITIONS if t[0] == "gpt-zero-to-replicated"][0]
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    ca, cb = hlib.describe_config(m, pa), hlib.describe_config(m, pb)
    boxes = hlib.plan_intersections(ca, cb, -1).get_boxes()
    assert oracle.check_boxes(a, b, *parity.boxes_to_oracle_arrays(boxes))[0] == 0
    big = int(np.argmax(np.prod(boxes["ext"].astype(np.int64), axis=1)))

    def planted(edit):
        bad = boxes.copy()
        edit(bad)
        return oracle.check_boxes(a, b, *parity.boxes_to_oracle_arrays(bad))

    def shift(field, k=big, by=1):
        def edit(bx):
            bx[field][k] += by
        return edit

    for edit in (shift("src_off"), shift("dst_off"), shift("src_off", by=-1)):
        nbad, first = planted(edit)
        assert nbad > 0 and first == big

    def wrong_stride(bx):
        ax = int(np.argmax(bx["ext"][big]))
        bx["dst_stride"][big][ax] += 1
    assert planted(wrong_stride)[0] > 0

    def moved_box(bx):
        ax = int(np.argmax(bx["ext"][big]))
        bx["lo"][big][ax] += 1
    assert planted(moved_box)[0] > 0

    # another replica of the same data: the bits would be right, the route is not the rule's
    moving = np.nonzero(boxes["src_rank"] != boxes["dst_rank"])[0]
    hits = 0
    for k in moving:
        if hits >= 5:
            break
        t, kind, lo = int(boxes["tensor"][k]), int(boxes["kind"][k]), tuple(int(v) for v in boxes["lo"][k])
        others = [o for o in a.owners(kind, t, lo) if o[0] != int(boxes["src_rank"][k])]
        if not others:
            continue
        r, buf, off = others[0]

        def other_replica(bx, k=k, r=r, buf=buf, off=off):
            bx["src_rank"][k], bx["src_buf"][k], bx["src_off"][k] = r, buf, off
        nbad, first = planted(other_replica)
        assert nbad > 0 and first == k
        hits += 1
    assert hits > 0


def test_plain_copy_reference(hlib):
    from paper_2605_18815_amd import binding as B
    mem = parity.HostMem(hlib)
    n = 8192 * 3 + 4096 + 16       # three full tiles and a ragged one
    src, dst = mem.alloc(n), mem.alloc(n + 32)
    src[:] = np.random.default_rng(5).integers(0, 256, n, dtype=np.uint8)
    mem.register_bounds()
    hlib.plain_copy(mem.ptr(dst), mem.ptr(src), n)
    assert mem.violations() == 0
    assert np.array_equal(dst[:n], src) and (dst[n:] == parity.SENTINEL).all()
    for bad in ((mem.ptr(dst) + 8, mem.ptr(src), 64), (mem.ptr(dst), mem.ptr(src), 40), (mem.ptr(src) + 16, mem.ptr(src), 64)):
        with pytest.raises(VpsError) as e:
            hlib.plain_copy(*bad)
        assert e.value.code == B.ERR_INVALID_ARG


def test_error_codes(hlib):
    check_error_codes(hlib, parity.HostMem(hlib))


def check_error_codes(hlib, mem):
    """Every documented error is reported with its code, before any device work is enqueued
    (also run against the HIP library by the GPU tests)."""
    from paper_2605_18815_amd import binding as B
    with pytest.raises(VpsError) as e:
        hlib.describe_config(cf.TINY_GPT, P(tp=3))
    assert e.value.code == B.ERR_INDIVISIBLE
    with pytest.raises(VpsError) as e:
        hlib.describe_config(cf.TINY_MOE, P(ep=3))
    assert e.value.code == B.ERR_INDIVISIBLE
    with pytest.raises(VpsError) as e:   # ep carved out of tp*dp must divide it
        hlib.describe_config(cf.TINY_MOE, P(tp=2, dp=3, ep=4, ep_placement=1))
    assert e.value.code == B.ERR_INDIVISIBLE
    with pytest.raises(VpsError) as e:
        hlib.describe_config(cf.TINY_MOE, P(ep_placement=2))
    assert e.value.code == B.ERR_INVALID_ARG
    with pytest.raises(VpsError) as e:
        hlib.describe_config(cf.TINY_GPT, P(tp=0))
    assert e.value.code == B.ERR_INVALID_ARG
    with pytest.raises(VpsError) as e:
        hlib.describe_config(cf.TINY_GPT, P(tp=2), rank=2)
    assert e.value.code == B.ERR_RANK_RANGE
    with pytest.raises(VpsError) as e:   # 20 M logical tensors: ids would not fit the sort keys
        hlib.describe_config(cf.model(cf.FAMILY_MOE, 1000, 16, 4, 4, 4, 0, 64, experts=10000, expert_ffn=8), P())
    assert e.value.code == B.ERR_INVALID_ARG
    ca = hlib.describe_config(cf.TINY_GPT, P(tp=2, dp=2))
    cb = hlib.describe_config(cf.TINY_GQA, P(tp=2, dp=2))
    with pytest.raises(VpsError) as e:
        hlib.plan_intersections(ca, cb, -1)
    assert e.value.code == B.ERR_MODEL_MISMATCH
    one = hlib.describe_config(cf.TINY_GPT, P(tp=2, dp=2), rank=1)
    assert one.num_pieces > 0 and set(one.get_pieces()["rank"]) == {1}
    with pytest.raises(VpsError) as e:
        hlib.plan_intersections(one, ca, -1)
    assert e.value.code == B.ERR_INVALID_ARG
    cb = hlib.describe_config(cf.TINY_GPT, P(tp=1, dp=4, zero=0))
    with pytest.raises(VpsError) as e:
        hlib.plan_intersections(ca, cb, 4)
    assert e.value.code == B.ERR_RANK_RANGE
    plan = hlib.plan_intersections(ca, cb, 1)
    info = plan.buffer_bytes(1)
    bufs = [mem.ptr(mem.alloc(max(ca.buffer_bytes(1, b), cb.buffer_bytes(1, b)))) for b in range(8)]
    with pytest.raises(VpsError) as e:
        hlib.apply_transition(plan, 1, bufs, bufs, mem.ptr(mem.alloc(16)), 16)
    assert e.value.code == B.ERR_SCRATCH_TOO_SMALL or info["scratch_needed"] <= 16
    with pytest.raises(VpsError) as e:
        hlib.apply_transition(plan, 2, bufs, bufs, 0, 0)
    assert e.value.code == B.ERR_RANK_RANGE
    big = mem.alloc(info["scratch_needed"])
    with pytest.raises(VpsError) as e:   # source passed as destination as well
        hlib.apply_transition(plan, 1, bufs, bufs, mem.ptr(big), info["scratch_needed"])
    assert e.value.code == B.ERR_INVALID_ARG
    assert ca.num_buffers(0) == 8
    with pytest.raises(VpsError) as e:
        hlib.pack(plan, 1, [0] * 8, mem.ptr(mem.alloc(info["send_total"])))
    assert e.value.code == B.ERR_INVALID_ARG

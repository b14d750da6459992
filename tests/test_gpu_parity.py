"""GPU parity: the HIP library through its C ABI against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import parity
from datagen import configs as cf
from test_oracle_pins import ALL_TRANSITIONS, TRANSITIONS
from test_hostcheck_parity import (BEYOND, COLLECTIVE_CASES, EDGE_TRANSITIONS, MEDIUM, SINGLE, STAGED, THROUGH, check_error_codes,
                                   run_plans_beyond_the_counting_limit, run_staged_long_runs)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2605_18815_amd as vps
    return vps.load()


@pytest.mark.parametrize("name,m,pa,pb", ALL_TRANSITIONS, ids=[c[0] for c in ALL_TRANSITIONS])
def test_all_ranks_resident(lib, name, m, pa, pb):
    out = parity.run_all_ranks(lib, parity.GpuMem(), m, pa, pb, seed=0x5EED + len(name))
    assert out["boxes"] > 0


@pytest.mark.parametrize("name,m,pa,pb", MEDIUM, ids=[c[0] for c in MEDIUM])
def test_medium_shapes_all_ranks(lib, name, m, pa, pb):
    """Several 64-element blocks with ragged tails: LDS-staged transposes and short-run tiles."""
    out = parity.run_all_ranks(lib, parity.GpuMem(), m, pa, pb, seed=0xC0FFEE)
    assert out["boxes"] > 0


@pytest.mark.parametrize("name,rank", SINGLE, ids=[f"{n}-r{r}" for n, r in SINGLE])
def test_single_rank_share(lib, name, rank):
    _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == name][0]
    parity.run_single_rank(lib, parity.GpuMem(), m, pa, pb, rank, seed=0xBEEF + rank)


@pytest.mark.parametrize("name,rank", THROUGH, ids=[f"{n}-r{r}" for n, r in THROUGH])
def test_rank_as_its_own_peer(lib, name, rank):
    _, m, pa, pb = [t for t in ALL_TRANSITIONS if t[0] == name][0]
    mem = parity.GpuMem()
    if rank < 0:
        parity.run_all_ranks(lib, mem, m, pa, pb, seed=0xD00D, through=True)
    else:
        parity.run_single_rank(lib, mem, m, pa, pb, rank, seed=0xD00D + rank, through=True)


@pytest.mark.parametrize("limit,pair_work", BEYOND, ids=[f"{a}-{['sort', 'bound-exceeded'][b] if b < 2 else 'pairs'}" for a, b in BEYOND])
def test_plans_beyond_the_counting_limit(lib, limit, pair_work):
    """The paths of the planner for many boxes on the device (pair-by-pair ordering, radix sort, and
    the switch from the first to the second), reached by lowering the limit of the counting path
    (see the CPU-build test of the same name)."""
    run_plans_beyond_the_counting_limit(lib, parity.GpuMem, limit, pair_work)


def test_staged_exchange_moves_long_runs(lib):
    run_staged_long_runs(lib, parity.GpuMem)


def test_sender_and_receiver_agree_on_segments_toy(lib):
    w = cf.WORKLOADS["toy"]
    assert parity.check_cross_plan_segments(lib, w["model"], w["src"], w["dst"], [(i, j) for i in range(4) for j in range(4)]) > 0


def test_toy_workload_all_ranks(lib):
    w = cf.WORKLOADS["toy"]
    out = parity.run_all_ranks(lib, parity.GpuMem(), w["model"], w["src"], w["dst"], seed=cf.seed_of("toy"))
    assert out["moved"] > 0


@pytest.mark.parametrize("tile", [4096, 262144])
def test_tile_size_does_not_change_results(lib, tile):
    lib.set_tile_bytes(tile)
    try:
        _, m, pa, pb = TRANSITIONS[3]
        parity.run_all_ranks(lib, parity.GpuMem(), m, pa, pb, seed=77)
        w = cf.WORKLOADS["toy"]
        parity.run_single_rank(lib, parity.GpuMem(), w["model"], w["src"], w["dst"], 1, seed=78)
    finally:
        lib.set_tile_bytes(8192)


@pytest.mark.parametrize("name,budget_kind", [(n, k) for n, _ in STAGED for k in ("tiny", "mid")],
                         ids=[f"{n}-{k}" for n, _ in STAGED for k in ("tiny", "mid")])
def test_staged_xor_exchange(lib, name, budget_kind):
    _, m, pa, pb = [t for t in TRANSITIONS if t[0] == name][0]
    probe = parity.run_staged(lib, parity.GpuMem(), m, pa, pb, seed=5, budget=1 << 60)
    budget = {"tiny": 1, "mid": max(probe["max_cost"] * 2, 1)}[budget_kind]
    out = parity.run_staged(lib, parity.GpuMem(), m, pa, pb, seed=6, budget=budget)
    assert out["stages"] >= 1


def test_staged_exchange_toy_workload(lib):
    w = cf.WORKLOADS["toy"]
    out = parity.run_staged(lib, parity.GpuMem(), w["model"], w["src"], w["dst"], seed=cf.seed_of("toy"), budget=8 << 20)
    assert out["stages"] >= 2


@pytest.mark.parametrize("name,m,pa,pb,expect", COLLECTIVE_CASES, ids=[c[0] for c in COLLECTIVE_CASES])
def test_collective_intent_cases(lib, name, m, pa, pb, expect):
    counts = parity.run_classify(lib, m, pa, pb)
    assert counts[expect] > 0, counts


@pytest.mark.parametrize("name,m,pa,pb", TRANSITIONS + [c[:4] for c in MEDIUM], ids=[c[0] for c in TRANSITIONS + MEDIUM])
def test_collective_intent_matches_bruteforce(lib, name, m, pa, pb):
    counts = parity.run_classify(lib, m, pa, pb)
    assert counts.sum() > 0


@pytest.mark.parametrize("name,m,pa,pb", EDGE_TRANSITIONS, ids=[c[0] for c in EDGE_TRANSITIONS])
def test_edge_transitions(lib, name, m, pa, pb):
    out = parity.run_all_ranks(lib, parity.GpuMem(), m, pa, pb, seed=3)
    if name == "identity":
        assert out["moved"] == 0
    import oracle
    wa, wb = oracle.Config(m, pa).world, oracle.Config(m, pb).world
    for r in sorted({0, wa - 1, wb - 1, max(wa, wb) - 1}):
        parity.run_single_rank(lib, parity.GpuMem(), m, pa, pb, r, seed=4)


def test_random_transitions(lib):
    import random_cases
    ran = sum(random_cases.run_case(lib, parity.GpuMem, c) for c in random_cases.cases(20260000, 150))
    assert ran >= 40


def test_plans_from_two_threads_on_two_streams(lib):
    """Calls are thread-safe on distinct handles: two host threads map and plan in loops, each on
    a stream of its own (single ranks and all ranks, so every planner path runs), while the
    library's pools, its cache of table sizes and the summary block that one plan clears for the
    next are shared.  Every plan must hold the boxes of the plan made alone."""
    import threading
    import torch
    cases = [(m, pa, pb, r) for _, m, pa, pb in MEDIUM[:3] for r in (-1, 0, 1)]
    cases += [(m, pb, pa, r) for _, m, pa, pb in MEDIUM[:3] for r in (-1, 1)]

    def boxes_of(m, pa, pb, r, stream):
        plan = lib.plan_intersections(lib.describe_config(m, pa), lib.describe_config(m, pb), r, stream)
        return plan.get_boxes(), plan.buffer_bytes(r)

    alone = [boxes_of(*c, 0) for c in cases]
    problems = []

    def work(first):
        try:
            stream = torch.cuda.Stream()
            for it in range(25):
                k = (first + 7 * it) % len(cases)
                boxes, info = boxes_of(*cases[k], stream.cuda_stream)
                if not np.array_equal(boxes, alone[k][0]) or info != alone[k][1]:
                    problems.append(("plan differs from the one made alone", first, it, k))
            stream.synchronize()
        except Exception as e:   # (an assertion in a thread would not fail the test by itself)
            problems.append((repr(e), first))

    threads = [threading.Thread(target=work, args=(f,)) for f in (0, 3)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not problems, problems[:3]


def test_largest_world(lib):
    m = cf.model(cf.FAMILY_GPT, 8, 32, 8, 8, 4, 64, 64)
    pa, pb = cf.parallel(tp=4, pp=8, dp=1024, zero=1), cf.parallel(tp=8, pp=8, dp=512, zero=1)
    for rank in (0, 32767, 12345):
        parity.run_single_rank(lib, parity.GpuMem(), m, pa, pb, rank, seed=9, box_samples=4, check_bytes=False,
                               send_payload_ranks=0)


@pytest.mark.parametrize("rank", [-1, 1])
def test_apply_transition_replayed_from_a_hip_graph(lib, rank):
    """vps_apply_transition enqueues kernels only, so it can be captured into a HIP graph.  The
    graph is replayed several times with eager work between the replays (new source data, cleared
    destinations); every replay must equal an eager call on the same data."""
    import torch
    w = cf.WORKLOADS["toy"]
    ca, cb = lib.describe_config(w["model"], w["src"]), lib.describe_config(w["model"], w["dst"])
    plan = lib.plan_intersections(ca, cb, rank)
    info = plan.buffer_bytes(rank)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    ra = range(ca.world) if rank < 0 else [rank]
    rb = range(cb.world) if rank < 0 else [rank]
    src = [torch.empty(ca.buffer_bytes(r, b), dtype=torch.uint8, device=dev) for r in ra for b in range(8)]
    dst = [torch.empty(cb.buffer_bytes(r, b), dtype=torch.uint8, device=dev) for r in rb for b in range(8)]
    ref = [torch.empty_like(t) for t in dst]
    scratch = torch.empty(info["scratch_needed"], dtype=torch.uint8, device=dev)
    scratch_ref = torch.empty_like(scratch)
    ptrs = lambda ts: [t.data_ptr() if t.numel() else 0 for t in ts]

    def new_inputs():
        for t in src:
            if t.numel():
                t.random_(0, 256, generator=gen)
        if scratch.numel():
            scratch.random_(0, 256, generator=gen)   # the receive part stands in for the peers' data
            scratch_ref.copy_(scratch)
        for t in dst + ref:
            t.fill_(0xA5)

    side = torch.cuda.Stream()
    new_inputs()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        lib.apply_transition(plan, rank, ptrs(src), ptrs(dst), scratch.data_ptr(), scratch.numel(), side.cuda_stream)
    for replay in range(4):
        new_inputs()
        torch.cuda.synchronize()
        graph.replay()
        lib.apply_transition(plan, rank, ptrs(src), ptrs(ref), scratch_ref.data_ptr(), scratch_ref.numel(),
                             torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for got, want in zip(dst, ref):
            assert torch.equal(got, want), f"replay {replay} differs from the eager call"
        assert any(bool((t != 0xA5).any()) for t in dst if t.numel())


def test_plain_copy_reference(lib):
    import torch
    n = 8192 * 1000 + 4096 + 16
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.full((n + 32,), 0xA5, dtype=torch.uint8, device="cuda:0")
    lib.plain_copy(dst.data_ptr(), src.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and bool((dst[n:] == 0xA5).all())


def test_plain_read_and_fill(lib):
    """The two halves of the plain copy that the benchmark times: the fill writes every byte of
    its range and nothing else, the read leaves its source and (bar a 2^-32 accident) the sink alone."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    n = 8192 * 777 + 4096 + 48
    dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda:0")
    lib.plain_fill(dst.data_ptr() + 32, n, stream)
    torch.cuda.synchronize()
    assert bool((dst[32:32 + n] == 0xA5).all()) and not bool(dst[:32].any()) and not bool(dst[32 + n:].any())
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0")
    keep = src.clone()
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    lib.plain_read(src.data_ptr(), n, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    assert torch.equal(src, keep) and not bool(sink.any())
    from paper_2605_18815_amd.binding import VpsError
    with pytest.raises(VpsError):
        lib.plain_fill(dst.data_ptr() + 8, 64, stream)
    with pytest.raises(VpsError):
        lib.plain_read(src.data_ptr(), 24, sink.data_ptr(), stream)
    lib.plain_fill(dst.data_ptr(), 0, stream)   # nothing to do


def test_error_codes(lib):
    check_error_codes(lib, parity.GpuMem())

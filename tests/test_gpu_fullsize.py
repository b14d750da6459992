"""GPU parity at the benchmark's full sizes (one rank's share of the large workloads)."""
import os

import pytest

import parity
from datagen import configs as cf

pytestmark = pytest.mark.gpu

FRACTION = float(os.environ.get("VPS_FULLSIZE_FRACTION", "1.0"))


@pytest.fixture(scope="module")
def lib():
    import paper_2605_18815_amd as vps
    return vps.load()


@pytest.fixture(autouse=True)
def _release_cached_device_memory():
    """These tests hold up to 130 GB each: give torch's cached blocks back between them."""
    import gc
    import torch
    gc.collect()
    torch.cuda.empty_cache()
    yield


def _run(lib, name, rank=None, src_over=None, dst_over=None, fraction=None, through=False):
    w = cf.workload(name)
    pa, pb = dict(w["src"]), dict(w["dst"])
    pa.update(src_over or {})
    pb.update(dst_over or {})
    rank = w["rank"] if rank is None else rank
    print(f"\n{name} rank {rank}", flush=True)
    out = parity.run_single_rank_fullsize(lib, parity.GpuMem(), w["model"], pa, pb, rank,
                                          seed=cf.seed_of(name), fraction=FRACTION if fraction is None else fraction,
                                          log=lambda s: print(s, flush=True), through=through)
    assert out["checked"] > 0
    return out


@pytest.mark.timeout(600)
def test_gqa70b_rank11_full_size(lib):
    out = _run(lib, "gqa70b")
    # first-stage rank: the embedding shifts the flat edges, fp32 state really moves
    assert out["info"]["send_total"] > 0 and out["info"]["recv_total"] > 0


@pytest.mark.timeout(600)
@pytest.mark.parametrize("through", [False, True], ids=["direct", "through-buffers"])
def test_gqa70b_odd_sizes_full_size(lib, through):
    """Every tensor starts at an odd element offset: the long runs take the paths for a source
    that is 2 bytes (bf16: through LDS) or a multiple of 4 bytes (fp32) off the destination's
    16-byte phase, and are cut at 256-byte boundaries of the destination."""
    out = _run(lib, "gqa70b-odd", through=through)
    assert out["info"]["send_total"] > 0


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["gqa70b", "gqa8b"])
def test_whole_share_through_the_buffers_full_size(lib, name):
    """The all-through-buffers stress at full size: the rank is its own peer, so pack and unpack
    each run over the whole share; every destination element and every byte of the send buffer is
    compared."""
    out = _run(lib, name, through=True)
    assert out["info"]["retain_total"] == 0 and out["stats"]["num_retain_tiles"] == 0
    assert out["info"]["send_total"] > 0


def test_sender_and_receiver_agree_on_segments_70b(lib):
    """Rank 11 of the 70B switch and each of its peers, planned independently: same boxes at the
    same offsets inside every segment (planning only: no state is resident)."""
    w = cf.WORKLOADS["gqa70b"]
    ca, cb = lib.describe_config(w["model"], w["src"]), lib.describe_config(w["model"], w["dst"])
    boxes = lib.plan_intersections(ca, cb, 11).get_boxes()
    pairs = sorted({(int(s), int(d)) for s, d in zip(boxes["src_rank"], boxes["dst_rank"]) if s != d})
    assert len(pairs) >= 6
    assert parity.check_cross_plan_segments(lib, w["model"], w["src"], w["dst"], pairs) > 0


@pytest.mark.timeout(600)
def test_gqa70b_mid_stage_rank_keeps_fp32(lib):
    out = _run(lib, "gqa70b", rank=43)
    w = cf.WORKLOADS["gqa70b"]
    import oracle
    b = oracle.Config(w["model"], w["dst"])
    fp32 = sum(4 * b.payload_elems(43, k) for k in (1, 2, 3))
    assert out["info"]["retain_total"] >= fp32


@pytest.mark.timeout(600)
def test_gqa8b_rank5_full_size(lib):
    out = _run(lib, "gqa8b")
    assert out["stats"]["num_peers_in"] >= 2


@pytest.mark.timeout(600)
def test_gqa8b_rank5_destination_blocked_qkv(lib):
    """Variant: the destination stores fused QKV as [all Q | all K | all V] blocks."""
    _run(lib, "gqa8b", dst_over=dict(qkv_layout=1))


@pytest.mark.timeout(600)
def test_gqa70b_rank11_reverse_flat_order(lib):
    """Variant: descending tensor order in the flat buffers, so that all fp32 state moves."""
    out = _run(lib, "gqa70b", src_over=dict(flat_order=1))
    assert out["info"]["recv_total"] > 0


@pytest.mark.timeout(900)
def test_moe235b_rank37_full_size(lib):
    out = _run(lib, "moe235b")
    assert out["stats"]["num_boxes"] > 1000


@pytest.mark.timeout(900)
def test_moe235b_rank37_destination_transposed_experts(lib):
    """Variant: the destination stores experts transposed, so every expert box goes through the
    LDS-staged transpose tiles."""
    # every chunk holding a box edge plus a quarter of the others (the row-major run above
    # compares every element of the same share)
    _run(lib, "moe235b", dst_over=dict(expert_layout=1), fraction=min(FRACTION, 0.25))


@pytest.mark.timeout(900)
def test_moe235b_rank37_more_tiles_than_one_dispatch_holds(lib):
    """With 4 KiB tiles the share has 13.8 M tiles; a dispatch of 256-lane workgroups holds fewer
    than 2^24 of them, and the library cuts the tile range into launches of 2^23."""
    lib.set_tile_bytes(4096)
    try:
        out = _run(lib, "moe235b", fraction=min(FRACTION, 0.03))
    finally:
        lib.set_tile_bytes(8192)
    st = out["stats"]
    assert st["num_retain_tiles"] + st["num_pack_tiles"] + st["num_unpack_tiles"] > 1 << 23


PAPER_CASES = [("llama70b-64-to-128", False, 127), ("llama70b-64-to-128", False, 40),
               ("llama70b-64-to-128", True, 100), ("llama13b-16-to-32", True, 5), ("llama7b-8-to-16", False, 15),
               ("llama13b-ablation-pair", False, 9),
               # the MoE pairs, EP carved out of the TP x DP ranks: one rank of each pair (both
               # directions are planned for all ranks on the CPU build) in each direction
               ("qwen30b-hybrid", False, 3), ("qwen235b-hybrid", False, 77)]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,reverse,rank", PAPER_CASES, ids=[f"{n}-{'back' if r else 'forward'}-r{k}" for n, r, k in PAPER_CASES])
def test_paper_table_transition_one_rank_full_size(lib, name, reverse, rank):
    """World-size-changing transitions of the paper's hybrid reconfiguration table at full model
    size: ranks that exist on the destination side only (everything arrives through the buffers),
    on the source side only (everything leaves), and on both."""
    w = cf.PAPER_TRANSITIONS[name]
    pa, pb = (w["dst"], w["src"]) if reverse else (w["src"], w["dst"])
    print(f"\n{name} {'back' if reverse else 'forward'} rank {rank}", flush=True)
    out = parity.run_single_rank_fullsize(lib, parity.GpuMem(), w["model"], pa, pb, rank, seed=0x7AB1E + rank,
                                          fraction=FRACTION, log=lambda s: print(s, flush=True))
    world_a, world_b = cf.world(pa), cf.world(pb)
    if rank >= world_a:
        assert out["info"]["retain_total"] == 0 and out["info"]["send_total"] == 0 and out["checked"] > 0
    if rank >= world_b:
        assert out["info"]["retain_total"] == 0 and out["info"]["recv_total"] == 0 and out["checked"] == 0


@pytest.mark.timeout(900)
def test_gpt1p3b_all_ranks_full_size(lib):
    w = cf.WORKLOADS["gpt1p3b"]
    print("\ngpt1p3b all 32 ranks", flush=True)
    out = parity.run_all_ranks_fullsize(lib, parity.GpuMem(), w["model"], w["src"], w["dst"],
                                        seed=cf.seed_of("gpt1p3b"), fraction=FRACTION, staged_budget=512 << 20,
                                        log=lambda s: print(s, flush=True))
    assert out["checked"] > 0


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["gqa70b", "moe235b"])
def test_all_ranks_planning_at_scale(lib, name):
    """Routes of all 128 ranks at once (no copy tables): every box validated by the oracle on its
    corners and random interior points, destination coverage exact for every rank."""
    import time
    import numpy as np
    import oracle
    from paper_2605_18815_amd import binding as B
    w = cf.WORKLOADS[name]
    a, b = oracle.Config(w["model"], w["src"]), oracle.Config(w["model"], w["dst"])
    t0 = time.time()
    ca, cb = lib.describe_config(w["model"], w["src"]), lib.describe_config(w["model"], w["dst"])
    t1 = time.time()
    plan = lib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_ROUTES_ONLY)
    t2 = time.time()
    boxes = plan.get_boxes()
    print(f"\n{name}: {ca.num_pieces} + {cb.num_pieces} pieces in {t1 - t0:.3f}s, {len(boxes)} boxes in {t2 - t1:.3f}s "
          f"({len(boxes) / (t2 - t1) / 1e6:.2f} M boxes/s)", flush=True)
    parity.validate_boxes(a, b, boxes, -1, samples=8, plan=plan)
    # one rank's plan is the restriction of the all-ranks plan
    r = w["rank"]
    one = lib.plan_intersections_ex(ca, cb, r, flags=B.PLAN_ROUTES_ONLY).get_boxes()
    sel = boxes[(boxes["src_rank"] == r) | (boxes["dst_rank"] == r)]
    keys = ["tensor", "kind", "src_rank", "dst_rank", "src_off", "dst_off"]
    assert len(one) == len(sel)
    assert np.array_equal(np.sort(one[keys], order=keys), np.sort(sel[keys], order=keys))
    # the two ways of ordering a large all-ranks plan (pair by pair, radix sort) and the switch from
    # the first to the second give the same table, positions included
    # (and, with the default bound again, the plan that knows its size from the ones before and
    # counts its boxes per pair while it emits them)
    for work in (0, 1, 32):
        lib.set_option(B.OPT_PAIR_ORDER_WORK, work)
        try:
            replan = lib.plan_intersections_ex(ca, cb, -1, flags=B.PLAN_ROUTES_ONLY)
            again = replan.get_boxes()
        finally:
            lib.set_option(B.OPT_PAIR_ORDER_WORK, 32)
        assert again.tobytes() == boxes.tobytes(), f"ordering with work bound 2^{work} differs"
        parity.check_stats(replan, again, -1)
        assert replan.buffer_bytes(-1) == plan.buffer_bytes(-1)
    cls = plan.classify_collectives(ca)
    print("  collective intent per (tensor, kind) [none, p2p, broadcast, scatter, gather]:", np.bincount(cls, minlength=5), flush=True)


@pytest.mark.timeout(900)
def test_contiguous_run_beyond_32_bit_extent(lib):
    """Regression: an embedding shard of 4.4e9 elements is one contiguous stretch whose element
    count does not fit 32 bits.  Rank 0 of a two-stage pipeline keeps its state but reverses the
    flat order, so every tensor moves to a new offset (124 GB resident).  Expected placement from
    the oracle's per-element maps: whole tensors compared on the device, plus sampled elements."""
    import numpy as np
    import torch
    import oracle
    m = cf.model(cf.FAMILY_GQA, 2, 8192, 64, 8, 128, 1024, 540_000)
    pa, pb = cf.parallel(tp=1, pp=2, dp=1), cf.parallel(tp=1, pp=2, dp=1, flat_order=1)
    a, b = oracle.Config(m, pa), oracle.Config(m, pb)
    rank = 0
    ca, cb = lib.describe_config(m, pa), lib.describe_config(m, pb)
    plan = lib.plan_intersections(ca, cb, rank)
    boxes = plan.get_boxes()
    parity.validate_boxes(a, b, boxes, rank, samples=16, plan=plan)
    info = plan.buffer_bytes(rank)
    assert info["send_total"] == 0 and info["recv_total"] == 0
    assert int(np.prod(boxes["ext"].astype(np.int64), axis=1).max()) > 1 << 32
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    dts = {2: torch.int16, 4: torch.int32}
    src, dst = [], []
    for buf in range(8):
        es = oracle.KIND_BYTES[buf % 4]
        s = torch.empty(a.buffer_elems(rank, buf), dtype=dts[es], device=dev)
        if s.numel():
            s.random_(generator=gen)
        src.append(s)
        dst.append(torch.full((b.buffer_elems(rank, buf),), -1, dtype=dts[es], device=dev))
    print(f"\n{sum(t.numel() * t.element_size() for t in src + dst) / 1e9:.1f} GB resident", flush=True)
    ptr = lambda ts: [t.data_ptr() if t.numel() else 0 for t in ts]
    lib.apply_transition(plan, rank, ptr(src), ptr(dst), 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    # whole tensors: under both configurations rank 0 stores a tensor's shard row-major in one piece
    step = 1 << 28
    compared = 0
    for t in range(a.num_tensors):
        for kind in range(4):
            own_a = [o for o in a.owners(kind, t, (0, 0, 0, 0)) if o[0] == rank]
            own_b = [o for o in b.owners(kind, t, (0, 0, 0, 0)) if o[0] == rank]
            assert len(own_a) == len(own_b)
            if not own_a:
                continue
            (_, buf_a, off_a), (_, buf_b, off_b) = own_a[0], own_b[0]
            n = int(np.prod(a.tensor_info(t)["shape"], dtype=np.int64))
            for o in range(0, n, step):
                k = min(step, n - o)
                assert torch.equal(dst[buf_b][off_b + o:off_b + o + k], src[buf_a][off_a + o:off_a + o + k]), (t, kind, o)
            compared += n
    assert compared == sum(b.payload_elems(rank, buf) for buf in range(8))
    # sampled elements through the per-element maps, and the padding is untouched
    rng = np.random.default_rng(3)
    for buf in range(8):
        n, pay = b.buffer_elems(rank, buf), b.payload_elems(rank, buf)
        if not n:
            continue
        offs = np.unique(np.concatenate([rng.integers(0, pay, 64), [0, pay - 1, (1 << 32) - 1, 1 << 32, (1 << 32) + 1]]))
        for off in offs[offs < pay]:
            t, cd = b.coord(rank, buf, int(off))
            r, sb, so = [o for o in a.owners(buf % 4, t, cd) if o[0] == rank][0]
            assert int(dst[buf][int(off)]) == int(src[sb][so]), (buf, off)
        assert bool((dst[buf][pay:] == -1).all())
    print(f"{compared} elements compared", flush=True)

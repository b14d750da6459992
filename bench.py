#!/usr/bin/env python3
"""Benchmark of the VPS state transition on one MI355X.

One step = one pass of the whole path for one rank's share of the workload: map both
configurations onto the VPS (vps_describe_config x2), plan the intersections
(vps_plan_intersections) and move the data (vps_apply_transition: retain + pack + unpack in one
launch).  State buffers and the peers' receive buffer are resident in HBM before the timed
region.  The JSON line reports bytes moved (read + write) per second over the whole step, and
for the copy kernel alone the achieved HBM rate against the 8 TB/s peak.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gqa70b")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--tile-bytes", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--apply-only", action="store_true", help="time only vps_apply_transition (plan reused)")
    ap.add_argument("--only", choices=["pack", "unpack"], default=None,
                    help="time vps_pack or vps_unpack alone (implies --apply-only)")
    ap.add_argument("--through-buffers", action="store_true",
                    help="stress mode: the rank is its own peer, so the whole share is packed and unpacked")
    ap.add_argument("--staged-mib", type=int, default=0,
                    help="all-ranks workloads: exchange in XOR step order under this per-rank buffer budget (MiB)")
    ap.add_argument("--src", default="", help="override source layout fields, e.g. flat_order=1")
    ap.add_argument("--dst", default="", help="override destination layout fields, e.g. expert_layout=1,qkv_layout=1")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="also run one plain device-to-device copy of MIB MiB (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every virtual rank or one rank's share is "
              "resident on a single MI355X); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2605_18815_amd as vps
    from datagen import configs as cf

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    lib = vps.load()
    if args.tile_bytes:
        lib.set_tile_bytes(args.tile_bytes)
    w = cf.workload(args.workload)
    model, pa, pb = w["model"], dict(w["src"]), dict(w["dst"])
    for spec, par in ((args.src, pa), (args.dst, pb)):
        for kv in filter(None, spec.split(",")):
            k, v = kv.split("=")
            par[k] = int(v)
    rank = args.rank if args.rank is not None else (w["rank"] if w["rank"] is not None else -1)
    if args.workload in cf.PAPER_TRANSITIONS and rank < 0:
        sys.exit("bench.py: the paper's transitions do not fit one GPU with every rank resident; pass --rank")
    stream = torch.cuda.current_stream().cuda_stream

    # ---- resident state: source buffers (seeded random bytes), destination buffers, scratch
    ca, cb = lib.describe_config(model, pa), lib.describe_config(model, pb)
    plan_flags = vps.binding.PLAN_THROUGH_BUFFERS if args.through_buffers else 0
    plan = lib.plan_intersections_ex(ca, cb, rank, plan_flags, stream)
    info = plan.buffer_bytes(rank)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cf.seed_of(args.workload))

    def alloc(nbytes, rand):
        t = torch.empty(int(nbytes), dtype=torch.uint8, device=dev)
        if rand and nbytes:
            t.view(torch.int32)[: nbytes // 4].random_(generator=gen) if nbytes % 4 == 0 else t.random_(generator=gen)
        return t

    src_ranks = [rank] if rank >= 0 else list(range(ca.world))
    dst_ranks = [rank] if rank >= 0 else list(range(cb.world))
    src = [alloc(ca.buffer_bytes(r, b) if r < ca.world else 0, True) for r in src_ranks for b in range(8)]
    dst = [alloc(cb.buffer_bytes(r, b) if r < cb.world else 0, False) for r in dst_ranks for b in range(8)]
    scratch = alloc(info["scratch_needed"], True)   # the receive part stands in for the peers' packed data
    sp = [t.data_ptr() if t.numel() else 0 for t in src]
    dp = [t.data_ptr() if t.numel() else 0 for t in dst]
    payload = info["send_total"] + info["recv_total"] + info["retain_total"]
    if rank < 0:
        payload = 2 * info["send_total"] + info["retain_total"]   # every byte is packed and unpacked here
    bytes_moved = 2 * payload
    if args.only:
        assert rank >= 0, "--only needs a single-rank workload"
        args.apply_only = True
        bytes_moved = 2 * (info["send_total"] if args.only == "pack" else info["recv_total"])
    stage = None
    if args.staged_mib:
        assert rank < 0, "--staged-mib needs a workload with all ranks resident"
        stage = lib.stage_exchange(plan, args.staged_mib << 20, stream)
        sinfo = stage.info()
        scratch = alloc(sinfo["scratch_needed"], False)
        # pack, exchange and unpack each read and write the exchanged bytes once
        bytes_moved = 2 * (3 * info["send_total"] + info["retain_total"])
    torch.cuda.synchronize()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t_desc, t_plan = [], []

    def one_step(k=None):
        if args.apply_only:
            p = plan
        else:
            a2, b2 = lib.describe_config(model, pa), lib.describe_config(model, pb)
            p = lib.plan_intersections_ex(a2, b2, rank, plan_flags, stream)
        stg = None
        if stage is not None:
            stg = stage if args.apply_only else lib.stage_exchange(p, args.staged_mib << 20, stream)
        if k is not None:
            ev[k][0].record()
        if stg is not None:
            lib.apply_transition_staged(stg, sp, dp, scratch.data_ptr(), scratch.numel(), stream)
            if k is not None:
                ev[k][1].record()
            return (p, stg)
        if args.only == "pack":
            lib.pack(p, rank, sp, scratch.data_ptr(), stream)
        elif args.only == "unpack":
            lib.unpack(p, rank, scratch.data_ptr() + info["recv_offset"], dp, stream)
        else:
            lib.apply_transition(p, rank, sp, dp, scratch.data_ptr(), scratch.numel(), stream)
        if k is not None:
            ev[k][1].record()
        return p

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        x = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        y = torch.empty(n, dtype=torch.uint8, device=dev)
        y.copy_(x)   # a plain copy kernel of known size: n bytes read, n bytes written
        torch.cuda.synchronize()
        del x, y

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    # host wall time of mapping and planning with an idle device (not part of the timed region)
    for _ in range(5):
        torch.cuda.synchronize()
        ta = time.perf_counter()
        a2, b2 = lib.describe_config(model, pa), lib.describe_config(model, pb)
        tb = time.perf_counter()
        p2 = lib.plan_intersections_ex(a2, b2, rank, plan_flags, stream)
        tc = time.perf_counter()
        t_desc.append((tb - ta) * 1e3)
        t_plan.append((tc - tb) * 1e3)
        del a2, b2, p2
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    keep = [one_step(k) for k in range(args.steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    del keep
    ms_per_step = wall * 1e3 / args.steps
    apply_ms = sorted(a.elapsed_time(b) for a, b in ev)
    apply_avg = sum(apply_ms) / len(apply_ms)

    st = plan.stats()
    launches = 1 if rank >= 0 and not args.through_buffers else 2
    if stage is not None:
        launches = 1 + 3 * sinfo["num_stages"]
    # HBM bytes per launch as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE for this very
    # workload and tile size (profiles/); null for any other configuration
    traffic = None
    prof = os.path.join(ROOT, "profiles", f"k_copy_tiles_{args.workload}_rank{rank}_hbm_traffic.txt")
    if os.path.exists(prof) and not (args.tile_bytes or args.src or args.dst or args.through_buffers or args.only or args.staged_mib):
        for line in open(prof):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = int(line.split("=")[1])
    # the practical ceiling in the same process: a plain contiguous copy in the same launch shape
    ceil_bytes = min(bytes_moved // 2, 8 << 30) // 16 * 16
    plain_gbps = None
    if ceil_bytes >= (64 << 20):
        # destination 8448 bytes off the source's alignment: with equal offsets on both sides the
        # reads and writes of a tile fall on the same memory channels and a plain copy loses 2 %
        shift = 8448
        x, y = alloc(ceil_bytes, True), alloc(ceil_bytes + shift, False)
        cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for k in range(-2, 10):
            if k >= 0:
                cev[k][0].record()
            lib.plain_copy(y.data_ptr() + shift, x.data_ptr(), ceil_bytes, stream)
            if k >= 0:
                cev[k][1].record()
        torch.cuda.synchronize()
        plain_ms = sum(a.elapsed_time(b) for a, b in cev) / len(cev)
        plain_gbps = 2 * ceil_bytes / (plain_ms * 1e-3) / 1e9
        del x, y
    roofline = dict(bound="hbm", achieved=bytes_moved / (apply_avg * 1e-3) / 1e9, peak=HBM_PEAK_GBPS,
                    unit="GB/s", frac=bytes_moved / (apply_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, traffic=traffic,
                    kernel="k_copy_tiles", launches_per_step=launches, kernel_ms_avg=apply_avg,
                    kernel_ms_median=apply_ms[len(apply_ms) // 2], algorithmic_bytes_per_step=bytes_moved,
                    plain_copy_gbps=plain_gbps,
                    frac_of_plain_copy=(bytes_moved / (apply_avg * 1e-3) / 1e9 / plain_gbps) if plain_gbps else None)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(model, pa, pb, rank if rank >= 0 else 0, cf.seed_of(args.workload))

    out = {
        "metric": "resharded state GB/s (read+write)", "value": bytes_moved / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16+u32", "data": "synthetic",
        "config": {"workload": f"{args.workload} rank {rank}" if rank >= 0 else f"{args.workload} all ranks",
                   "src": pa, "dst": pb, "step": (args.only + " only") if args.only else ("apply only" if args.apply_only else "describe x2 + plan + apply"),
                   "through_buffers": bool(args.through_buffers),
                   "tile_bytes": args.tile_bytes or 8192},
        "breakdown_ms": {"describe_x2": _median(t_desc), "plan": _median(t_plan), "apply_kernels": apply_avg},
        "apply_gbps": bytes_moved / (apply_avg * 1e-3) / 1e9,
        "pct_hbm_peak_apply": 100.0 * bytes_moved / (apply_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "bytes": {"send": info["send_total"], "recv": info["recv_total"], "retain": info["retain_total"],
                  "moved_read_plus_write": bytes_moved},
        "plan": {k: st[k] for k in ("num_boxes", "num_retain_tiles", "num_pack_tiles", "num_unpack_tiles",
                                    "num_peers_out", "num_peers_in")},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if stage is not None:
        out["staged"] = dict(budget_mib=args.staged_mib, **sinfo, one_shot_scratch=info["scratch_needed"])
    print(json.dumps(out))


def _median(v):
    return sorted(v)[len(v) // 2] if v else None


def cpu_baseline(model, pa, pb, rank, seed, target_seconds=12.0):
    """The per-element oracle on the host cores, on a bounded sample of the same rank's share:
    the first `per` offsets of every destination buffer, `per` sized from a short pilot so that
    the sample takes about target_seconds."""
    import oracle
    a, b = oracle.Config(model, pa), oracle.Config(model, pb)
    bufs = [buf for buf in range(8) if b.buffer_elems(rank, buf)]
    pilot = 4_000_000
    t0 = time.perf_counter()
    done = 0
    for buf in bufs:
        n = min(pilot, b.buffer_elems(rank, buf))
        oracle.expected(a, b, rank, buf, seed, n=n)
        done += n
    rate = done / (time.perf_counter() - t0)
    per = max(pilot, int(rate * target_seconds) // max(len(bufs), 1))
    nbytes = 0
    t0 = time.perf_counter()
    for buf in bufs:
        n = min(per, b.buffer_elems(rank, buf))
        oracle.expected(a, b, rank, buf, seed, n=n)
        nbytes += n * oracle.KIND_BYTES[buf % 4]
    dt = time.perf_counter() - t0
    # the same on one core, on a sixteenth of the sample
    cores = oracle.num_threads()
    oracle.set_num_threads(1)
    nb1 = 0
    t1 = time.perf_counter()
    for buf in bufs:
        n = min(per // 16, b.buffer_elems(rank, buf))
        oracle.expected(a, b, rank, buf, seed, n=n)
        nb1 += n * oracle.KIND_BYTES[buf % 4]
    dt1 = time.perf_counter() - t1
    oracle.set_num_threads(cores)
    return dict(value=2 * nbytes / dt / 1e9, unit="GB/s", cores=cores, kind="oracle",
                value_one_core=2 * nb1 / dt1 / 1e9,
                sample=f"first {per} elements (or all) of each of the {len(bufs)} destination buffers of rank {rank} "
                       f"({nbytes} bytes) through the per-element oracle (coordinate, owners, source rule, word)",
                seconds=dt)


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the VPS state transition on one MI355X.

One step = one pass of the whole path for one rank's share of the workload: map both
configurations onto the VPS (vps_describe_config x2), plan the intersections
(vps_plan_intersections) and move the data (vps_apply_transition: retain + pack + unpack in one
launch).  State buffers and the peers' receive buffer are resident in HBM before the timed
region.  The JSON line reports bytes moved (read + write) per second over the whole step, and
for the copy kernel alone the achieved HBM rate against the 8 TB/s peak.

After the headline the default run also times, with the plan reused, the copy of every other
workload (`workloads`), the planning of all ranks of the two large transitions (`planning`) and
a plain copy, a read-only and a write-only kernel in the copy engine's launch shape (inside
`roofline`); `--headline-only` skips the first two.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def kernel_sources_fingerprint():
    """Hash of the library's sources: a stored counter figure is only reported next to a run of
    the same kernels."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2605_18815_amd", "csrc")
    for name in sorted(os.listdir(d)):
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def _median(v):
    return sorted(v)[len(v) // 2] if v else None


class Resident:
    """One workload with its state resident in HBM: source buffers (seeded random bytes),
    destination buffers, scratch (its receive part stands in for the peers' packed data)."""

    def __init__(self, lib, vps, cf, torch, name, rank=None, src_over=None, dst_over=None, through=False):
        self.lib, self.torch, self.name = lib, torch, name
        w = cf.workload(name)
        self.model, self.pa, self.pb = w["model"], dict(w["src"]), dict(w["dst"])
        self.pa.update(src_over or {})
        self.pb.update(dst_over or {})
        # the C structs of the three descriptors, made once: the timed calls pass them as they are
        self.model_c, self.pa_c, self.pb_c = (vps.binding.model_desc(self.model), vps.binding.parallel_desc(self.pa),
                                              vps.binding.parallel_desc(self.pb))
        self.rank = rank if rank is not None else (w["rank"] if w["rank"] is not None else -1)
        self.flags = vps.binding.PLAN_THROUGH_BUFFERS if through else 0
        self.through = through
        self.stream = torch.cuda.current_stream().cuda_stream
        dev = torch.device("cuda:0")
        ca, cb = lib.describe_config(self.model, self.pa), lib.describe_config(self.model, self.pb)
        self.plan = lib.plan_intersections_ex(ca, cb, self.rank, self.flags, self.stream)
        self.info = self.plan.buffer_bytes(self.rank)
        gen = torch.Generator(device=dev)
        gen.manual_seed(cf.seed_of(name))

        def alloc(nbytes, rand):
            t = torch.empty(int(nbytes), dtype=torch.uint8, device=dev)
            if rand and nbytes:
                t.view(torch.int32)[: nbytes // 4].random_(generator=gen) if nbytes % 4 == 0 else t.random_(generator=gen)
            return t

        self.alloc = alloc
        rank = self.rank
        src_ranks = [rank] if rank >= 0 else list(range(ca.world))
        dst_ranks = [rank] if rank >= 0 else list(range(cb.world))
        self.src = [alloc(ca.buffer_bytes(r, b) if r < ca.world else 0, True) for r in src_ranks for b in range(8)]
        self.dst = [alloc(cb.buffer_bytes(r, b) if r < cb.world else 0, False) for r in dst_ranks for b in range(8)]
        self.scratch = alloc(self.info["scratch_needed"], True)
        self.sp = [t.data_ptr() if t.numel() else 0 for t in self.src]
        self.dp = [t.data_ptr() if t.numel() else 0 for t in self.dst]
        info = self.info
        payload = info["send_total"] + info["recv_total"] + info["retain_total"]
        if rank < 0:
            payload = 2 * info["send_total"] + info["retain_total"]   # every byte is packed and unpacked here
        self.bytes_moved = 2 * payload
        torch.cuda.synchronize()

    def label(self):
        return f"{self.name} rank {self.rank}" if self.rank >= 0 else f"{self.name} all ranks"

    def apply(self, plan=None):
        self.lib.apply_transition(plan or self.plan, self.rank, self.sp, self.dp, self.scratch.data_ptr(),
                                  self.scratch.numel(), self.stream)

    def full_step(self):
        a, b = self.lib.describe_config(self.model_c, self.pa_c), self.lib.describe_config(self.model_c, self.pb_c)
        p = self.lib.plan_intersections_ex(a, b, self.rank, self.flags, self.stream)
        self.apply(p)
        return p

    def time_apply(self, steps, warmup):
        torch = self.torch
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for k in range(-warmup, steps):
            if k >= 0:
                ev[k][0].record()
            self.apply()
            if k >= 0:
                ev[k][1].record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in ev)


def time_calls(torch, fn, reps=10, warm=2):
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for k in range(-warm, reps):
        if k >= 0:
            ev[k][0].record()
        fn()
        if k >= 0:
            ev[k][1].record()
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in ev) / reps


def memory_system_rates(lib, torch, nbytes, stream):
    """A plain copy, a read-only and a write-only kernel in the copy engine's launch shape."""
    dev = torch.device("cuda:0")
    # destination 8448 bytes off the source's alignment: with equal offsets on both sides the
    # reads and writes of a tile fall on the same memory channels and a plain copy loses 2 %
    shift = 8448
    x = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    x.view(torch.int32).random_()
    y = torch.empty(nbytes + shift, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4, dtype=torch.uint8, device=dev)
    copy_ms = time_calls(torch, lambda: lib.plain_copy(y.data_ptr() + shift, x.data_ptr(), nbytes, stream))
    read_ms = time_calls(torch, lambda: lib.plain_read(x.data_ptr(), nbytes, sink.data_ptr(), stream))
    fill_ms = time_calls(torch, lambda: lib.plain_fill(y.data_ptr() + shift, nbytes, stream))
    del x, y
    rd, wr = nbytes / (read_ms * 1e-3) / 1e9, nbytes / (fill_ms * 1e-3) / 1e9
    return dict(plain_copy_gbps=2 * nbytes / (copy_ms * 1e-3) / 1e9, read_only_gbps=rd, write_only_gbps=wr,
                read_write_harmonic_gbps=2.0 / (1.0 / rd + 1.0 / wr))


def planning_rate(lib, vps, cf, torch, name, reps=5):
    """All ranks of a transition planned at once (routes only): boxes per second."""
    w = cf.workload(name)
    stream = torch.cuda.current_stream().cuda_stream
    t_desc, t_plan, boxes = [], [], 0
    for _ in range(reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a, b = lib.describe_config(w["model"], w["src"]), lib.describe_config(w["model"], w["dst"])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        p = lib.plan_intersections_ex(a, b, -1, vps.binding.PLAN_ROUTES_ONLY, stream)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        t_desc.append((t1 - t0) * 1e3)
        t_plan.append((t2 - t1) * 1e3)
        boxes = p.num_boxes
        del a, b, p
    ms = _median(t_plan[1:])
    return dict(workload=f"{name} all {cf.world(w['src'])} -> {cf.world(w['dst'])} ranks, routes only", boxes=boxes,
                describe_x2_ms=_median(t_desc[1:]), ms=ms, mboxes_per_s=boxes / (ms * 1e-3) / 1e6)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gqa70b")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--tile-bytes", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="skip the other workloads and the planning rates")
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

    def overrides(spec):
        return {k: int(v) for k, v in (kv.split("=") for kv in filter(None, spec.split(",")))}

    if args.workload in cf.PAPER_TRANSITIONS and args.rank is None:
        sys.exit("bench.py: the paper's transitions do not fit one GPU with every rank resident; pass --rank")
    variant = bool(args.tile_bytes or args.src or args.dst or args.through_buffers or args.only or args.staged_mib)
    extras = not args.headline_only and not variant and args.workload == "gqa70b" and args.rank is None
    if extras:
        # One all-ranks plan of each kind before anything else, so that the library's table pool gets
        # its blocks while device memory is fresh.  (Blocks first allocated after the 100 GB workloads
        # below have come and gone make the same plans 35 % slower: 0.36 / 0.68 instead of 0.27 / 0.50 ms.)
        for n in ("gqa70b", "moe235b"):
            planning_rate(lib, vps, cf, torch, n, reps=1)
    R = Resident(lib, vps, cf, torch, args.workload, args.rank, overrides(args.src), overrides(args.dst), args.through_buffers)
    rank, info, stream, plan = R.rank, R.info, R.stream, R.plan
    bytes_moved = R.bytes_moved
    if args.only:
        assert rank >= 0, "--only needs a single-rank workload"
        args.apply_only = True
        bytes_moved = 2 * (info["send_total"] if args.only == "pack" else info["recv_total"])
    stage = None
    if args.staged_mib:
        assert rank < 0, "--staged-mib needs a workload with all ranks resident"
        stage = lib.stage_exchange(plan, args.staged_mib << 20, stream)
        sinfo = stage.info()
        R.scratch = R.alloc(sinfo["scratch_needed"], False)
        # pack, exchange and unpack each read and write the exchanged bytes once
        bytes_moved = 2 * (3 * info["send_total"] + info["retain_total"])
    torch.cuda.synchronize()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]

    def one_step(k=None):
        if args.apply_only:
            p = plan
        else:
            a2, b2 = lib.describe_config(R.model_c, R.pa_c), lib.describe_config(R.model_c, R.pb_c)
            p = lib.plan_intersections_ex(a2, b2, rank, R.flags, stream)
        stg = None
        if stage is not None:
            stg = stage if args.apply_only else lib.stage_exchange(p, args.staged_mib << 20, stream)
        if k is not None:
            ev[k][0].record()
        if stg is not None:
            lib.apply_transition_staged(stg, R.sp, R.dp, R.scratch.data_ptr(), R.scratch.numel(), stream)
        elif args.only == "pack":
            lib.pack(p, rank, R.sp, R.scratch.data_ptr(), stream)
        elif args.only == "unpack":
            lib.unpack(p, rank, R.scratch.data_ptr() + info["recv_offset"], R.dp, stream)
        else:
            R.apply(p)
        if k is not None:
            ev[k][1].record()
        return (p, stg)

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
    # mapping and planning alone, device idle before and after each (not part of the timed region)
    t_desc, t_plan = [], []
    for _ in range(7):
        torch.cuda.synchronize()
        ta = time.perf_counter()
        a2, b2 = lib.describe_config(R.model_c, R.pa_c), lib.describe_config(R.model_c, R.pb_c)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        p2 = lib.plan_intersections_ex(a2, b2, rank, R.flags, stream)
        torch.cuda.synchronize()
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
    # HBM bytes per launch as measured beforehand with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE for
    # this very workload and tile size: a stored figure of profiles/, null for anything else
    traffic, traffic_source = None, None
    prof = os.path.join(ROOT, "profiles", f"k_copy_tiles_{args.workload}_rank{rank}_hbm_traffic.txt")
    fingerprint = kernel_sources_fingerprint()
    if os.path.exists(prof) and not variant:
        stored = {k.strip(): v.strip() for k, v in (ln.split("=", 1) for ln in open(prof) if "=" in ln and not ln.startswith(" "))}
        if stored.get("kernel_sources_fingerprint") == fingerprint and "traffic_bytes_per_launch" in stored:
            traffic = int(stored["traffic_bytes_per_launch"])
            traffic_source = "stored profile figure: profiles/" + os.path.basename(prof)
        else:
            traffic_source = ("none: profiles/" + os.path.basename(prof) + " was measured on other kernel sources (fingerprint "
                              + stored.get("kernel_sources_fingerprint", "missing") + ", now " + fingerprint + ")")
    achieved = bytes_moved / (apply_avg * 1e-3) / 1e9
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s", frac=achieved / HBM_PEAK_GBPS,
                    traffic=traffic, traffic_source=traffic_source,
                    kernel_sources_fingerprint=fingerprint,
                    kernel="k_copy_tiles", launches_per_step=launches, kernel_ms_avg=apply_avg,
                    kernel_ms_median=apply_ms[len(apply_ms) // 2], algorithmic_bytes_per_step=bytes_moved)

    out = {
        "metric": "resharded state GB/s (read+write)", "value": bytes_moved / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16+u32", "data": "synthetic",
        "config": {"workload": R.label(),
                   "src": R.pa, "dst": R.pb, "step": (args.only + " only") if args.only else ("apply only" if args.apply_only else "describe x2 + plan + apply"),
                   "through_buffers": bool(args.through_buffers),
                   "tile_bytes": args.tile_bytes or 8192},
        "breakdown_ms": {"describe_x2": _median(t_desc), "plan": _median(t_plan), "apply_kernels": apply_avg},
        "apply_gbps": achieved,
        "pct_hbm_peak_apply": 100.0 * achieved / HBM_PEAK_GBPS,
        "bytes": {"send": info["send_total"], "recv": info["recv_total"], "retain": info["retain_total"],
                  "moved_read_plus_write": bytes_moved},
        "plan": {k: st[k] for k in ("num_boxes", "num_retain_tiles", "num_pack_tiles", "num_unpack_tiles",
                                    "num_peers_out", "num_peers_in")},
        "roofline": roofline,
    }
    if stage is not None:
        out["staged"] = dict(budget_mib=args.staged_mib, **sinfo, one_shot_scratch=info["scratch_needed"])

    # ---- the memory system under the same launch shape
    ceil_bytes = min(bytes_moved // 2, 8 << 30) // 16 * 16
    del R, plan, stage
    gc.collect()
    torch.cuda.empty_cache()
    if ceil_bytes >= (64 << 20):
        rates = memory_system_rates(lib, torch, ceil_bytes, stream)
        roofline.update(rates)
        roofline["frac_of_plain_copy"] = achieved / rates["plain_copy_gbps"]
        roofline["frac_of_read_write_harmonic"] = achieved / rates["read_write_harmonic_gbps"]

    # ---- every other workload (copy alone, plan reused) and the planning of all ranks
    if extras:
        others = [("toy", {}, {}), ("gpt1p3b", {}, {}), ("gqa8b", {}, {}), ("moe235b", {}, {}),
                  ("moe235b", {}, {"expert_layout": 1}), ("gqa70b-odd", {}, {})]
        rows = [dict(workload="gqa70b rank 11", moved=bytes_moved, apply_ms=apply_avg, gbps=achieved, frac=achieved / HBM_PEAK_GBPS)]
        for name, so, do in others:
            gc.collect()
            torch.cuda.empty_cache()
            W = Resident(lib, vps, cf, torch, name, None, so, do)
            ms = W.time_apply(steps=10, warmup=2)
            avg = sum(ms) / len(ms)
            g = W.bytes_moved / (avg * 1e-3) / 1e9
            label = W.label() + ("".join(f", destination {k}={v}" for k, v in do.items()))
            rows.append(dict(workload=label, moved=W.bytes_moved, apply_ms=avg, gbps=g, frac=g / HBM_PEAK_GBPS))
            del W
        out["workloads"] = rows
        gc.collect()
        torch.cuda.empty_cache()
        out["planning"] = [planning_rate(lib, vps, cf, torch, n) for n in ("gqa70b", "moe235b")]

    cpu = None
    if not args.no_cpu_baseline:
        w = cf.workload(args.workload)
        pa, pb = dict(w["src"]), dict(w["dst"])
        pa.update(overrides(args.src))
        pb.update(overrides(args.dst))
        cpu = cpu_baseline(w["model"], pa, pb, rank if rank >= 0 else 0, cf.seed_of(args.workload))
    out["cpu_baseline"] = cpu
    print(json.dumps(out))


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

"""Is the parity suite sharp?  Plant one plausible mistake at a time in a copy of the library's
per-item code, build the CPU variant of it (tests/hostcheck), and require that the parity
procedures against the oracle notice.  Everything here runs on the CPU; the mistake is never
compiled for, or run on, a GPU."""
import os
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTANTS = [m for m in [
    ("V block of blocked QKV at K's place", "vps_core.h", "bo = b == 0 ? 0 : (b == 1 ? P.q_per_g : P.q_per_g + 1);",
     "bo = b == 0 ? 0 : (b == 1 ? P.q_per_g + 1 : P.q_per_g);"),
    ("source offset of a box with the destination's strides", "vps_core.h",
     "b.src_off += (int64_t)(b.lo[a] - sp.lo[a]) * sp.stride[a];", "b.src_off += (int64_t)(b.lo[a] - sp.lo[a]) * dp.stride[a];"),
    ("replica choice ignores the data-parallel index", "vps_core.h", "int32_t want = dpj % n_node;", "int32_t want = 0 % n_node;"),
    ("partial last vector of a run dropped at a window end", "vps_core.h",
     "const bool has_tail = tailb && !(wl == 0 && head) && wl >= w0 && wl < wend_win;",
     "const bool has_tail = tailb && !(wl == 0 && head) && wl >= w0 && wl + 1 < wend_win;"),
    ("retained boxes get buffer positions", "vps_core.h",
     "    if (!box_retained(b, through_buffers)) {\n        if (planned_rank < 0 || b.src_rank == planned_rank) r.bytes_flags |= ORD_SENDS;",
     "    if (b.tensor >= 0) {\n        if (planned_rank < 0 || b.src_rank == planned_rank) r.bytes_flags |= ORD_SENDS;"),
    ("receive order counted with the send key", "vps_core.h",
     "const bool less_r = r.key_r < me.key_r || (r.key_r == me.key_r && r.klo < me.klo);",
     "const bool less_r = r.key_s < me.key_s || (r.key_s == me.key_s && r.klo < me.klo);"),
    ("positions counted from the start of all buffers", "vps_pipeline.h",
     "if (rec.bytes_flags & ORD_SENDS) b.send_pos = o.gpos_s - o.base_s;", "if (rec.bytes_flags & ORD_SENDS) b.send_pos = o.gpos_s;"),
    ("sorted path: positions counted from the start of all buffers", "vps_pipeline.h",
     "const uint64_t rel = g[k] - g[lo];", "const uint64_t rel = g[k];"),
    ("pair by pair: receive offsets from the box counts", "vps_pipeline.h",
     "for (int64_t q = 0; q < i; ++q) { at += pcount[q * WB + d]; off += pbytes[q * WB + d]; }",
     "for (int64_t q = 0; q < i; ++q) { at += pcount[q * WB + d]; off += pcount[q * WB + d]; }"),
    ("pair by pair: a box counts itself among those before it", "vps_core.h",
     "VPS_HD bool pair_rec_less(const PairRec& a, const PairRec& b) { return a.key < b.key || (a.key == b.key && a.klo < b.klo); }",
     "VPS_HD bool pair_rec_less(const PairRec& a, const PairRec& b) { return a.key < b.key || (a.key == b.key && a.klo <= b.klo); }"),
    ("cuts of a long run follow the descriptor to its new place", "vps_core.h",
     "const int64_t pre = (int64_t)((d.xa + to) & (run_cut_align(d.vec_window) - 1)), win = 16ll * d.vec_window;",
     "const int64_t pre = (int64_t)((d.dst_byte + to) & (run_cut_align(d.vec_window) - 1)), win = 16ll * d.vec_window;"),
    ("expert ranks with ep and expert-dp digits swapped", "vps_core.h",
     "return group ? t + P.etp * (ep + P.ep * (d + P.edp * pp)) : t + P.tp * (d + P.ddp * pp);",
     "return group ? t + P.etp * (d + P.edp * (ep + P.ep * pp)) : t + P.tp * (d + P.ddp * pp);"),
    ("kinds in plain order inside a peer segment", "vps_core.h", "const uint64_t korder = (uint64_t)((b.kind + 3) & 3);",
     "const uint64_t korder = (uint64_t)b.kind;"),
    ("unpack reads at the sender's position", "vps_core.h", "d.src_byte = b.recv_pos;", "d.src_byte = b.send_pos;"),
    ("a rank's first box counted by the boxes it receives", "vps_pipeline.h", "be_atomic_add(rank_rows + b.src_rank, 1);",
     "be_atomic_add(rank_rows + b.dst_rank, 1);"),
    ("axes merged when only the source side is contiguous", "vps_core.h",
     "if (m > 0 && o3.s == x[i].s * x[i].e && o3.d == x[i].d * x[i].e && o3.e * x[i].e < ((int64_t)1 << 31)) {",
     "if (m > 0 && o3.s == x[i].s * x[i].e && o3.e * x[i].e < ((int64_t)1 << 31)) {"),
    ("large plans: a rank's first box moved to its last", "vps_pipeline.h",
     "for (int32_t r = ps + 1; r <= cs; ++r) rt[0 * (W + 1) + r] = k;",
     "for (int32_t r = ps < 0 ? 0 : ps; r <= cs; ++r) rt[0 * (W + 1) + r] = k;"),
    ("pair by pair: what a rank keeps counted as sent", "vps_pipeline.h",
     "const uint64_t own = (!through_buffers && i < WB) ? pcount[i * WB + i] : 0;", "const uint64_t own = 0;"),
    ("pairs counted by the emission: every box counts as travelling", "vps_core.h",
     "be_atomic_add_runs(pc.bytes, pr, (rec.bytes_flags & ORD_SENDS) ? (rec.bytes_flags & ~(uint64_t)15) : 0);",
     "be_atomic_add_runs(pc.bytes, pr, rec.bytes_flags & ~(uint64_t)15);"),
    ("block extent of a transpose not clipped", "vps_core.h",
     "ta = ext_xa - a0 < (uint32_t)XPOSE_T ? ext_xa - a0 : (uint32_t)XPOSE_T;", "ta = (uint32_t)XPOSE_T;"),
] if m[2] is not None]   # (entries without a site are mistakes only a device build could hold)

PARITY = "all_ranks_resident or single_rank_share or medium_shapes or beyond_the_counting_limit"
# the tests expected to notice a mistake first, for mistakes on paths that few tests take
FIRST = {
    "sorted path: positions counted from the start of all buffers": "beyond_the_counting_limit and sort",
    "pair by pair: receive offsets from the box counts": "beyond_the_counting_limit and pairs",
    "pair by pair: a box counts itself among those before it": "beyond_the_counting_limit and pairs",
    "cuts of a long run follow the descriptor to its new place": "moves_long_runs",
    "large plans: a rank's first box moved to its last": "beyond_the_counting_limit",
    "pair by pair: what a rank keeps counted as sent": "beyond_the_counting_limit and pairs",
    "pairs counted by the emission: every box counts as travelling": "beyond_the_counting_limit and pairs",
}


@pytest.mark.parametrize("name,header,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_parity_suite_catches_planted_mistake(name, header, old, new):
    with tempfile.TemporaryDirectory() as tmp:
        shutil.copytree(os.path.join(ROOT, "paper_2605_18815_amd", "csrc"), os.path.join(tmp, "paper_2605_18815_amd", "csrc"))
        shutil.copytree(os.path.join(ROOT, "include"), os.path.join(tmp, "include"))
        os.makedirs(os.path.join(tmp, "tests", "hostcheck"))
        shutil.copy(os.path.join(ROOT, "tests", "hostcheck", "hostcheck.cpp"), os.path.join(tmp, "tests", "hostcheck"))
        path = os.path.join(tmp, "paper_2605_18815_amd", "csrc", header)
        src = open(path).read()
        assert src.count(old) == 1, f"mutation site for '{name}' not found exactly once"
        open(path, "w").write(src.replace(old, new))
        lib = os.path.join(tmp, "libmutant.so")
        subprocess.run(["g++", "-std=c++17", "-O0", "-fPIC", "-shared", "-o", lib,
                        os.path.join(tmp, "tests", "hostcheck", "hostcheck.cpp")], check=True)
        res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_hostcheck_parity.py"), "-x", "-q",
                              "-k", FIRST.get(name, PARITY), "-p", "no:cacheprovider"], env=dict(os.environ, VPSH_LIB=lib), cwd=ROOT,
                             capture_output=True, text=True)
        # a failed comparison, or the CPU build running off its tables (it is then killed by a signal)
        assert res.returncode != 0, f"no parity test noticed the planted mistake '{name}'"

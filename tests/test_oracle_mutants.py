"""Are the pins of the oracle sharp?  Plant one plausible mistake at a time in a copy of the
oracle's source (on the CPU), rebuild it, and require that the pin suite notices.

Every mutant is a single edit of oracle/vps_oracle.c: a dropped term, a wrong index, a swapped
operand.  The pins run in a subprocess against the mutated library (ORACLE_LIB)."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "vps_oracle.c")

MUTANTS = [
    ("pipeline split rounds up", "long lo = ((long)p * L) / PP, hi = ((long)(p + 1) * L) / PP;",
     "long lo = ((long)p * L + PP - 1) / PP, hi = ((long)(p + 1) * L + PP - 1) / PP;"),
    ("rank digits swapped", "return tp + c->p.tp * (ddp + c->ddp * pp);",
     "return ddp + c->ddp * (tp + c->p.tp * pp);"),
    ("transposed gate_up stored as (h, f, 2)", "s->order[1] = 3; s->order[2] = 1; s->order[3] = 2;",
     "s->order[1] = 3; s->order[2] = 2; s->order[3] = 1;"),
    ("padding quantum 4*D", "uint64_t q = 8ull * (uint64_t)(g == 0 ? c->ddp : c->edp);",
     "uint64_t q = 4ull * (uint64_t)(g == 0 ? c->ddp : c->edp);"),
    ("K and V blocks swapped", "s->blo[1] = c->q_per_g;      s->blen[1] = 1;          /* K */\n        s->blo[2] = c->q_per_g + 1;  s->blen[2] = 1;          /* V */",
     "s->blo[1] = c->q_per_g + 1;  s->blen[1] = 1;\n        s->blo[2] = c->q_per_g;      s->blen[2] = 1;"),
    ("flat shard owner off by one element", "if (f / per != (uint64_t)di) continue;", "if ((f + 1) / per != (uint64_t)di) continue;"),
    ("descending flat order ignored", "int t = p->flat_order ? c->nt - 1 - q : q;", "int t = q;"),
    ("linear index uses the wrong extent", "return (((uint64_t)cd[0] * (uint64_t)s[1] + (uint64_t)cd[1]) * (uint64_t)s[2] + (uint64_t)cd[2]) *",
     "return (((uint64_t)cd[0] * (uint64_t)s[1] + (uint64_t)cd[1]) * (uint64_t)s[1] + (uint64_t)cd[2]) *"),
    ("TP shards in reverse order", "s->lo[x->tp_axis] = tp * s->ext[x->tp_axis];", "s->lo[x->tp_axis] = (c->p.tp - 1 - tp) * s->ext[x->tp_axis];"),
    ("expert block by modulo", "return expert / (c->m.experts / c->p.ep);", "return expert % c->p.ep;"),
    ("retain rule dropped", "if (r[k] == j) pick = k; /* the destination rank already holds it: retain */", "(void)j;"),
    ("node preference ignored", "if (r[k] / a->p.gpus_per_node == node) idx[m++] = k;", "if (node >= 0) idx[m++] = k;"),
    ("replica chosen by the destination's rank instead of its data-parallel index", "pick = idx[dpi % m];", "pick = idx[j % m];"),
    ("piece level ignores the end of the flat range", "if (unit >= v0 && unit + st[q] <= v1) break;", "if (unit >= v0) break;"),
    ("peer buffer orders kinds 0, 1, 2, 3", "const int kx = (x->id.kind + 3) & 3, ky = (y->id.kind + 3) & 3; /* kinds 1, 2, 3, then 0 */",
     "const int kx = x->id.kind, ky = y->id.kind;"),
    ("boxes of a peer buffer not aligned to 16 bytes", "pos += (ord[k]->count * (ord[k]->id.kind == 0 ? 2u : 4u) + 15u) & ~(uint64_t)15;",
     "pos += ord[k]->count * (ord[k]->id.kind == 0 ? 2u : 4u);"),
    ("expert ranks: ep and expert-dp digits swapped", "return etp + c->etp * (ep + c->p.ep * (edp + c->edp * pp));",
     "return etp + c->etp * (edp + c->edp * (ep + c->p.ep * pp));"),
    ("carved expert dp degree forgets tp", "c->ddp = p->dp; c->etp = 1; c->edp = p->tp * p->dp / p->ep;", "c->ddp = p->dp; c->etp = 1; c->edp = p->dp;"),
    ("box serialised with the two inner axes swapped", "for (int ax = 0; ax < 4; ++ax) idx = idx * (uint64_t)(e->hi[ax] - e->lo[ax] + 1) + (uint64_t)(cd[ax] - e->lo[ax]);",
     "for (int q = 0; q < 4; ++q) { int ax = q == 2 ? 3 : (q == 3 ? 2 : q); idx = idx * (uint64_t)(e->hi[ax] - e->lo[ax] + 1) + (uint64_t)(cd[ax] - e->lo[ax]); }"),
    ("transition copies from the wrong offset", "if (kind == 0) ((uint16_t*)dst)[k] = ((const uint16_t*)src)[so];", "if (kind == 0) ((uint16_t*)dst)[k] = ((const uint16_t*)src)[so ^ 1];"),
]

PINS = ("textbook or bruteforce or assemble or closed_form or figure4 or figure6 or identity or region_algebra or moves_whole "
        "or hand_table or hand_example or pieces or recv_payload or source_rule or written_out_by_hand")


# The pins that are expected to notice each mistake first (running only those keeps the CPU suite
# short); a mutant without an entry runs the whole selection above.
FIRST_PINS = {
    "pipeline split rounds up": "hand_table",
    "rank digits swapped": "bruteforce and gpt-tp2dp2z1",
    "padding quantum 4*D": "textbook and odd",
    "expert block by modulo": "hand_table",
    "retain rule dropped": "identity",
    "node preference ignored": "source_rule",
    "replica chosen by the destination's rank instead of its data-parallel index": "source_rule or region_algebra",
    "piece level ignores the end of the flat range": "pieces",
    "peer buffer orders kinds 0, 1, 2, 3": "written_out_by_hand",
    "boxes of a peer buffer not aligned to 16 bytes": "written_out_by_hand or (recv_payload and gpt-odd)",
    "expert ranks: ep and expert-dp digits swapped": "bruteforce and moe",
    "carved expert dp degree forgets tp": "hand_example or (textbook and carved)",
    "box serialised with the two inner axes swapped": "recv_payload and gpt-tp-pp",
    "transition copies from the wrong offset": "assemble and gpt-tp-pp",
}


def _run_pins(lib_path, select):
    env = dict(os.environ, ORACLE_LIB=lib_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-k", select, "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True)


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        msrc = os.path.join(tmp, "vps_oracle.c")
        open(msrc, "w").write(src.replace(old, new).replace('#include "vps_oracle.h"', f'#include "{ROOT}/oracle/vps_oracle.h"')
                              .replace('#include "../datagen/pattern.h"', f'#include "{ROOT}/datagen/pattern.h"'))
        lib = os.path.join(tmp, "libmutant.so")
        subprocess.run(["gcc", "-std=c11", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", lib, msrc], check=True)
        res = _run_pins(lib, FIRST_PINS.get(name, PINS))
        assert res.returncode != 0, f"no pin noticed the planted mistake '{name}'"
        assert "failed" in res.stdout or "error" in res.stdout.lower()

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
    ("padding quantum 4*D", "uint64_t q = 8ull * (uint64_t)(g == 0 ? c->ddp : p->dp);",
     "uint64_t q = 4ull * (uint64_t)(g == 0 ? c->ddp : p->dp);"),
    ("K and V blocks swapped", "s->blo[1] = c->q_per_g;      s->blen[1] = 1;          /* K */\n        s->blo[2] = c->q_per_g + 1;  s->blen[2] = 1;          /* V */",
     "s->blo[1] = c->q_per_g + 1;  s->blen[1] = 1;\n        s->blo[2] = c->q_per_g;      s->blen[2] = 1;"),
    ("flat shard owner off by one element", "if (f / per != (uint64_t)di) continue;", "if ((f + 1) / per != (uint64_t)di) continue;"),
    ("descending flat order ignored", "int t = p->flat_order ? c->nt - 1 - q : q;", "int t = q;"),
    ("linear index uses the wrong extent", "return (((uint64_t)cd[0] * (uint64_t)s[1] + (uint64_t)cd[1]) * (uint64_t)s[2] + (uint64_t)cd[2]) *",
     "return (((uint64_t)cd[0] * (uint64_t)s[1] + (uint64_t)cd[1]) * (uint64_t)s[1] + (uint64_t)cd[2]) *"),
    ("TP shards in reverse order", "s->lo[x->tp_axis] = tp * s->ext[x->tp_axis];", "s->lo[x->tp_axis] = (c->p.tp - 1 - tp) * s->ext[x->tp_axis];"),
    ("expert block by modulo", "return expert / (c->m.experts / c->p.ep);", "return expert % c->p.ep;"),
    ("retain rule dropped", "if (r[k] == j) pick = k; /* the destination rank already holds it: retain */", "(void)j;"),
    ("transition copies from the wrong offset", "if (kind == 0) ((uint16_t*)dst)[k] = ((const uint16_t*)src)[so];", "if (kind == 0) ((uint16_t*)dst)[k] = ((const uint16_t*)src)[so ^ 1];"),
]

PINS = "textbook or bruteforce or assemble or closed_form or figure4 or figure6 or identity or region_algebra or moves_whole"


def _run_pins(lib_path):
    env = dict(os.environ, ORACLE_LIB=lib_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-k", PINS, "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True)


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
        res = _run_pins(lib)
        assert res.returncode != 0, f"no pin noticed the planted mistake '{name}'"
        assert "failed" in res.stdout or "error" in res.stdout.lower()

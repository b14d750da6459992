"""Seeded random transitions on tiny models: random degrees, layouts, ZeRO on/off, node sizes
and world-size changes.  A configuration is kept only if the oracle accepts it; the library has
to agree on which ones are legal."""
import random

import oracle
import parity
from datagen import configs as cf

MODELS = [cf.TINY_GPT, cf.TINY_GQA, cf.TINY_MOE, cf.ODD_GPT, cf.ODD_MOE]
MAX_WORLD = 48


def random_parallel(rng, m):
    moe = m["family"] == cf.FAMILY_MOE
    return cf.parallel(tp=rng.choice([1, 1, 2, 2, 3, 4]), pp=rng.choice([1, 1, 2, 3, 4]),
                       dp=rng.choice([1, 1, 2, 3, 4]), ep=rng.choice([1, 2, 3, 4]) if moe else 1,
                       zero=rng.choice([0, 1, 1]), gpus_per_node=rng.choice([2, 4, 8]),
                       qkv_layout=rng.choice([0, 1]), expert_layout=rng.choice([0, 1]) if moe else 0,
                       flat_order=rng.choice([0, 0, 1]),
                       # drawn from a stream of its own, so that the other fields keep their values
                       ep_placement=random.Random(rng.random()).choice([0, 0, 1]) if moe else 0)


def legal(lib, m, p):
    from paper_2605_18815_amd.binding import VpsError
    try:
        oracle.Config(m, p)
        ok = True
    except oracle.OracleError:
        ok = False
    try:
        lib.describe_config(m, p)
        lib_ok = True
    except VpsError:
        lib_ok = False
    assert ok == lib_ok, ("the oracle and the library disagree on whether a configuration is legal", m, p)
    return ok


def cases(first_seed, count):
    """(seed, model, source, destination, mode, rank) of `count` cases, without calling the library."""
    out, s = [], first_seed
    while len(out) < count:
        rng = random.Random(s)
        m = rng.choice(MODELS)
        pa, pb = random_parallel(rng, m), random_parallel(rng, m)
        mode = rng.choice(["all", "all", "single", "through", "staged", "classify"])
        rank = rng.randrange(max(cf.world(pa), cf.world(pb)))
        if cf.world(pa) <= MAX_WORLD and cf.world(pb) <= MAX_WORLD:
            out.append((s, m, pa, pb, mode, rank))
        s += 1
    return out


def run_case(lib, mem_factory, case):
    s, m, pa, pb, mode, rank = case
    if not (legal(lib, m, pa) and legal(lib, m, pb)):
        return False
    if mode == "single":
        parity.run_single_rank(lib, mem_factory(), m, pa, pb, rank, seed=s)
    elif mode == "staged":
        # budget drawn from the seed: from "every step its own stage" to "one stage"
        budget = [1, 1 << 12, 1 << 16, 1 << 60][s % 4]
        parity.run_staged(lib, mem_factory(), m, pa, pb, seed=s, budget=budget)
    elif mode == "classify":
        parity.run_classify(lib, m, pa, pb)
    else:
        parity.run_all_ranks(lib, mem_factory(), m, pa, pb, seed=s, through=(mode == "through"))
    return True

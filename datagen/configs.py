"""Synthetic workload recipes: model shapes and (source, destination) parallel configurations.

Only shapes and degrees live here, no layout or routing arithmetic.  Both the CPU oracle
and the HIP library take these dictionaries as input.

Field meaning
-------------
model:    family 0 = GPT (LayerNorm + bias, MHA), 1 = GQA + SwiGLU dense, 2 = GQA + MoE.
parallel: tp, pp, dp, ep degrees.  World size is tp*pp*dp*ep.  ``dp`` is the data-parallel
          degree of the expert group; dense tensors are replicated over dp*ep ranks.
          zero = 1 shards the fp32 kinds over the data-parallel group by flat offset.
          qkv_layout 0 = interleaved per kv group, 1 = [all Q | all K | all V] blocks.
          expert_layout 0 = row-major, 1 = transposed storage.
          flat_order 0 = ascending tensor id in the flat buffer, 1 = descending.
          ep_placement 0 = EP and expert-DP form a grid beside TP (world = tp*pp*dp*ep);
          1 = EP is carved out of the tp*dp ranks of a pipeline stage (world = tp*pp*dp, experts
          not TP-sharded, expert data-parallel degree tp*dp/ep), the form of the MoE tuples
          (TP, PP, DP, EP) in the paper's hybrid reconfiguration table.
"""

FAMILY_GPT = 0
FAMILY_GQA = 1
FAMILY_MOE = 2


def model(family, layers, hidden, q_heads, kv_heads, head_dim, ffn, vocab, experts=0, expert_ffn=0):
    return dict(family=family, layers=layers, hidden=hidden, q_heads=q_heads, kv_heads=kv_heads,
                head_dim=head_dim, ffn=ffn, vocab=vocab, experts=experts, expert_ffn=expert_ffn)


def parallel(tp=1, pp=1, dp=1, ep=1, zero=1, gpus_per_node=8, qkv_layout=0, expert_layout=0,
             flat_order=0, ep_placement=0):
    return dict(tp=tp, pp=pp, dp=dp, ep=ep, zero=zero, gpus_per_node=gpus_per_node,
                qkv_layout=qkv_layout, expert_layout=expert_layout, flat_order=flat_order,
                ep_placement=ep_placement)


def world(p):
    if p.get("ep_placement", 0) == 1:
        return p["tp"] * p["pp"] * p["dp"]
    return p["tp"] * p["pp"] * p["dp"] * p["ep"]


SEED_BASE = 0x5EED0000

# The five benchmark workloads.  "rank" is the rank whose share is materialised when the
# whole job does not fit one GPU (None = every virtual rank is resident).
WORKLOADS = {
    "toy": dict(
        index=1,
        model=model(FAMILY_GPT, 2, 256, 4, 4, 64, 1024, 1024),
        src=parallel(tp=2, dp=2, zero=1),
        dst=parallel(tp=1, dp=4, zero=0),
        rank=None,
    ),
    "gpt1p3b": dict(
        index=2,
        model=model(FAMILY_GPT, 24, 2048, 16, 16, 128, 8192, 50304),
        src=parallel(tp=4, pp=2, dp=4, zero=1),
        dst=parallel(tp=2, pp=4, dp=4, zero=1),
        rank=None,
    ),
    "gqa8b": dict(
        index=3,
        model=model(FAMILY_GQA, 32, 4096, 32, 8, 128, 14336, 128256),
        src=parallel(tp=8, dp=2, zero=1),
        dst=parallel(tp=4, pp=2, dp=2, zero=1),
        rank=5,
    ),
    "gqa70b": dict(
        index=4,
        model=model(FAMILY_GQA, 80, 8192, 64, 8, 128, 28672, 128256),
        src=parallel(tp=8, pp=8, dp=2, zero=1),
        dst=parallel(tp=8, pp=4, dp=4, zero=1),
        rank=11,
    ),
    "moe235b": dict(
        index=5,
        model=model(FAMILY_MOE, 94, 4096, 64, 4, 128, 0, 151936, experts=128, expert_ffn=1536),
        src=parallel(tp=1, pp=8, dp=2, ep=8, zero=1),
        dst=parallel(tp=1, pp=4, dp=2, ep=16, zero=1),
        rank=37,
    ),
}


# Transitions of the paper's evaluation on the published model shapes: the world-size-changing
# dense rows of its hybrid reconfiguration table, the pair of its ablation (tuples there are
# (TP, PP, DP)) and the table's two MoE pairs.  ZeRO-1 on both sides.  Planned at model
# scale (routes, dry runs); no state of this size is materialised.
PAPER_TRANSITIONS = {
    "llama7b-8-to-16": dict(model=model(FAMILY_GQA, 32, 4096, 32, 32, 128, 11008, 32000),
                            src=parallel(tp=2, pp=2, dp=2), dst=parallel(tp=4, pp=4, dp=1)),
    "llama13b-16-to-32": dict(model=model(FAMILY_GQA, 40, 5120, 40, 40, 128, 13824, 32000),
                              src=parallel(tp=4, pp=4, dp=1), dst=parallel(tp=2, pp=8, dp=2)),
    # the pair of the paper's ablation of its communication optimizations (16 GPUs on both sides)
    "llama13b-ablation-pair": dict(model=model(FAMILY_GQA, 40, 5120, 40, 40, 128, 13824, 32000),
                                   src=parallel(tp=2, pp=8, dp=1), dst=parallel(tp=2, pp=2, dp=4)),
    "llama70b-64-to-128": dict(model=model(FAMILY_GQA, 80, 8192, 64, 8, 128, 28672, 32000),
                               src=parallel(tp=4, pp=8, dp=2), dst=parallel(tp=8, pp=16, dp=1)),
    # the MoE rows of the same table, tuples (TP, PP, DP, EP) with EP carved out of the TP x DP
    # ranks of a stage (world = TP * PP * DP: 32 and 128 GPUs), on the published Qwen3-MoE shapes.
    # The 235B model has 4 KV heads; its TP = 8 side would need replicated KV heads, which the
    # paper does not describe: the stand-in has 8 KV heads (every other size as published).
    "qwen30b-hybrid": dict(model=model(FAMILY_MOE, 48, 2048, 32, 4, 128, 0, 151936, experts=128, expert_ffn=768),
                           src=parallel(tp=4, pp=8, dp=1, ep=4, ep_placement=1),
                           dst=parallel(tp=2, pp=4, dp=4, ep=2, ep_placement=1)),
    "qwen235b-hybrid": dict(model=model(FAMILY_MOE, 94, 4096, 64, 8, 128, 0, 151936, experts=128, expert_ffn=1536),
                            src=parallel(tp=4, pp=8, dp=4, ep=16, ep_placement=1),
                            dst=parallel(tp=8, pp=16, dp=1, ep=8, ep_placement=1)),
}


# Variants of the benchmark workloads for the copy engine's unfavourable cases.
EXTRA_WORKLOADS = {
    # the 70B switch with odd sizes everywhere: rows of 8191, 3585 and 1016 elements, so that the
    # tensors of a flat buffer start at odd element offsets and the 16-byte phase of the source
    # differs from that of the destination for most runs
    "gqa70b-odd": dict(
        index=6,
        model=model(FAMILY_GQA, 80, 8191, 64, 8, 127, 28680, 128264),
        src=parallel(tp=8, pp=8, dp=2, zero=1),
        dst=parallel(tp=8, pp=4, dp=4, zero=1),
        rank=11,
    ),
}


def workload(name):
    """A benchmark workload, a variant of one, or one of the paper's transitions (those have no
    default rank)."""
    if name in WORKLOADS:
        return WORKLOADS[name]
    if name in EXTRA_WORKLOADS:
        return EXTRA_WORKLOADS[name]
    return dict(PAPER_TRANSITIONS[name], rank=None, index=16 + sorted(PAPER_TRANSITIONS).index(name))


def seed_of(name):
    return SEED_BASE + workload(name)["index"]


# Small shapes for brute-force tests: every axis is tiny but each sharding rule is exercised.
TINY_GPT = model(FAMILY_GPT, 4, 16, 4, 4, 4, 32, 48)
TINY_GQA = model(FAMILY_GQA, 4, 32, 8, 4, 4, 48, 64)
TINY_MOE = model(FAMILY_MOE, 4, 16, 8, 4, 4, 0, 32, experts=8, expert_ffn=8)
# Odd sizes: local strides and flat edges are not multiples of any vector width.
ODD_GPT = model(FAMILY_GPT, 3, 18, 6, 6, 3, 30, 42)
ODD_MOE = model(FAMILY_MOE, 5, 12, 6, 2, 6, 0, 20, experts=6, expert_ffn=10)

# Medium shapes: several 64-element blocks and ragged tails on every axis, still small enough for
# the per-element oracle to verify every element in seconds.
MID_MOE = model(FAMILY_MOE, 2, 136, 4, 2, 34, 0, 96, experts=4, expert_ffn=200)
MID_GPT = model(FAMILY_GPT, 2, 192, 6, 6, 32, 516, 300)

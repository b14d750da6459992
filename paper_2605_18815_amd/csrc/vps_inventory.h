// vps_inventory.h - host side: validate descriptors and expand a model description into the
// table of logical tensors of the VPS (DynaTrain Section 4.1: every tensor in complete,
// unsharded form with position and partitioning attributes).  This is argument handling; all
// layout arithmetic happens afterwards in kernels.
#pragma once

#include <string>
#include <vector>

#include "vps_core.h"

namespace vps {

struct Error {
    int code;
    std::string msg;
};

inline void check_descs(const vps_model_desc& m, const vps_parallel_desc& p)
{
    auto bad = [](int code, const std::string& s) { throw Error{ code, s }; };
    if (m.family < 0 || m.family > 2) bad(VPS_ERR_INVALID_ARG, "unknown model family");
    if (m.layers < 1 || m.hidden < 1 || m.q_heads < 1 || m.kv_heads < 1 || m.head_dim < 1 || m.vocab < 1)
        bad(VPS_ERR_INVALID_ARG, "model sizes must be positive");
    if (m.family != VPS_FAMILY_MOE && m.ffn < 1) bad(VPS_ERR_INVALID_ARG, "ffn must be positive");
    if (m.family == VPS_FAMILY_MOE && (m.experts < 1 || m.expert_ffn < 1))
        bad(VPS_ERR_INVALID_ARG, "MoE family needs experts and expert_ffn");
    if (p.tp < 1 || p.pp < 1 || p.dp < 1 || p.ep < 1 || p.gpus_per_node < 1)
        bad(VPS_ERR_INVALID_ARG, "parallel degrees must be positive");
    if (p.zero_stage != 0 && p.zero_stage != 1) bad(VPS_ERR_INVALID_ARG, "zero_stage must be 0 or 1");
    if ((p.qkv_layout | p.expert_layout | p.flat_order) & ~1) bad(VPS_ERR_INVALID_ARG, "layout flags must be 0 or 1");
    if ((int64_t)p.tp * p.pp * p.dp * p.ep > 32768) bad(VPS_ERR_INVALID_ARG, "world size above 32768");
    if (m.q_heads % m.kv_heads) bad(VPS_ERR_INDIVISIBLE, "q_heads is not a multiple of kv_heads");
    if (m.family == VPS_FAMILY_GPT && m.q_heads != m.kv_heads)
        bad(VPS_ERR_INVALID_ARG, "GPT family is multi-head: kv_heads must equal q_heads");
    if (m.family != VPS_FAMILY_MOE && p.ep != 1) bad(VPS_ERR_INVALID_ARG, "ep > 1 needs the MoE family");
    if (m.kv_heads % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide the kv groups");
    if (m.vocab % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide vocab");
    if (m.family != VPS_FAMILY_MOE && m.ffn % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide ffn");
    if (m.family == VPS_FAMILY_MOE && m.expert_ffn % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide expert_ffn");
    if (m.family == VPS_FAMILY_MOE && m.experts % p.ep) bad(VPS_ERR_INDIVISIBLE, "ep does not divide experts");
    if (p.pp > m.layers) bad(VPS_ERR_INDIVISIBLE, "pp exceeds the number of layers");
    // tensor ids take 24 bits of the planner's sort keys
    const int64_t per_layer = 12 + (m.family == VPS_FAMILY_MOE ? 2 * (int64_t)m.experts : 0);
    if ((int64_t)m.layers * per_layer + 4 >= ((int64_t)1 << 24)) bad(VPS_ERR_INVALID_ARG, "more than 2^24 logical tensors");
    if ((int64_t)m.q_heads * m.head_dim >= ((int64_t)1 << 31)) bad(VPS_ERR_INVALID_ARG, "q_heads * head_dim does not fit 31 bits");
}

inline ParConst make_par_const(const vps_model_desc& m, const vps_parallel_desc& p, int32_t nt)
{
    ParConst P;
    P.tp = p.tp; P.pp = p.pp; P.dp = p.dp; P.ep = p.ep; P.zero = p.zero_stage; P.gpn = p.gpus_per_node;
    P.qkv_layout = p.qkv_layout; P.expert_layout = p.expert_layout; P.flat_order = p.flat_order;
    P.ddp = p.dp * p.ep;
    P.world = p.tp * p.pp * P.ddp;
    P.layers = m.layers;
    P.experts = m.family == VPS_FAMILY_MOE ? m.experts : 1;
    P.q_per_g = m.q_heads / m.kv_heads;
    P.nt = nt;
    P.ncls = p.pp + p.pp * p.ep;
    return P;
}

// Column-parallel weights [out, in] are cut on `out`, row-parallel ones on `in`; norms,
// row-parallel biases, the router and q/k norms are replicated over TP.  Fused QKV is the 4-D
// tensor (kv group, slot, head_dim, hidden) whose last two slots per group are K and V; fused
// SwiGLU is (2, ffn, hidden).
inline void build_inventory(const vps_model_desc& m, std::vector<TensorRec>& out)
{
    out.clear();
    auto add = [&](int s0, int s1, int s2, int s3, int tp_axis, int group, int blk_axis, int perm,
                   int layer, int expert) {
        TensorRec t;
        t.shape[0] = s0; t.shape[1] = s1; t.shape[2] = s2; t.shape[3] = s3;
        t.tp_axis = (int8_t)tp_axis; t.group = (int8_t)group; t.blk_axis = (int8_t)blk_axis;
        t.perm = (int8_t)perm; t.layer = layer; t.expert = expert;
        out.push_back(t);
    };
    auto vec = [&](int n, int layer) { add(1, 1, 1, n, -1, 0, -1, PERM_NONE, layer, -1); };
    const int h = m.hidden, d = m.head_dim, g = m.kv_heads, slots = m.q_heads / m.kv_heads + 2;
    const int qd = m.q_heads * d, L = m.layers;
    add(1, 1, m.vocab, h, 2, 0, -1, PERM_NONE, -1, -1);
    for (int l = 0; l < L; ++l) {
        if (m.family == VPS_FAMILY_GPT) {
            vec(h, l); vec(h, l);
            add(g, slots, d, h, 0, 0, 1, PERM_NONE, l, -1);
            add(1, g, slots, d, 1, 0, 2, PERM_NONE, l, -1);
            add(1, 1, h, qd, 3, 0, -1, PERM_NONE, l, -1);
            vec(h, l); vec(h, l); vec(h, l);
            add(1, 1, m.ffn, h, 2, 0, -1, PERM_NONE, l, -1);
            add(1, 1, 1, m.ffn, 3, 0, -1, PERM_NONE, l, -1);
            add(1, 1, h, m.ffn, 3, 0, -1, PERM_NONE, l, -1);
            vec(h, l);
        } else {
            vec(h, l);
            add(g, slots, d, h, 0, 0, 1, PERM_NONE, l, -1);
            if (m.family == VPS_FAMILY_MOE) { vec(d, l); vec(d, l); }
            add(1, 1, h, qd, 3, 0, -1, PERM_NONE, l, -1);
            vec(h, l);
            if (m.family == VPS_FAMILY_GQA) {
                add(1, 2, m.ffn, h, 2, 0, -1, PERM_NONE, l, -1);
                add(1, 1, h, m.ffn, 3, 0, -1, PERM_NONE, l, -1);
            } else {
                add(1, 1, m.experts, h, -1, 0, -1, PERM_NONE, l, -1);
                for (int e = 0; e < m.experts; ++e) {
                    add(1, 2, m.expert_ffn, h, 2, 1, -1, PERM_GATE_UP, l, e);
                    add(1, 1, h, m.expert_ffn, 3, 1, -1, PERM_DOWN, l, e);
                }
            }
        }
    }
    vec(h, L);
    if (m.family == VPS_FAMILY_GPT) vec(h, L);
    add(1, 1, m.vocab, h, 2, 0, -1, PERM_NONE, L, -1);
}

}  // namespace vps

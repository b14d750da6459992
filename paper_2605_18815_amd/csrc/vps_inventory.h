// vps_inventory.h - validate descriptors (host) and expand a model description into the table of
// logical tensors of the VPS (DynaTrain Section 4.1: every tensor in complete, unsharded form
// with position and partitioning attributes): one kernel lane per tensor id.
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
    if (p.ep_placement != 0 && p.ep_placement != 1) bad(VPS_ERR_INVALID_ARG, "ep_placement must be 0 or 1");
    if ((int64_t)p.tp * p.pp * p.dp * (p.ep_placement ? 1 : p.ep) > 32768) bad(VPS_ERR_INVALID_ARG, "world size above 32768");
    if (p.ep_placement == 1 && ((int64_t)p.tp * p.dp) % p.ep) bad(VPS_ERR_INDIVISIBLE, "ep does not divide tp*dp");
    if (m.q_heads % m.kv_heads) bad(VPS_ERR_INDIVISIBLE, "q_heads is not a multiple of kv_heads");
    if (m.family == VPS_FAMILY_GPT && m.q_heads != m.kv_heads)
        bad(VPS_ERR_INVALID_ARG, "GPT family is multi-head: kv_heads must equal q_heads");
    if (m.family != VPS_FAMILY_MOE && p.ep != 1) bad(VPS_ERR_INVALID_ARG, "ep > 1 needs the MoE family");
    if (m.kv_heads % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide the kv groups");
    if (m.vocab % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide vocab");
    if (m.family != VPS_FAMILY_MOE && m.ffn % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide ffn");
    if (m.family == VPS_FAMILY_MOE && p.ep_placement == 0 && m.expert_ffn % p.tp) bad(VPS_ERR_INDIVISIBLE, "tp does not divide expert_ffn");
    if (m.family == VPS_FAMILY_MOE && m.experts % p.ep) bad(VPS_ERR_INDIVISIBLE, "ep does not divide experts");
    if (p.pp > m.layers) bad(VPS_ERR_INDIVISIBLE, "pp exceeds the number of layers");
    // tensor ids take 24 bits of the planner's sort keys
    const int64_t per_layer = 12 + (m.family == VPS_FAMILY_MOE ? 2 * (int64_t)m.experts : 0);
    if ((int64_t)m.layers * per_layer + 4 >= ((int64_t)1 << 24)) bad(VPS_ERR_INVALID_ARG, "more than 2^24 logical tensors");
    if ((int64_t)m.q_heads * m.head_dim >= ((int64_t)1 << 31)) bad(VPS_ERR_INVALID_ARG, "q_heads * head_dim does not fit 31 bits");
}

// The model description in the form the inventory lanes use.
struct ModelConst {
    int32_t family, layers, hidden, head_dim, kv_groups, slots, qd, ffn, vocab, experts, expert_ffn;
    int32_t per_layer;  // logical tensors per layer
    int32_t nt;         // logical tensors in all
};

inline ModelConst make_model_const(const vps_model_desc& m)
{
    ModelConst M;
    M.family = m.family; M.layers = m.layers; M.hidden = m.hidden; M.head_dim = m.head_dim;
    M.kv_groups = m.kv_heads; M.slots = m.q_heads / m.kv_heads + 2; M.qd = m.q_heads * m.head_dim;
    M.ffn = m.ffn; M.vocab = m.vocab;
    M.experts = m.family == VPS_FAMILY_MOE ? m.experts : 0;
    M.expert_ffn = m.expert_ffn;
    M.per_layer = m.family == VPS_FAMILY_GPT ? 12 : (m.family == VPS_FAMILY_GQA ? 6 : 7 + 2 * m.experts);
    M.nt = 1 + m.layers * M.per_layer + (m.family == VPS_FAMILY_GPT ? 3 : 2);
    return M;
}

inline ParConst make_par_const(const vps_model_desc& m, const vps_parallel_desc& p, int32_t nt)
{
    ParConst P;
    P.tp = p.tp; P.pp = p.pp; P.dp = p.dp; P.ep = p.ep; P.zero = p.zero_stage; P.gpn = p.gpus_per_node;
    P.qkv_layout = p.qkv_layout; P.expert_layout = p.expert_layout; P.flat_order = p.flat_order;
    if (p.ep_placement == 0) { P.ddp = p.dp * p.ep; P.etp = p.tp; P.edp = p.dp; }
    else { P.ddp = p.dp; P.etp = 1; P.edp = p.tp * p.dp / p.ep; }
    P.dmax = P.ddp > P.edp ? P.ddp : P.edp;
    P.world = p.tp * p.pp * P.ddp;
    P.layers = m.layers;
    P.experts = m.family == VPS_FAMILY_MOE ? m.experts : 1;
    P.q_per_g = m.q_heads / m.kv_heads;
    P.nt = nt;
    P.ncls = p.pp + p.pp * p.ep;
    P.per_layer = make_model_const(m).per_layer;
    P.expert_pl = m.family == VPS_FAMILY_MOE ? 2 * m.experts : 0;
    return P;
}

// Logical tensor `t` of the model.  Column-parallel weights [out, in] are cut on `out`,
// row-parallel ones on `in`; norms, row-parallel biases, the router and q/k norms are replicated
// over TP.  Fused QKV is the 4-D tensor (kv group, slot, head_dim, hidden) whose last two slots
// per group are K and V; fused SwiGLU is (2, ffn, hidden).
VPS_HD TensorRec inventory_rec(const ModelConst& M, int32_t t)
{
    TensorRec r;
    r.shape[0] = r.shape[1] = r.shape[2] = 1; r.shape[3] = M.hidden;
    r.tp_axis = -1; r.group = 0; r.blk_axis = -1; r.perm = PERM_NONE; r.layer = -1; r.expert = -1;
    auto mat = [&](int s0, int s1, int s2, int s3, int tp_axis) {
        r.shape[0] = s0; r.shape[1] = s1; r.shape[2] = s2; r.shape[3] = s3; r.tp_axis = (int8_t)tp_axis;
    };
    const int32_t h = M.hidden, d = M.head_dim, g = M.kv_groups;
    const int32_t body = M.layers * M.per_layer;
    if (t == 0) { mat(1, 1, M.vocab, h, 2); return r; }                 // word embedding
    if (t > body) {                                                     // final norm(s), output layer
        r.layer = M.layers;
        if (t == M.nt - 1) mat(1, 1, M.vocab, h, 2);
        return r;
    }
    r.layer = (t - 1) / M.per_layer;
    const int32_t k = (t - 1) % M.per_layer;
    if (M.family == VPS_FAMILY_GPT) {
        // ln1.w ln1.b qkv.w qkv.b proj.w proj.b ln2.w ln2.b fc1.w fc1.b fc2.w fc2.b
        if (k == 2) { mat(g, M.slots, d, h, 0); r.blk_axis = 1; }
        else if (k == 3) { mat(1, g, M.slots, d, 1); r.blk_axis = 2; }
        else if (k == 4) mat(1, 1, h, M.qd, 3);
        else if (k == 8) mat(1, 1, M.ffn, h, 2);
        else if (k == 9) mat(1, 1, 1, M.ffn, 3);
        else if (k == 10) mat(1, 1, h, M.ffn, 3);
        return r;
    }
    if (M.family == VPS_FAMILY_GQA) {
        // in_norm qkv.w o.w post_norm gate_up.w down.w
        if (k == 1) { mat(g, M.slots, d, h, 0); r.blk_axis = 1; }
        else if (k == 2) mat(1, 1, h, M.qd, 3);
        else if (k == 4) mat(1, 2, M.ffn, h, 2);
        else if (k == 5) mat(1, 1, h, M.ffn, 3);
        return r;
    }
    // in_norm qkv.w q_norm k_norm o.w post_norm router.w, then gate_up.w down.w per expert
    if (k == 1) { mat(g, M.slots, d, h, 0); r.blk_axis = 1; }
    else if (k == 2 || k == 3) r.shape[3] = d;
    else if (k == 4) mat(1, 1, h, M.qd, 3);
    else if (k == 6) mat(1, 1, M.experts, h, -1);
    else if (k >= 7) {
        r.group = 1;
        r.expert = (k - 7) / 2;
        if ((k - 7) % 2 == 0) { mat(1, 2, M.expert_ffn, h, 2); r.perm = PERM_GATE_UP; }
        else { mat(1, 1, h, M.expert_ffn, 3); r.perm = PERM_DOWN; }
    }
    return r;
}

// Elements of the largest logical tensor (width of the lo-corner sort keys): the embedding or a
// tensor of the first layer.
inline uint64_t model_numel_max(const ModelConst& M)
{
    uint64_t best = 1;
    const int32_t last = 1 + M.per_layer < M.nt ? 1 + M.per_layer : M.nt;
    for (int32_t t = 0; t < last; ++t) {
        const TensorRec r = inventory_rec(M, t);
        if (numel4(r.shape) > best) best = numel4(r.shape);
    }
    return best;
}

}  // namespace vps

// vps_core.h - per-item arithmetic of the mapper, the planner and the copy engine.
//
// Every function here handles one work item (one tensor shard, one piece pair, one copy
// slot) and is callable from a HIP kernel lane.  The same source also compiles as plain C++
// so that bounds and index logic can be exercised in a CPU build by the test-suite; the
// product library only ever runs it on the device.
//
// Paper references: the VPS and F_P (DynaTrain Section 4.1), region intersection and
// send/retain/receive classification (Section 4.2.1), inversion of ZeRO flat-buffer shards
// into VPS sub-regions (Section 4.2.2), per-peer contiguous buffers (Section 4.3).
#pragma once

#include <stdint.h>

#include "../../include/vps.h"

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define VPS_HD __host__ __device__ inline
#else
#define VPS_HD inline
#endif

// unroll hint for loops whose loads are independent (n iterations' loads in flight together)
#define VPS_PRAGMA(x) _Pragma(#x)
#if defined(__clang__)
#define VPS_UNROLL(n) VPS_PRAGMA(unroll n)
#else
#define VPS_UNROLL(n) VPS_PRAGMA(GCC unroll n)
#endif

namespace vps {

enum { PERM_NONE = 0, PERM_GATE_UP = 1, PERM_DOWN = 2 };

// One logical tensor of the VPS: complete unsharded shape plus its position attributes
// (layer, expert, group) and partitioning attributes (TP axis, fused-QKV slot axis, which
// transposed storage applies).  Section 4.1.
struct TensorRec {
    int32_t shape[4];
    int8_t tp_axis;   // -1: replicated over TP
    int8_t group;     // 0 dense, 1 expert
    int8_t blk_axis;  // axis holding the Q/K/V slot index of a fused QKV tensor, or -1
    int8_t perm;      // PERM_*
    int32_t layer;    // -1 before the first layer, `layers` after the last
    int32_t expert;   // -1 or expert id
};

// Constants of one parallel configuration, passed to kernels by value.
struct ParConst {
    int32_t tp, pp, dp, ep, zero, gpn, qkv_layout, expert_layout, flat_order;
    int32_t ddp;      // dense data-parallel degree
    int32_t etp, edp; // tensor- and data-parallel degree of the expert group (etp*ep*edp = tp*ddp)
    int32_t dmax;     // max(ddp, edp): data-parallel extent of the mapper's item grid
    int32_t world;    // tp*pp*ddp
    int32_t layers, experts, q_per_g;
    int32_t nt;       // logical tensors
    int32_t ncls;     // flat-buffer classes: pp dense + pp*ep expert
    int32_t per_layer; // logical tensors per layer (ids 1 + l*per_layer .. of layer l)
    int32_t expert_pl; // of which the last expert_pl belong to experts (group 1); 0 without experts
};

// Where a tensor's local shard sits in the flat buffer of the ranks that hold it.
struct TensorLayout {
    uint64_t start;      // offset in the unsharded flat buffer
    uint64_t shard_len;  // elements of one local shard
    int32_t cls;         // flat-buffer class: dense -> pp, expert -> PP + pp*EP + ep
    int32_t stage;       // pipeline stage that holds the tensor
};

struct ClassRec {
    uint64_t len;     // unpadded flat length
    uint64_t padded;  // rounded up to 8*D
    uint64_t per;     // padded / D: elements of one data-parallel rank's range
};

struct RankCoord {
    int32_t tp, ddp, pp, ep, edp, etp;
};

// 64-bit division, out of line on the device.  The GPU divides integers in software, and a
// 64-bit division is about a kilobyte of instructions wherever it is expanded; the planner needs
// one only for tensors or item grids above 2^32, next to a 32-bit form that nearly always runs.
// Its kernels run once per plan, from a cold instruction cache: what they do not have to fetch
// is the time they save.
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __attribute__((noinline)) uint64_t udiv64(uint64_t a, uint64_t b) { return a / b; }
#else
inline uint64_t udiv64(uint64_t a, uint64_t b) { return a / b; }
#endif
template <class U> VPS_HD U quot(U a, U b) { return a / b; }
template <> VPS_HD uint64_t quot<uint64_t>(uint64_t a, uint64_t b) { return udiv64(a, b); }

// Dense tensors see a rank as tp + TP*(ddp + DDP*pp).  The expert group sees the rank's position
// inside its pipeline stage as etp + ETP*(ep + EP*edp): with EP and expert-DP as a grid beside TP
// (ETP = TP, EDP = DP, DDP = EP*DP) or with EP carved out of the TP x DP ranks (ETP = 1,
// EDP = TP*DP/EP, DDP = DP).
VPS_HD RankCoord decode_rank(const ParConst& P, int32_t r)
{
    RankCoord c;
    c.tp = r % P.tp;
    const int32_t q = r / P.tp;
    c.ddp = q % P.ddp;
    c.pp = q / P.ddp;
    const int32_t s = r % (P.tp * P.ddp);
    c.etp = s % P.etp;
    c.ep = (s / P.etp) % P.ep;
    c.edp = s / (P.etp * P.ep);
    return c;
}

// Rank of group `group` (0 dense, 1 expert) with tensor-parallel index t, data-parallel index d
// of that group, pipeline stage pp and (expert group only) expert-parallel index ep.
VPS_HD int32_t encode_rank(const ParConst& P, int32_t group, int32_t t, int32_t d, int32_t pp, int32_t ep)
{
    return group ? t + P.etp * (ep + P.ep * (d + P.edp * pp)) : t + P.tp * (d + P.ddp * pp);
}

VPS_HD int32_t group_tp(const ParConst& P, int32_t group) { return group ? P.etp : P.tp; }
VPS_HD int32_t group_dp(const ParConst& P, int32_t group) { return group ? P.edp : P.ddp; }

// Pipeline stage of a layer when stage p owns layers [floor(p*L/PP), floor((p+1)*L/PP)):
// the largest p with p*L/PP < layer+1.  The embedding (-1) is on the first stage, everything
// after the last layer on the last one.
VPS_HD int32_t stage_of_layer(const ParConst& P, int32_t layer)
{
    if (layer < 0) return 0;
    if (layer >= P.layers) return P.pp - 1;
    const int64_t num = ((int64_t)layer + 1) * P.pp + P.layers - 1;
    // (in 32 bits when it fits: the GPU divides in software, the 64-bit form is several times the work)
    if (num <= 0x7fffffffll) return (int32_t)((uint32_t)num / (uint32_t)P.layers) - 1;
    return (int32_t)udiv64((uint64_t)num, (uint64_t)P.layers) - 1;
}

// The tensor ids [lo, hi) that live on pipeline stage p: its layers, the embedding on the first
// stage, everything after the last layer on the last one (ids ascend in forward order).
VPS_HD void stage_tensor_range(const ParConst& P, int32_t p, int32_t& lo, int32_t& hi)
{
    const int32_t l0 = (int32_t)((int64_t)p * P.layers / P.pp), l1 = (int32_t)(((int64_t)p + 1) * P.layers / P.pp);
    lo = p == 0 ? 0 : 1 + l0 * P.per_layer;
    hi = p == P.pp - 1 ? P.nt : 1 + l1 * P.per_layer;
}

VPS_HD int32_t class_of_tensor(const ParConst& P, const TensorRec& x)
{
    const int32_t pp = stage_of_layer(P, x.layer);
    if (x.group == 0) return pp;
    return P.pp + pp * P.ep + x.expert / (P.experts / P.ep);
}

// Length of a flat-buffer class and its size padded to 8 elements per data-parallel rank.
VPS_HD ClassRec make_class_rec(const ParConst& P, int32_t cls, uint64_t len)
{
    ClassRec r;
    r.len = len;
    const uint64_t quantum = 8ull * (uint64_t)(cls < P.pp ? P.ddp : P.edp);
    r.padded = udiv64(len + quantum - 1, quantum) * quantum;
    r.per = udiv64(r.padded, (uint64_t)(cls < P.pp ? P.ddp : P.edp));
    return r;
}

VPS_HD uint64_t numel4(const int32_t* s)
{
    return (uint64_t)s[0] * (uint64_t)s[1] * (uint64_t)s[2] * (uint64_t)s[3];
}

VPS_HD uint64_t shard_elems(const ParConst& P, const TensorRec& x)
{
    const uint64_t n = numel4(x.shape);
    if (x.tp_axis < 0) return n;
    const uint32_t tp = (uint32_t)group_tp(P, x.group);
    if (n <= 0xffffffffull) return (uint32_t)n / tp;   // (see stage_of_layer)
    return udiv64(n, tp);
}

// ------------------------------------------------------------------------------------------
// Mapper: one item per (tensor, kind, tp index, data-parallel index).
// ------------------------------------------------------------------------------------------

struct MapCtx {
    ParConst P;
    const TensorRec* T;
    const TensorLayout* TL;
    const ClassRec* C;
    int32_t rank_filter;  // -1: all ranks
};

VPS_HD int64_t map_num_items(const ParConst& P) { return (int64_t)P.nt * 4 * P.tp * P.dmax; }

VPS_HD int64_t map_group_item(const ParConst& P, int32_t tensor, int32_t kind)
{
    return ((int64_t)tensor * 4 + kind) * P.tp * P.dmax;
}

// Cut the linear range [v0, v1) of a row-major array with dimensions n[0..3] into the
// canonical minimal set of boxes (at most 7): climb to coarser axes while the position is
// aligned and the unit still fits, descend again near the end.  Calls emit(start, axis, count)
// for each box: it begins at linear position `start`, spans `count` units of `axis` and is
// full on all finer axes.
// (Entry q of a four-entry table by selects: an array indexed at run time would be kept in
// scratch memory, and the planner's kernels are chains of dependent accesses.)
template <class V>
VPS_HD V pick4(int q, V a0, V a1, V a2, V a3) { return q == 0 ? a0 : (q == 1 ? a1 : (q == 2 ? a2 : a3)); }

template <class U, class Emit>
VPS_HD int split_linear_range_t(const int64_t* n, U v0, U v1, Emit emit)
{
    const U n0 = (U)n[0], n1 = (U)n[1], n2 = (U)n[2], n3 = (U)n[3];
    const U st3 = 1, st2 = n3, st1 = st2 * n2, st0 = st1 * n1;
    int count = 0;
    U cur = v0;
    while (cur < v1) {
        int q = 3;   // the coarsest axis on whose unit `cur` is aligned and whose unit still fits
        auto multiple_of = [](U a, U b) { return a - quot(a, b) * b == 0; };
        if (v1 - cur >= st2 && multiple_of(cur, st2)) {
            q = 2;
            if (v1 - cur >= st1 && multiple_of(cur, st1)) {
                q = 1;
                if (v1 - cur >= st0 && multiple_of(cur, st0)) q = 0;
            }
        }
        const U sq = pick4(q, st0, st1, st2, st3), nq = pick4(q, n0, n1, n2, n3);
        const U units = quot(cur, sq);
        const U cq = units - quot(units, nq) * nq;
        U cnt = nq - cq;
        const U fit = quot((U)(v1 - cur), sq);
        if (fit < cnt) cnt = fit;
        emit((uint64_t)cur, q, (uint64_t)cnt);
        cur += cnt * sq;
        ++count;
    }
    return count;
}

template <class Emit>
VPS_HD int split_linear_range(const int64_t* n, uint64_t v0, uint64_t v1, Emit emit)
{
    // the same in 32-bit arithmetic when the array has fewer than 2^32 elements (integer
    // division is several times cheaper there)
    const uint64_t vol = (uint64_t)n[0] * (uint64_t)n[1] * (uint64_t)n[2] * (uint64_t)n[3];
    if (vol <= 0xffffffffull && v1 <= 0xffffffffull) return split_linear_range_t<uint32_t>(n, (uint32_t)v0, (uint32_t)v1, emit);
    return split_linear_range_t<uint64_t>(n, v0, v1, emit);
}

// Pieces of one (tensor, kind, tp, dp-index) item: the part of the local shard that lies in
// the rank's flat range, as boxes in global coordinates with local offsets and strides.
// Calls f(piece) for each of them, in storage order; returns their number.
template <class F>
VPS_HD int map_item_each_piece(const MapCtx& c, int32_t t, int32_t kind, int32_t tp, int32_t didx, F f)
{
    const ParConst& P = c.P;
    const TensorRec x = c.T[t];
    const int32_t D = group_dp(P, x.group), TPg = group_tp(P, x.group);
    if (didx >= D || tp >= TPg) return 0;
    const TensorLayout tl = c.TL[t];
    const int32_t ep = x.group ? x.expert / (P.experts / P.ep) : 0;
    const int32_t rank = encode_rank(P, x.group, tp, didx, tl.stage, ep);
    if (c.rank_filter >= 0 && rank != c.rank_filter) return 0;

    const ClassRec cl = c.C[tl.cls];
    const bool sharded = P.zero == 1 && kind != 0;
    const uint64_t r0 = sharded ? cl.per * (uint64_t)didx : 0;
    const uint64_t r1 = sharded ? r0 + cl.per : cl.padded;
    const uint64_t f0 = tl.start > r0 ? tl.start : r0;
    const uint64_t fe = tl.start + tl.shard_len;
    const uint64_t f1 = fe < r1 ? fe : r1;
    if (f0 >= f1) return 0;
    const uint64_t u0 = f0 - tl.start, u1 = f1 - tl.start;

    // the shard's box in global coordinates
    int32_t slo[4], sext[4];
    VPS_UNROLL(4)
    for (int a = 0; a < 4; ++a) {
        slo[a] = 0; sext[a] = x.shape[a];
        if (a == x.tp_axis) { sext[a] = x.shape[a] / TPg; slo[a] = tp * sext[a]; }
    }
    // storage order of the axes, outermost first: 0,1,2,3; gate/up experts stored transposed
    // 0,3,1,2; down experts 0,1,3,2.  ord_q is the axis at position q, e_q the shard's extent there.
    const int mode = (P.expert_layout == 1 && x.perm == PERM_GATE_UP) ? 1 : ((P.expert_layout == 1 && x.perm == PERM_DOWN) ? 2 : 0);
    const int ord1 = mode == 1 ? 3 : 1, ord2 = mode == 1 ? 1 : (mode == 2 ? 3 : 2), ord3 = mode == 0 ? 3 : 2;
    const int32_t e0 = sext[0], e1 = mode == 1 ? sext[3] : sext[1];
    const int32_t e2 = mode == 1 ? sext[1] : (mode == 2 ? sext[3] : sext[2]), e3 = mode == 0 ? sext[3] : sext[2];
    // the entry of tensor axis a (a constant wherever this is called) in a table kept in storage order
    auto of_axis = [mode](int a, auto v0, auto v1, auto v2, auto v3) {
        if (a == 0) return v0;
        if (a == 1) return mode == 1 ? v2 : v1;
        if (a == 2) return mode == 0 ? v2 : v3;
        return mode == 1 ? v1 : (mode == 2 ? v2 : v3);
    };
    const bool blocked = x.blk_axis >= 0 && P.qkv_layout == 1;
    const int nblk = blocked ? 3 : 1;

    int npieces = 0;
    uint64_t bbase = 0;
    for (int b = 0; b < nblk; ++b) {
        int32_t bo = 0, bl = 0;
        if (blocked) {
            bo = b == 0 ? 0 : (b == 1 ? P.q_per_g : P.q_per_g + 1);
            bl = b == 0 ? P.q_per_g : 1;
        }
        int64_t n[4];
        n[0] = (blocked && 0 == x.blk_axis) ? bl : e0;
        n[1] = (blocked && ord1 == x.blk_axis) ? bl : e1;
        n[2] = (blocked && ord2 == x.blk_axis) ? bl : e2;
        n[3] = (blocked && ord3 == x.blk_axis) ? bl : e3;
        const uint64_t bvol = (uint64_t)n[0] * (uint64_t)n[1] * (uint64_t)n[2] * (uint64_t)n[3];
        const uint64_t lo = u0 > bbase ? u0 : bbase;
        const uint64_t hi = u1 < bbase + bvol ? u1 : bbase + bvol;
        if (lo < hi) {
            int64_t st[4];
            st[3] = 1; st[2] = n[3]; st[1] = n[3] * n[2]; st[0] = n[3] * n[2] * n[1];
            npieces += split_linear_range(n, lo - bbase, hi - bbase,
                [&](uint64_t start, int axis, uint64_t cnt) {
                    vps_piece p;
                    p.tensor = t; p.rank = rank; p.kind = kind; p.buf = x.group * 4 + kind;
                    // coordinates and extents of the piece along the storage positions
                    int32_t cq[4], xq[4];
                    uint64_t rem = start;
                    VPS_UNROLL(4)
                    for (int q = 0; q < 4; ++q) {
                        const int64_t c = bvol <= 0xffffffffull ? (int64_t)((uint32_t)rem / (uint32_t)st[q])
                                                                : (int64_t)udiv64(rem, (uint64_t)st[q]);
                        rem -= (uint64_t)c * (uint64_t)st[q];
                        cq[q] = (int32_t)c;
                        xq[q] = q < axis ? 1 : (q == axis ? (int32_t)cnt : (int32_t)n[q]);
                    }
                    VPS_UNROLL(4)
                    for (int a = 0; a < 4; ++a) {
                        p.lo[a] = slo[a] + ((blocked && a == x.blk_axis) ? bo : 0) + of_axis(a, cq[0], cq[1], cq[2], cq[3]);
                        p.ext[a] = of_axis(a, xq[0], xq[1], xq[2], xq[3]);
                        p.stride[a] = of_axis(a, st[0], st[1], st[2], st[3]);
                    }
                    p.off = (int64_t)(tl.start + bbase + start - r0);
                    f(p);
                });
        }
        bbase += bvol;
    }
    return npieces;
}

// Does data-parallel index didx hold any part of tensor t's shard for this kind?  (The flat
// range of the rank against the shard's place in the flat buffer: no division, no pieces.)
VPS_HD bool map_item_nonempty(const MapCtx& c, int32_t t, int32_t kind, int32_t didx)
{
    if (!(c.P.zero == 1 && kind != 0)) return true;
    const TensorLayout tl = c.TL[t];
    const ClassRec cl = c.C[tl.cls];
    const uint64_t r0 = cl.per * (uint64_t)didx, r1 = r0 + cl.per;
    return tl.start < r1 && r0 < tl.start + tl.shard_len;
}

// a / b and the remainder for a >= 0, b > 0: in 32 bits when a fits (the GPU divides integers in
// software, and the 64-bit form is several times the work of the 32-bit one).
VPS_HD int64_t div_small(int64_t a, int32_t b, int32_t& rem)
{
    if ((uint64_t)a <= 0xffffffffull) {
        const uint32_t q = (uint32_t)a / (uint32_t)b;
        rem = (int32_t)((uint32_t)a - q * (uint32_t)b);
        return (int64_t)q;
    }
    const int64_t q = (int64_t)udiv64((uint64_t)a, (uint64_t)b);
    rem = (int32_t)(a - q * b);
    return q;
}

VPS_HD void map_decode_item(const ParConst& P, int64_t item, int32_t& t, int32_t& kind, int32_t& tp, int32_t& didx)
{
    int64_t r = div_small(item, P.dmax, didx);
    r = div_small(r, P.tp, tp);
    kind = (int32_t)(r & 3);
    t = (int32_t)(r >> 2);
}

// The pieces of mapper item `item`; writes them when out != nullptr.  Returns their number.
VPS_HD int map_item_pieces(const MapCtx& c, int64_t item, vps_piece* out)
{
    int32_t t, kind, tp, didx;
    map_decode_item(c.P, item, t, kind, tp, didx);
    int k = 0;
    return map_item_each_piece(c, t, kind, tp, didx, [&](const vps_piece& p) { if (out) out[k++] = p; });
}

// ------------------------------------------------------------------------------------------
// Planner: one item per (destination mapper item, distinct piece of source data).
// ------------------------------------------------------------------------------------------

VPS_HD int32_t floor_div(int32_t a, int32_t b) { return a / b - ((a % b != 0) && ((a < 0) != (b < 0)) ? 1 : 0); }

// The source rank selected for destination rank j among the ranks that hold the same data as
// source rank i (i's TP replicas when the tensor is TP-replicated, i's data-parallel replicas
// when the kind is not ZeRO-sharded).  Rule: j itself if it is among them; else those on j's
// node if any, else all; in ascending rank order take index (data-parallel index of j under
// the destination configuration) modulo count.  Section 4.3 asks for a proximity-based choice;
// the tie-break is a convention of this library.
//
// Evaluated in closed form: the candidates form a grid (tp range x data-parallel range) whose
// ranks are, for every data-parallel index, one run of consecutive integers; a node is an
// interval of ranks, so only the few runs that can touch the node are looked at.
//
// Source rank i is given by its coordinates in the tensor's group (tensor-parallel index ti,
// data-parallel index di, stage, expert-parallel index): the callers have them, and a rank number
// would only be taken apart again.  ja / jb: j's coordinates under A and B when the caller holds
// them (the planned rank of a single-rank plan), else nullptr.
VPS_HD int32_t select_source_rank(const ParConst& A, const ParConst& B, const TensorRec& x, int32_t kind,
                                  int32_t ti, int32_t di, int32_t ppi, int32_t epi, int32_t j,
                                  const RankCoord* ja = nullptr, const RankCoord* jb = nullptr)
{
    RankCoord ci;
    ci.pp = ppi; ci.ep = epi;
    const bool sharded = A.zero == 1 && kind != 0;
    const int32_t D = group_dp(A, x.group), T = group_tp(A, x.group);
    const int32_t t0 = x.tp_axis < 0 ? 0 : ti, t1 = x.tp_axis < 0 ? T : ti + 1;
    const int32_t d0 = sharded ? di : 0, d1 = sharded ? di + 1 : D;
    // (1) the destination rank itself, if it is one of the candidates
    if (j < A.world) {
        const RankCoord cj = ja ? *ja : decode_rank(A, j);
        const int32_t dj = x.group ? cj.edp : cj.ddp, tj = x.group ? cj.etp : cj.tp;
        if (cj.pp == ci.pp && tj >= t0 && tj < t1 && dj >= d0 && dj < d1 && (!x.group || cj.ep == ci.ep))
            return j;
    }
    const RankCoord cb = jb ? *jb : decode_rank(B, j);
    const int32_t dpj = x.group ? cb.edp : cb.ddp;
    const int32_t nt = t1 - t0;
    // (2) candidates on j's node.  Row q holds the ranks T*q + t: q = d + DDP*pp for dense
    // tensors, q = ep + EP*(d + EDP*pp) for experts.  (Ranks are below 2^15, rows and counts too:
    // 32-bit arithmetic throughout.)
    const int32_t n0 = (j / A.gpn) * A.gpn, n1 = n0 + A.gpn;
    const int32_t step = x.group ? A.ep : 1;                       // rows of consecutive candidates
    const int32_t qfirst = x.group ? ci.ep + A.ep * (d0 + A.edp * ci.pp) : d0 + A.ddp * ci.pp;
    const int32_t qlast = qfirst + step * (d1 - d0 - 1);
    int32_t qlo = floor_div(n0 - t1, T) + 1, qhi = floor_div(n1 - t0 - 1, T);
    if (qlo < qfirst) qlo = qfirst;
    if (qhi > qlast) qhi = qlast;
    // align qlo up to a candidate row
    if (qlo > qfirst && step > 1) qlo = qfirst + (qlo - qfirst + step - 1) / step * step;
    int32_t n_node = 0;
    for (int32_t q = qlo; q <= qhi; q += step) {
        const int32_t lo = T * q + t0 > n0 ? T * q + t0 : n0;
        const int32_t hi = T * q + t1 < n1 ? T * q + t1 : n1;
        if (hi > lo) n_node += hi - lo;
    }
    if (n_node > 0) {
        int32_t want = dpj % n_node;
        for (int32_t q = qlo; q <= qhi; q += step) {
            const int32_t lo = T * q + t0 > n0 ? T * q + t0 : n0;
            const int32_t hi = T * q + t1 < n1 ? T * q + t1 : n1;
            if (hi <= lo) continue;
            if (want < hi - lo) return lo + want;
            want -= hi - lo;
        }
        return -1;
    }
    // (3) no candidate on the node: index into all of them, ascending
    const int32_t want = dpj % (nt * (d1 - d0));
    const int32_t q = qfirst + step * (want / nt);
    return T * q + t0 + want % nt;
}

struct PlanCtx {
    ParConst A, B;
    MapCtx ma, mb;             // the two configurations' layout tables (rank_filter = -1)
    int32_t rank;              // planned rank or -1
    // single-rank plans: the tensor ids the rank can hold as a destination / as a source
    int32_t recv_lo, recv_n, send_lo, send_n;
    // all-ranks plans: bits of the (destination tp, dp index) field and of the slot field of a lane
    // index (both padded to powers of two, so that a lane finds its item with shifts)
    int32_t item_bits, slot_bits;
    // single-rank plans: the planned rank's coordinates under the two configurations (the same
    // for every lane, so they are decoded once, on the host)
    RankCoord ra, rb;
};

// A destination item is paired with every distinct piece of source data of its (tensor, kind):
// one slot per source tp index if the tensor is TP-sharded, times one slot per source
// data-parallel index if the kind is ZeRO-sharded.  Replicas are not enumerated: the rank that
// serves a slot is computed from the selection rule.
VPS_HD int32_t plan_piece_slots(const ParConst& A, const TensorRec& x, int32_t kind)
{
    const int32_t nt = x.tp_axis < 0 ? 1 : group_tp(A, x.group);
    const int32_t nd = (A.zero == 1 && kind != 0) ? group_dp(A, x.group) : 1;
    return nt * nd;
}

VPS_HD int32_t plan_max_slots(const ParConst& A) { return A.tp * A.dmax; }

// Fill the lane geometry of a plan: tensor ranges from the planned rank's pipeline stages,
// field widths of an all-ranks lane index.
VPS_HD void plan_set_rank_ranges(PlanCtx& c)
{
    c.recv_lo = c.recv_n = c.send_lo = c.send_n = 0;
    c.item_bits = c.slot_bits = 0;
    while ((1 << c.item_bits) < c.B.tp * c.B.dmax) ++c.item_bits;
    while ((1 << c.slot_bits) < plan_max_slots(c.A)) ++c.slot_bits;
    c.ra = c.rb = RankCoord();
    if (c.rank < 0) return;
    int32_t lo, hi;
    if (c.rank < c.B.world) { c.rb = decode_rank(c.B, c.rank); stage_tensor_range(c.B, c.rb.pp, lo, hi); c.recv_lo = lo; c.recv_n = hi - lo; }
    if (c.rank < c.A.world) { c.ra = decode_rank(c.A, c.rank); stage_tensor_range(c.A, c.ra.pp, lo, hi); c.send_lo = lo; c.send_n = hi - lo; }
}


// Which lanes a planning launch enumerates.
//   PLAN_ALL   every (tensor, kind, destination tp, destination dp index, slot)
//   PLAN_RECV  destination items of the planned rank only: (tensor, kind, slot)
//   PLAN_SEND  the slot that the planned rank serves: (tensor, kind, destination tp, dp index);
//              boxes that stay on the rank are left to PLAN_RECV
//   PLAN_RANK  the lanes of PLAN_RECV followed by those of PLAN_SEND: everything of one rank
enum { PLAN_ALL = 0, PLAN_RECV = 1, PLAN_SEND = 2, PLAN_RANK = 3 };

VPS_HD int64_t plan_num_lanes(const PlanCtx& c, int mode)
{
    const int64_t tk = (int64_t)c.A.nt * 4;
    if (mode == PLAN_RECV) return (int64_t)c.recv_n * 4 * plan_max_slots(c.A);
    if (mode == PLAN_SEND) return (int64_t)c.send_n * 4 * c.B.tp * c.B.dmax;
    if (mode == PLAN_RANK) return plan_num_lanes(c, PLAN_RECV) + plan_num_lanes(c, PLAN_SEND);
    return tk << (c.item_bits + c.slot_bits);
}

// What a lane works on: one destination item and one slot of source data.
struct LaneItem {
    TensorRec x;
    int32_t t, kind, tpb, db, dst_rank, tp_rep, d_rep;
};

// The tensors of one group in ascending id order.  The inventory is the embedding, then per layer
// per_layer tensors of which the last expert_pl are the experts', then the closing tensors.
VPS_HD int32_t group_tensor_count(const ParConst& P, int group)
{
    const int32_t ne = P.layers * P.expert_pl;
    return group ? ne : P.nt - ne;
}
VPS_HD int32_t group_tensor_id(const ParConst& P, int group, int32_t i)
{
    const int32_t dpl = P.per_layer - P.expert_pl;
    if (group) { const int32_t layer = i / P.expert_pl; return 1 + layer * P.per_layer + dpl + (i - layer * P.expert_pl); }
    if (i == 0) return 0;
    const int32_t body = P.layers * dpl;
    if (i > body) return 1 + P.layers * P.per_layer + (i - 1 - body);
    const int32_t layer = (i - 1) / dpl;
    return 1 + layer * P.per_layer + (i - 1 - layer * dpl);
}

// PLAN_ALL with lane ranges per group: group g has count[g] tensors x 4 kinds x 2^item_bits[g]
// destination items x 2^slot_bits[g] source slots, the fields sized for the group's own degrees.
struct PlanGroupLanes {
    int64_t lanes[2];
    int32_t item_bits[2], slot_bits[2];
};
VPS_HD PlanGroupLanes plan_group_lanes(const PlanCtx& c)
{
    PlanGroupLanes g;
    for (int q = 0; q < 2; ++q) {
        g.item_bits[q] = g.slot_bits[q] = 0;
        while ((1 << g.item_bits[q]) < group_tp(c.B, q) * group_dp(c.B, q)) ++g.item_bits[q];
        while ((1 << g.slot_bits[q]) < group_tp(c.A, q) * group_dp(c.A, q)) ++g.slot_bits[q];
        g.lanes[q] = ((int64_t)group_tensor_count(c.A, q) * 4) << (g.item_bits[q] + g.slot_bits[q]);
    }
    return g;
}

VPS_HD bool plan_pair_check(const PlanCtx& c, int mode, const TensorRec& x, int32_t t, int32_t kind, int32_t tpb,
                            int32_t db, int32_t u, LaneItem& it);

// The item of a lane, or false when the lane has nothing to do: an index beyond the item grid, a
// tensor that the rank does not hold, a destination item and a slot that share no data.  Cheap:
// no division by a run-time 64-bit value, no pieces, no source selection.
VPS_HD bool plan_lane_decode(const PlanCtx& c, int mode, int64_t lane, LaneItem& it)
{
    const ParConst& A = c.A;
    const ParConst& B = c.B;
    int32_t t, kind, tpb, db, u;
    if (mode == PLAN_RANK) {
        const int64_t nrecv = plan_num_lanes(c, PLAN_RECV);
        mode = lane < nrecv ? PLAN_RECV : PLAN_SEND;
        if (mode == PLAN_SEND) lane -= nrecv;
    }
    if (mode == PLAN_ALL) {
        u = (int32_t)(lane & ((1 << c.slot_bits) - 1));
        const int32_t ib = (int32_t)((lane >> c.slot_bits) & ((1 << c.item_bits) - 1));
        const int32_t tk = (int32_t)(lane >> (c.slot_bits + c.item_bits));
        if (ib >= B.tp * B.dmax) return false;
        kind = tk & 3; t = tk >> 2;
        tpb = ib / B.dmax; db = ib - tpb * B.dmax;
    } else if (mode == PLAN_RECV) {
        const int64_t tk = div_small(lane, plan_max_slots(A), u);
        kind = (int32_t)(tk & 3);
        t = c.recv_lo + (int32_t)(tk >> 2);
        tpb = db = 0;
    } else {
        map_decode_item(B, lane, t, kind, tpb, db);
        t += c.send_lo;
        u = 0;
    }
    return plan_pair_check(c, mode, c.ma.T[t], t, kind, tpb, db, u, it);
}

// The second half of plan_lane_decode, from the tensor's record on (mode: PLAN_ALL, PLAN_RECV or
// PLAN_SEND).
VPS_HD bool plan_pair_check(const PlanCtx& c, int mode, const TensorRec& x, int32_t t, int32_t kind, int32_t tpb,
                            int32_t db, int32_t u, LaneItem& it)
{
    const ParConst& A = c.A;
    const ParConst& B = c.B;
    if (mode == PLAN_RECV) {
        if (c.rank >= B.world) return false;
        const RankCoord cr = c.rb;
        tpb = x.group ? cr.etp : cr.tp;
        db = x.group ? cr.edp : cr.ddp;
        // the rank holds the tensor only on its own stage (and expert block)
        if (c.mb.TL[t].stage != cr.pp || (x.group && x.expert / (B.experts / B.ep) != cr.ep)) return false;
    }
    if (tpb >= group_tp(B, x.group) || db >= group_dp(B, x.group)) return false;
    const int32_t nd = (A.zero == 1 && kind != 0) ? group_dp(A, x.group) : 1;
    if (mode == PLAN_SEND) {
        if (c.rank >= A.world) return false;
        const RankCoord cs = c.ra;
        if (c.ma.TL[t].stage != cs.pp || (x.group && x.expert / (A.experts / A.ep) != cs.ep)) return false;
        u = (x.tp_axis < 0 ? 0 : (x.group ? cs.etp : cs.tp)) * nd + (nd > 1 ? (x.group ? cs.edp : cs.ddp) : 0);
    }
    if (u >= plan_piece_slots(A, x, kind)) return false;
    const int32_t ppb = c.mb.TL[t].stage, epb = x.group ? x.expert / (B.experts / B.ep) : 0;
    const int32_t dst_rank = encode_rank(B, x.group, tpb, db, ppb, epb);
    if (mode == PLAN_SEND && dst_rank == c.rank) return false;
    const int32_t tp_rep = x.tp_axis < 0 ? 0 : u / nd, d_rep = u % nd;
    // cheap rejections first: most pairs of a destination item and a slot share no data
    if (!map_item_nonempty(c.mb, t, kind, db) || !map_item_nonempty(c.ma, t, kind, d_rep)) return false;
    if (x.tp_axis >= 0) {
        // the two shards must overlap on the tensor-parallel axis
        const int32_t ea = x.shape[x.tp_axis] / group_tp(A, x.group), eb = x.shape[x.tp_axis] / group_tp(B, x.group);
        if (tp_rep * ea >= (tpb + 1) * eb || tpb * eb >= (tp_rep + 1) * ea) return false;
    }
    it.x = x; it.t = t; it.kind = kind; it.tpb = tpb; it.db = db; it.dst_rank = dst_rank;
    it.tp_rep = tp_rep; it.d_rep = d_rep;
    return true;
}

// Lane gl_lane of the per-group ranges: false when it has nothing to do, else `lane` is its index
// in the PLAN_ALL numbering.
VPS_HD bool plan_group_lane_check(const PlanCtx& c, const PlanGroupLanes& g, int64_t gl_lane, int64_t& lane)
{
    const int q = gl_lane < g.lanes[0] ? 0 : 1;
    if (q) gl_lane -= g.lanes[0];
    const int32_t u = (int32_t)(gl_lane & ((1 << g.slot_bits[q]) - 1));
    const int32_t ib = (int32_t)((gl_lane >> g.slot_bits[q]) & ((1 << g.item_bits[q]) - 1));
    const int32_t tk = (int32_t)(gl_lane >> (g.slot_bits[q] + g.item_bits[q]));
    const int32_t kind = tk & 3, t = group_tensor_id(c.A, q, tk >> 2);
    const int32_t gd = group_dp(c.B, q), tpb = ib / gd, db = ib - tpb * gd;
    if (tpb >= group_tp(c.B, q)) return false;
    LaneItem it;
    if (!plan_pair_check(c, PLAN_ALL, c.ma.T[t], t, kind, tpb, db, u, it)) return false;
    lane = ((((int64_t)t * 4 + kind) << c.item_bits | (int64_t)(tpb * c.B.dmax + db)) << c.slot_bits) | u;
    return true;
}

// The routed boxes of one item: the pieces of the destination item intersected with the pieces
// of the source rank that serves the slot.  Calls f(box) for each non-empty intersection (lo
// corners ascending within one pair of pieces only); returns their number.  With parts > 1 only
// the destination pieces number part, part + parts, ... are taken: the item's work split over
// `parts` callers.
template <class F>
VPS_HD int plan_item_boxes(const PlanCtx& c, const LaneItem& it, F f, int part = 0, int parts = 1)
{
    const ParConst& A = c.A;
    const ParConst& B = c.B;
    const TensorRec& x = it.x;
    const int32_t t = it.t, kind = it.kind, tpb = it.tpb, db = it.db, dst_rank = it.dst_rank;
    const int32_t ppa = c.ma.TL[t].stage, epa = x.group ? x.expert / (A.experts / A.ep) : 0;
    const bool planned_dst = c.rank >= 0 && dst_rank == c.rank;   // (then its coordinates are at hand)
    const int32_t src = select_source_rank(A, B, x, kind, it.tp_rep, it.d_rep, ppa, epa, dst_rank,
                                           planned_dst && c.rank < A.world ? &c.ra : nullptr, planned_dst ? &c.rb : nullptr);
    if (c.rank >= 0 && dst_rank != c.rank && src != c.rank) return 0;
    const RankCoord cs = decode_rank(A, src);
    const int32_t tps = x.group ? cs.etp : cs.tp, ds = x.group ? cs.edp : cs.ddp;
    int n = 0, dpi = 0;
    map_item_each_piece(c.mb, t, kind, tpb, db, [&](const vps_piece& dp) {
        if (parts > 1 && (dpi++ & (parts - 1)) != part) return;
        map_item_each_piece(c.ma, t, kind, tps, ds, [&](const vps_piece& sp) {
            vps_box b;
            for (int a = 0; a < 4; ++a) {
                const int32_t l = sp.lo[a] > dp.lo[a] ? sp.lo[a] : dp.lo[a];
                const int32_t hs = sp.lo[a] + sp.ext[a], hd = dp.lo[a] + dp.ext[a];
                const int32_t h = hs < hd ? hs : hd;
                if (l >= h) return;
                b.lo[a] = l; b.ext[a] = h - l;
            }
            b.tensor = t; b.kind = kind;
            b.src_rank = sp.rank; b.dst_rank = dp.rank;
            b.src_buf = sp.buf; b.dst_buf = dp.buf;
            b.src_off = sp.off; b.dst_off = dp.off;
            for (int a = 0; a < 4; ++a) {
                b.src_stride[a] = sp.stride[a]; b.dst_stride[a] = dp.stride[a];
                b.src_off += (int64_t)(b.lo[a] - sp.lo[a]) * sp.stride[a];
                b.dst_off += (int64_t)(b.lo[a] - dp.lo[a]) * dp.stride[a];
            }
            b.send_pos = UINT64_MAX; b.recv_pos = UINT64_MAX;
            f(b);
            ++n;
        });
    });
    return n;
}

template <class F>
VPS_HD int plan_lane_boxes(const PlanCtx& c, int mode, int64_t lane, F f, int part = 0, int parts = 1)
{
    LaneItem it;
    if (!plan_lane_decode(c, mode, lane, it)) return 0;
    return plan_item_boxes(c, it, f, part, parts);
}

// A single-rank plan is a few hundred items of which a handful are cut into many pieces (the
// tensors that a data-parallel range begins or ends in), and the pieces of the source are made
// again for every piece of the destination: the item with the most pieces is the length of the
// whole launch.  So such a plan gives every item 2^PLAN_PART_BITS callers, one per residue of the
// destination piece's number.  All-ranks plans have items enough to fill the chip as they are.
constexpr int PLAN_PART_BITS = 3;
VPS_HD int plan_part_bits(int mode) { return mode == PLAN_ALL ? 0 : PLAN_PART_BITS; }

VPS_HD uint64_t box_volume(const vps_box& b)
{
    return (uint64_t)b.ext[0] * (uint64_t)b.ext[1] * (uint64_t)b.ext[2] * (uint64_t)b.ext[3];
}

VPS_HD uint32_t kind_bytes(int32_t kind) { return kind == 0 ? 2u : 4u; }

// Payload bytes of a box inside a peer buffer: every box starts on a 16-byte boundary.
VPS_HD uint64_t box_slot_bytes(const vps_box& b)
{
    return (box_volume(b) * kind_bytes(b.kind) + 15ull) & ~15ull;
}

// A box whose source and destination rank coincide is copied directly old-local -> new-local
// (T_retain of Section 4.2.1), unless the plan sends everything through the peer buffers: then
// a rank is its own peer and the box is packed and unpacked like any other.
VPS_HD bool box_retained(const vps_box& b, bool through_buffers)
{
    return !through_buffers && b.src_rank == b.dst_rank;
}

// Order inside a peer buffer: kinds 1,2,3 then 0; tensor id; lo corner in row-major order.
VPS_HD uint64_t box_major_key(const vps_box& b, bool by_dst)
{
    const uint64_t first = (uint64_t)(by_dst ? b.dst_rank : b.src_rank);
    const uint64_t second = (uint64_t)(by_dst ? b.src_rank : b.dst_rank);
    const uint64_t korder = (uint64_t)((b.kind + 3) & 3);
    return (((first << 16 | second) << 2 | korder) << 24) | (uint64_t)b.tensor;
}
enum { MAJOR_KEY_OWNER_SHIFT = 42 };  // key >> 42 = the rank that owns the buffer

// The same order in fewer bits, for the radix sort: rank fields of rank_bits, tensor ids of
// tensor_bits (2 * rank_bits + 2 + tensor_bits bits in all).
VPS_HD uint64_t compact_major_key(uint64_t key, int rank_bits, int tensor_bits)
{
    const uint64_t first = key >> MAJOR_KEY_OWNER_SHIFT, second = (key >> 26) & 0xffffull;
    const uint64_t korder = (key >> 24) & 3ull, tensor = key & 0xffffffull;
    return (((first << rank_bits | second) << 2 | korder) << tensor_bits) | tensor;
}

VPS_HD uint64_t box_minor_key(const vps_box& b, const TensorRec& x)
{
    return (((uint64_t)b.lo[0] * (uint64_t)x.shape[1] + (uint64_t)b.lo[1]) * (uint64_t)x.shape[2] +
            (uint64_t)b.lo[2]) * (uint64_t)x.shape[3] + (uint64_t)b.lo[3];
}

// What the ordering passes need of a box: its keys in the send and in the receive order and the
// bytes it takes in a peer buffer (a multiple of 16; the low bits say whether it counts in its
// source's send buffer and in its destination's receive buffer: it travels and that rank's
// buffers are on this GPU).
struct OrderRec {
    uint64_t key_s, key_r, klo, bytes_flags;
};
enum : uint64_t { ORD_SENDS = 1, ORD_RECEIVES = 2 };

VPS_HD OrderRec make_order_rec(const vps_box& b, const TensorRec& x, int32_t planned_rank, bool through_buffers)
{
    OrderRec r;
    r.key_s = box_major_key(b, false);
    r.key_r = box_major_key(b, true);
    r.klo = box_minor_key(b, x);
    r.bytes_flags = box_slot_bytes(b);
    if (!box_retained(b, through_buffers)) {
        if (planned_rank < 0 || b.src_rank == planned_rank) r.bytes_flags |= ORD_SENDS;
        if (planned_rank < 0 || b.dst_rank == planned_rank) r.bytes_flags |= ORD_RECEIVES;
    }
    return r;
}

// Place of a box in both orders by counting over all n boxes: its index is the number of boxes
// with a smaller key, its cumulative buffer position the bytes of the counted ones among them;
// base_* are the bytes that belong to ranks before the box's owner.  Keys are unique (boxes of
// one tensor and kind between two ranks are disjoint), so the indices are a permutation.
struct OrderPlace {
    uint32_t idx_s, idx_r;
    uint64_t gpos_s, gpos_r, base_s, base_r;
};

VPS_HD OrderPlace order_place_zero()
{
    OrderPlace o;
    o.idx_s = o.idx_r = 0;
    o.gpos_s = o.gpos_r = o.base_s = o.base_r = 0;
    return o;
}

VPS_HD uint64_t order_send_bytes(const OrderRec& r) { return (r.bytes_flags & ORD_SENDS) ? r.bytes_flags & ~(uint64_t)15 : 0; }
VPS_HD uint64_t order_recv_bytes(const OrderRec& r) { return (r.bytes_flags & ORD_RECEIVES) ? r.bytes_flags & ~(uint64_t)15 : 0; }

// One more box r for the place of box `me`; floor_* is the smallest key of me's owner rank.
VPS_HD void order_count_one(const OrderRec& r, const OrderRec& me, uint64_t floor_s, uint64_t floor_r, OrderPlace& o)
{
    const uint64_t sb = order_send_bytes(r), rb = order_recv_bytes(r);
    const bool less_s = r.key_s < me.key_s || (r.key_s == me.key_s && r.klo < me.klo);
    const bool less_r = r.key_r < me.key_r || (r.key_r == me.key_r && r.klo < me.klo);
    o.idx_s += less_s ? 1u : 0u;
    o.idx_r += less_r ? 1u : 0u;
    o.gpos_s += less_s ? sb : 0;
    o.gpos_r += less_r ? rb : 0;
    o.base_s += r.key_s < floor_s ? sb : 0;
    o.base_r += r.key_r < floor_r ? rb : 0;
}

VPS_HD uint64_t order_owner_floor(uint64_t key) { return key >> MAJOR_KEY_OWNER_SHIFT << MAJOR_KEY_OWNER_SHIFT; }

VPS_HD OrderPlace order_by_counting(const OrderRec* recs, uint32_t n, uint32_t k)
{
    const OrderRec me = recs[k];
    const uint64_t floor_s = order_owner_floor(me.key_s), floor_r = order_owner_floor(me.key_r);
    OrderPlace o = order_place_zero();
    for (uint32_t q = 0; q < n; ++q) order_count_one(recs[q], me, floor_s, floor_r, o);
    return o;
}

// Where the emission also counts its boxes per (source, destination) pair (all-ranks plans that
// are known to be large: the pair-by-pair ordering then starts from these counts instead of a
// pass of its own over the boxes).  count == nullptr: not counted.
struct PairCounts {
    uint64_t* count;   // [src * wb + dst] boxes
    uint64_t* bytes;   // [src * wb + dst] 16-byte-rounded bytes of the boxes that travel
    int32_t wb;
};

VPS_HD void be_atomic_add_runs(uint64_t* base, int64_t index, uint64_t v);

// One emitted box: its slot k of the raw table (boxes beyond the capacity are counted only).
VPS_HD void emit_box(const vps_box& b, const OrderRec& rec, uint64_t k, vps_box* raw, OrderRec* recs, uint64_t cap, const PairCounts& pc)
{
    if (k < cap) {
        raw[k] = b;
        recs[k] = rec;
    }
    if (pc.count) {
        const int64_t pr = (int64_t)b.src_rank * pc.wb + b.dst_rank;
        be_atomic_add_runs(pc.count, pr, 1);
        be_atomic_add_runs(pc.bytes, pr, (rec.bytes_flags & ORD_SENDS) ? (rec.bytes_flags & ~(uint64_t)15) : 0);
    }
}

// Words at the head of a plan's summary block.
enum { SUM_NBOXES = 0, SUM_NRETAIN = 1, SUM_NSEND = 2, SUM_NRECV = 3, SUM_NLISTED = 4, SUM_PAIR_WORK = 5, SUM_HEADER = 8 };

// All-ranks plans with many boxes are ordered pair by pair: both orders keep the boxes of one
// (source, destination) pair together and order them alike inside, by (kind order, tensor, lo
// corner).  What the passes need of a box, in the pair's bucket:
struct PairRec {
    uint64_t key;          // pair index << 26 | kind order << 24 | tensor
    uint64_t klo;          // lo corner, linearised
    uint64_t bytes_flags;  // as in OrderRec
    uint64_t box;          // index in the raw table
};
VPS_HD uint64_t pair_rec_key(const OrderRec& r, int64_t pair) { return ((uint64_t)pair << 26) | (r.key_s & 0x3ffffffull); }
VPS_HD bool pair_rec_less(const PairRec& a, const PairRec& b) { return a.key < b.key || (a.key == b.key && a.klo < b.klo); }
constexpr int64_t PAIR_BUCKET_MAX_PAIRS = (int64_t)1 << 20;     // source ranks x destination ranks
constexpr int PAIR_BUCKET_WORK_LOG2 = 32;                      // bound (log2) on the sum over the pairs of (boxes of the pair)^2

// Accumulate into a counter shared by all items of a step.
VPS_HD void be_atomic_add(uint64_t* p, uint64_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    atomicAdd((unsigned long long*)p, (unsigned long long)v);
#else
    *p += v;
#endif
}

// The same, returning the value before the addition.
VPS_HD uint64_t be_atomic_fetch_add(uint64_t* p, uint64_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint64_t)atomicAdd((unsigned long long*)p, (unsigned long long)v);
#else
    const uint64_t old = *p;
    *p += v;
    return old;
#endif
}

// base[index] += v where neighbouring items often share the index (boxes in send order share their
// (source, destination) pair): on the device the lanes of a wavefront first add up over runs of
// consecutive lanes with the same index (a segmented scan over the wavefront), and the last lane
// of every run does one atomic.  Same-address atomics are served one after the other, so this is
// what keeps a pass over 10^5 boxes from waiting on a few hundred hot addresses.
VPS_HD void be_atomic_add_runs(uint64_t* base, int64_t index, uint64_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const unsigned lane = threadIdx.x & 63u;
    const uint64_t active = __ballot(1);
    const int ilo = (int)(uint32_t)index, ihi = (int)(uint32_t)((uint64_t)index >> 32);
    const bool prev_same = __shfl_up(ilo, 1, 64) == ilo && __shfl_up(ihi, 1, 64) == ihi;
    const bool next_same = __shfl_down(ilo, 1, 64) == ilo && __shfl_down(ihi, 1, 64) == ihi;
    int head = (lane == 0 || !((active >> (lane - 1)) & 1ull) || !prev_same) ? 1 : 0;
    uint32_t slo = (uint32_t)v, shi = (uint32_t)(v >> 32);
    for (unsigned d = 1; d < 64; d <<= 1) {
        const uint32_t ulo = (uint32_t)__shfl_up((int)slo, d, 64), uhi = (uint32_t)__shfl_up((int)shi, d, 64);
        const int uhead = __shfl_up(head, d, 64);
        if (lane >= d && !head) {   // (then every lane down to lane - d is active and of this run)
            const uint64_t sum = (((uint64_t)shi << 32) | slo) + (((uint64_t)uhi << 32) | ulo);
            slo = (uint32_t)sum; shi = (uint32_t)(sum >> 32);
            head = uhead;
        }
    }
    const bool tail = lane == 63 || !((active >> (lane + 1)) & 1ull) || !next_same;
    if (tail) atomicAdd((unsigned long long*)(base + index), (unsigned long long)(((uint64_t)shi << 32) | slo));
#else
    base[index] += v;
#endif
}

// Count the lanes for which `pred` holds into a counter that every item of a step shares: on the
// device one atomic per wavefront (a ballot names the lanes) instead of one per lane.
VPS_HD void be_atomic_count(uint64_t* p, bool pred)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const uint64_t mask = __ballot(pred ? 1 : 0);
    if (mask && (threadIdx.x & 63u) == (unsigned)(__ffsll((unsigned long long)mask) - 1))
        atomicAdd((unsigned long long*)p, (unsigned long long)__popcll(mask));
#else
    if (pred) *p += 1;
#endif
}

VPS_HD void be_atomic_or(uint32_t* p, uint32_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    atomicOr(p, v);
#else
    *p |= v;
#endif
}

// ------------------------------------------------------------------------------------------
// Copy engine: strided box -> strided box, descriptor driven.
// ------------------------------------------------------------------------------------------

enum { OP_RETAIN = 0, OP_PACK = 1, OP_UNPACK = 2 };
enum { MODE_RUN = 0, MODE_ELEM = 1, MODE_XPOSE = 2 };
enum { XPOSE_T = 64 };  // edge of a transposed block, in elements

// Pointer table slots of a single-rank plan.  All-ranks plans use
// [src: rank*8+buf][dst: WA*8 + rank*8+buf][send: (WA+WB)*8 + rank][recv: (WA+WB)*8 + WA + rank].
enum { PT_SRC = 0, PT_DST = 8, PT_SEND = 16, PT_RECV = 17, PT_INLINE = 18 };

struct CopyDesc {
    uint64_t src_byte;    // byte offset of the first element in its buffer
    uint64_t dst_byte;
    int64_t sstr[4];      // element strides after axis collapse (outer -> inner)
    int64_t dstr[4];
    uint32_t ext[4];
    int32_t src_slot;     // pointer-table slot of the source buffer
    int32_t dst_slot;
    int32_t alt_src_slot; // unpack only: the sender's send buffer, for in-place exchange
    uint32_t es;          // element bytes
    uint64_t alt_src_byte;
    uint32_t mode;
    uint32_t rows_per_tile;  // RUN, short runs: runs per tile.  ELEM: elements per tile.
                             // XPOSE: super-block shape sa | sb << 16
    uint32_t vec_window;     // RUN: 16-byte destination vectors of a run that one tile covers.
                             // XPOSE: number of blocks along axis 3
    uint32_t chunks_per_row; // RUN, long runs: tiles per run (0 = short-run tiling).
                             // XPOSE: number of blocks along axis xa
    uint32_t ntiles;
    uint32_t xa;             // XPOSE: the collapsed axis (0..2) that is contiguous in the source.
                             // RUN, long runs: dst_byte modulo the cut alignment when the descriptor was made
};

struct PtrLayout {
    int32_t all_ranks;  // 0: single-rank table of PT_INLINE slots
    int32_t wa, wb;
};

VPS_HD int32_t slot_src(const PtrLayout& L, int32_t rank, int32_t buf)
{
    return L.all_ranks ? rank * 8 + buf : PT_SRC + buf;
}
VPS_HD int32_t slot_dst(const PtrLayout& L, int32_t rank, int32_t buf)
{
    return L.all_ranks ? L.wa * 8 + rank * 8 + buf : PT_DST + buf;
}
VPS_HD int32_t slot_send(const PtrLayout& L, int32_t rank)
{
    return L.all_ranks ? (L.wa + L.wb) * 8 + rank : PT_SEND;
}
VPS_HD int32_t slot_recv(const PtrLayout& L, int32_t rank)
{
    return L.all_ranks ? (L.wa + L.wb) * 8 + L.wa + rank : PT_RECV;
}
VPS_HD int32_t num_slots(const PtrLayout& L)
{
    return L.all_ranks ? (L.wa + L.wb) * 9 : PT_INLINE;
}

// A box that would need 2^31 tiles or more saturates the count; the planner then reports
// VPS_ERR_OOM instead of building a wrapped-around table.
VPS_HD uint32_t clamp_tiles(uint64_t n) { return n >= (1ull << 31) ? (1u << 31) : (uint32_t)n; }

// Super-block shape of a transposed box as sa | sb << 16 (see xpose_plane_order), 64 blocks per
// super-block.  Rows of a block are 64 elements long and lie `pitch` bytes apart.  On the side
// whose pitch is the rounder number (more trailing zero bits: a power-of-two row length) the rows
// of neighbouring blocks fall on the same memory channels, so the blocks that run together are
// spread more over the other side's axis (16 x 4 instead of 8 x 8).  Measured on the 235B share
// with transposed experts on either side: 1-3 % against square super-blocks.
VPS_HD uint32_t xpose_auto_shape(int64_t src_pitch_bytes, int64_t dst_pitch_bytes)
{
    int zs = 0, zd = 0;
    while (zs < 30 && !((src_pitch_bytes >> zs) & 1)) ++zs;
    while (zd < 30 && !((dst_pitch_bytes >> zd) & 1)) ++zd;
    if (zs > zd) return 4u | 16u << 16;
    if (zd > zs) return 16u | 4u << 16;
    return 8u | 8u << 16;
}

// Long runs are cut into tiles at destination offsets that are multiples of this many bytes
// (when the tile size is such a multiple): a memory line that two workgroups share is written
// in two parts, which costs a few per cent of the copy rate; with the cuts on line boundaries
// only the two ends of a run are left with partial lines.  Offsets are relative to the buffer;
// allocations of the HIP runtime start on such a boundary.
constexpr uint64_t RUN_CUT_ALIGN = 256;
VPS_HD uint64_t run_cut_align(uint64_t tile_vectors) { return (tile_vectors * 16) % RUN_CUT_ALIGN ? 16 : RUN_CUT_ALIGN; }

// Build the copy descriptor of one box for one operation.  resident(rank) tells whether the
// rank's buffers exist on this GPU (planned rank, or every rank for all-ranks plans); boxes
// whose operation does not apply get ntiles = 0.
VPS_HD void make_copy_desc(const vps_box& b, int op, const PtrLayout& L, int32_t planned_rank,
                           bool through_buffers, uint32_t tile_bytes, uint32_t xpose_shape, CopyDesc& d)
{
    const bool retained = box_retained(b, through_buffers);
    const bool src_res = planned_rank < 0 || b.src_rank == planned_rank;
    const bool dst_res = planned_rank < 0 || b.dst_rank == planned_rank;
    d = CopyDesc();
    d.alt_src_slot = -1;
    d.es = kind_bytes(b.kind);
    bool active;
    int64_t ss[4], ds[4];
    // row-major strides of the box itself: its layout inside a peer buffer
    int64_t bs[4];
    bs[3] = 1; bs[2] = b.ext[3]; bs[1] = (int64_t)b.ext[3] * b.ext[2];
    bs[0] = (int64_t)b.ext[3] * b.ext[2] * b.ext[1];
    if (op == OP_RETAIN) {
        active = retained && src_res;
        d.src_slot = slot_src(L, b.src_rank, b.src_buf);
        d.dst_slot = slot_dst(L, b.dst_rank, b.dst_buf);
        d.src_byte = (uint64_t)b.src_off * d.es;
        d.dst_byte = (uint64_t)b.dst_off * d.es;
        for (int a = 0; a < 4; ++a) { ss[a] = b.src_stride[a]; ds[a] = b.dst_stride[a]; }
    } else if (op == OP_PACK) {
        active = !retained && src_res;
        d.src_slot = slot_src(L, b.src_rank, b.src_buf);
        d.dst_slot = slot_send(L, b.src_rank);
        d.src_byte = (uint64_t)b.src_off * d.es;
        d.dst_byte = b.send_pos;
        for (int a = 0; a < 4; ++a) { ss[a] = b.src_stride[a]; ds[a] = bs[a]; }
    } else {
        active = !retained && dst_res;
        d.src_slot = slot_recv(L, b.dst_rank);
        // the sender's segment is on this GPU when every rank is, or when the sender is the
        // planned rank itself
        if (L.all_ranks || b.src_rank == b.dst_rank) d.alt_src_slot = slot_send(L, b.src_rank);
        d.dst_slot = slot_dst(L, b.dst_rank, b.dst_buf);
        d.src_byte = b.recv_pos;
        d.alt_src_byte = b.send_pos;
        d.dst_byte = (uint64_t)b.dst_off * d.es;
        for (int a = 0; a < 4; ++a) { ss[a] = bs[a]; ds[a] = b.dst_stride[a]; }
    }
    if (!active) { d.ntiles = 0; return; }

    // Collapse: drop unit axes, order by destination stride (largest first, equal strides in axis
    // order), merge axes that are contiguous on both sides.  Written so that every index is a
    // constant once the loops are unrolled: arrays indexed at run time live in scratch memory,
    // and the planner's kernels are chains of dependent accesses.
    struct Axis { int64_t e, s, d; int32_t i; bool unit; };
    Axis x[4];
    VPS_UNROLL(4)
    for (int a = 0; a < 4; ++a) { x[a].e = b.ext[a]; x[a].s = ss[a]; x[a].d = ds[a]; x[a].i = a; x[a].unit = b.ext[a] == 1; }
    auto in_order = [](Axis& p, Axis& q) {   // p stands before q: exchange them if q belongs first
        const bool q_first = !q.unit && (p.unit || q.d > p.d || (q.d == p.d && q.i < p.i));
        if (q_first) { const Axis t = p; p = q; q = t; }
    };
    in_order(x[0], x[1]); in_order(x[2], x[3]); in_order(x[0], x[2]); in_order(x[1], x[3]); in_order(x[1], x[2]);
    Axis o0, o1, o2, o3;   // the merged axes, the innermost in o3; unused outer ones have extent 1
    o0.e = o1.e = o2.e = o3.e = 1; o0.s = o1.s = o2.s = o3.s = 0; o0.d = o1.d = o2.d = o3.d = 0;
    int m = 0;
    VPS_UNROLL(4)
    for (int i = 0; i < 4; ++i) {
        if (x[i].unit) continue;
        // (extents stay below 2^31: a longer contiguous stretch is kept as rows of a 2-D box)
        if (m > 0 && o3.s == x[i].s * x[i].e && o3.d == x[i].d * x[i].e && o3.e * x[i].e < ((int64_t)1 << 31)) {
            o3.e *= x[i].e; o3.s = x[i].s; o3.d = x[i].d;
        } else {
            o0 = o1; o1 = o2; o2 = o3; o3 = x[i]; ++m;
        }
    }
    d.ext[0] = (uint32_t)o0.e; d.sstr[0] = o0.s; d.dstr[0] = o0.d;
    d.ext[1] = (uint32_t)o1.e; d.sstr[1] = o1.s; d.dstr[1] = o1.d;
    d.ext[2] = (uint32_t)o2.e; d.sstr[2] = o2.s; d.dstr[2] = o2.d;
    d.ext[3] = (uint32_t)o3.e; d.sstr[3] = o3.s; d.dstr[3] = o3.d;
    if (m == 0) { d.sstr[3] = 1; d.dstr[3] = 1; }

    const uint64_t vol = (uint64_t)d.ext[0] * d.ext[1] * d.ext[2] * d.ext[3];
    if (d.sstr[3] == 1 && d.dstr[3] == 1) {
        d.mode = MODE_RUN;
        const uint64_t run_bytes = (uint64_t)d.ext[3] * d.es;
        const uint64_t rows = udiv64(vol, d.ext[3]);
        if (rows >= (1ull << 31)) { d.ntiles = clamp_tiles(rows); return; }  // run index is 32-bit
        // 16-byte destination vectors a run can touch, counted from the 16-byte boundary at or
        // below its first byte: exact when every run of the box starts on such a boundary
        bool aligned = (d.dst_byte & 15) == 0;
        for (int a = 0; a < 3; ++a)
            if (d.ext[a] > 1 && ((d.dstr[a] * (int64_t)d.es) & 15)) aligned = false;
        const uint64_t nv_max = (run_bytes + (aligned ? 15 : 30)) / 16;
        const uint64_t vt = tile_bytes / 16;
        if (nv_max > vt) {
            // chunks are cut at multiples of the tile size counted from the RUN_CUT_ALIGN boundary
            // at or below the run's first destination byte (see make_tile): room for the bytes
            // between that boundary and the run, exact when every run starts at the same phase
            const uint64_t cut = run_cut_align(vt);
            bool same_phase = true;
            for (int a = 0; a < 3; ++a)
                if (d.ext[a] > 1 && ((uint64_t)(d.dstr[a] * (int64_t)d.es) & (cut - 1))) same_phase = false;
            const uint64_t pre = same_phase ? (d.dst_byte & (cut - 1)) : cut - d.es;
            d.xa = (uint32_t)(d.dst_byte & (cut - 1));   // kept with the descriptor: see make_tile
            d.chunks_per_row = (uint32_t)udiv64(pre + run_bytes + vt * 16 - 1, vt * 16);
            d.vec_window = (uint32_t)vt;
            d.rows_per_tile = 1;
            d.ntiles = clamp_tiles(rows * d.chunks_per_row);
        } else {
            // short runs: k consecutive runs along axis 2 per tile, never across a slab
            // (fixed coordinates on axes 0 and 1), so that run addresses are affine in a tile
            d.chunks_per_row = 0;
            d.vec_window = (uint32_t)nv_max;
            uint64_t k = udiv64(vt, nv_max);
            if (k < 1) k = 1;
            if (k > d.ext[2]) k = d.ext[2];
            d.rows_per_tile = (uint32_t)k;
            const uint64_t tps = udiv64(d.ext[2] + k - 1, k);
            d.ntiles = clamp_tiles((uint64_t)d.ext[0] * d.ext[1] * tps);
        }
    } else if (d.dstr[3] == 1 && ((d.sstr[2] == 1 && d.ext[2] > 1) || (d.sstr[1] == 1 && d.ext[1] > 1) ||
                                  (d.sstr[0] == 1 && d.ext[0] > 1))) {
        // The destination is contiguous along axis 3, the source along another axis: 2-D
        // transposes of XPOSE_T x XPOSE_T element blocks staged through LDS.
        d.mode = MODE_XPOSE;
        d.xa = (d.sstr[2] == 1 && d.ext[2] > 1) ? 2u : ((d.sstr[1] == 1 && d.ext[1] > 1) ? 1u : 0u);
        const uint32_t ext_xa = d.xa == 2u ? d.ext[2] : (d.xa == 1u ? d.ext[1] : d.ext[0]);   // (no run-time index, see above)
        const int64_t dstr_xa = d.xa == 2u ? d.dstr[2] : (d.xa == 1u ? d.dstr[1] : d.dstr[0]);
        const uint64_t na = (ext_xa + XPOSE_T - 1) / XPOSE_T, nb = (d.ext[3] + XPOSE_T - 1) / XPOSE_T;
        d.chunks_per_row = (uint32_t)na;
        d.vec_window = (uint32_t)nb;
        d.rows_per_tile = xpose_shape ? xpose_shape : xpose_auto_shape(d.sstr[3] * (int64_t)d.es, dstr_xa * (int64_t)d.es);
        d.ntiles = clamp_tiles(udiv64(udiv64(vol, ext_xa), d.ext[3]) * na * nb);
    } else {
        d.mode = MODE_ELEM;
        uint64_t per = tile_bytes / (4 * d.es);
        if (per < 256) per = 256;
        d.rows_per_tile = (uint32_t)per;
        d.ntiles = clamp_tiles(udiv64(vol + per - 1, per));
    }
}

struct PtrArgs {
    char* inl[PT_INLINE];  // single-rank plans: the 18 buffer pointers by value
    char* const* tbl;      // all-ranks plans: table in device memory (nullptr otherwise)
};

// One tile of the copy engine (48 bytes, read by the workgroup with scalar loads).
//   run tiles    a contiguous piece of one long run, or several short runs at a constant pitch
//   transposes   a block of up to XPOSE_T x XPOSE_T elements (TILE_XPOSE)
//                for both, everything the kernel needs is here: a workgroup does no index arithmetic
//   indirect     an element-wise tile: tile q of descriptor `desc` (TILE_INDIRECT)
struct TileRef {
    uint64_t src;      // slot << 44 | byte offset in the slot's buffer (first run / element (0,0))
    uint64_t dst;
    uint64_t alt_src;  // the sender's send buffer for in-place exchange (or TILE_NO_ALT)
                       // indirect: q << 32 | desc
    int64_t src_pitch; // several runs: bytes between consecutive runs
                       // transpose: bytes between consecutive b in the source
    int64_t dst_pitch; // transpose: bytes between consecutive a in the destination
    uint32_t nbytes;   // bytes of one run (piece).  transpose: ta | tb << 16
    uint32_t nruns_flags;  // bits 0..7 flags, bits 8..31 number of runs
};
enum : uint32_t { TILE_INDIRECT = 1u, TILE_XPOSE = 2u, TILE_ES2 = 4u };
#define VPS_TILE_NO_ALT (~0ull)

VPS_HD uint64_t tile_pack_addr(int32_t slot, uint64_t byte_off) { return ((uint64_t)slot << 44) | byte_off; }
VPS_HD int32_t tile_slot(uint64_t a) { return (int32_t)(a >> 44); }
VPS_HD uint64_t tile_offset(uint64_t a) { return a & ((1ull << 44) - 1); }

// How one run is moved by the caller responsible for the window [w0, w0 + nw) of its
// destination-aligned 16-byte vectors.  The run covers dst bytes [drow, drow + run_bytes) and
// the same number of src bytes from srow.  Vector w is dst [dvec + 16w, +16), src svec + 16w.
struct RunWindow {
    uint64_t svec, dvec;     // src / dst address of vector 0 (dvec is 16-byte aligned)
    uint32_t wbeg, wend;     // full vectors [wbeg, wend) to move with 16-byte accesses
    uint32_t head_bytes;     // partial first vector: bytes to move from srow to drow (0 = none)
    uint32_t tail_bytes;     // partial last vector: bytes to move at offset tail_off (0 = none)
    uint64_t tail_off;       // byte offset from svec / dvec
};

VPS_HD RunWindow run_window(uint64_t srow, uint64_t drow, uint64_t run_bytes, uint32_t w0, uint32_t nw)
{
    RunWindow g;
    const uint32_t head = (uint32_t)(drow & 15);        // bytes of vector 0 before the run
    const uint64_t span = (uint64_t)head + run_bytes;     // run end relative to vector 0
    const uint32_t wf = head ? 1u : 0u;                   // first full vector
    const uint32_t wl = (uint32_t)(span >> 4);            // one past the last full vector
    const uint32_t wend_win = w0 + nw;
    g.dvec = drow - head;
    g.svec = srow - head;
    g.wbeg = w0 > wf ? w0 : wf;
    g.wend = wend_win < wl ? wend_win : wl;
    if (g.wend < g.wbeg) g.wend = g.wbeg;
    g.head_bytes = (head && w0 == 0) ? (span < 16 ? (uint32_t)run_bytes : 16 - head) : 0;
    const uint32_t tailb = (uint32_t)(span & 15);
    // the last partial vector, unless it is the same vector as the head one
    const bool has_tail = tailb && !(wl == 0 && head) && wl >= w0 && wl < wend_win;
    g.tail_bytes = has_tail ? tailb : 0;
    g.tail_off = (uint64_t)wl * 16;
    return g;
}

// Byte offsets of the first element of run `row` relative to the descriptor bases.
VPS_HD void run_row_offsets(const CopyDesc& d, uint32_t row, uint64_t& so, uint64_t& to)
{
    if (d.ext[0] == 1 && d.ext[1] == 1) {   // the rows lie along one axis: no division
        so = (uint64_t)((int64_t)row * d.sstr[2] * (int64_t)d.es);
        to = (uint64_t)((int64_t)row * d.dstr[2] * (int64_t)d.es);
        return;
    }
    const uint32_t c2 = row % d.ext[2];
    const uint32_t r1 = row / d.ext[2];
    const uint32_t c1 = r1 % d.ext[1];
    const uint32_t c0 = r1 / d.ext[1];
    so = (uint64_t)(((int64_t)c0 * d.sstr[0] + (int64_t)c1 * d.sstr[1] + (int64_t)c2 * d.sstr[2]) * (int64_t)d.es);
    to = (uint64_t)(((int64_t)c0 * d.dstr[0] + (int64_t)c1 * d.dstr[1] + (int64_t)c2 * d.dstr[2]) * (int64_t)d.es);
}

// Order of the na x nb blocks of one plane: super-blocks of sa x sb blocks (sa along the source's
// contiguous axis, sb along the destination's), row-major over the super-blocks and inside
// them.  Blocks that are launched together then touch neighbouring stretches of the same rows on
// the source side and on the destination side, where a plain row-major order would give that to
// one side only.
VPS_HD void xpose_plane_order(uint32_t w, uint32_t na, uint32_t nb, uint32_t sa, uint32_t sb,
                              uint32_t& ia, uint32_t& ib)
{
    const uint32_t sr = w / (sa * nb);                          // super-row: sa * nb blocks each
    const uint32_t w1 = w - sr * sa * nb;
    const uint32_t rows = na - sr * sa < sa ? na - sr * sa : sa;
    const uint32_t cfull = nb / sb;                             // full super-columns
    uint32_t sc = w1 / (rows * sb);
    if (sc > cfull) sc = cfull;
    const uint32_t w2 = w1 - sc * rows * sb;
    const uint32_t cols = sc < cfull ? sb : nb - cfull * sb;
    ia = sr * sa + w2 / cols;
    ib = sc * sb + w2 % cols;
}

// Tile q of an XPOSE descriptor: a block of ta x tb elements in the plane of axis xa (contiguous
// in the source) and axis 3 (contiguous in the destination), at fixed coordinates of the two
// other axes.  so/to are the byte offsets of its first element; element (a, b) of the block
// lies at so + (a + b*sstr[3])*es in the source and to + (a*dstr[xa] + b)*es in the destination.
VPS_HD void xpose_tile_geometry(const CopyDesc& d, uint32_t q, uint64_t& so, uint64_t& to,
                                uint32_t& ta, uint32_t& tb)
{
    const uint32_t na = d.chunks_per_row, nb = d.vec_window;
    uint32_t o = q / (na * nb);
    uint32_t ia, ib;
    xpose_plane_order(q - o * na * nb, na, nb, d.rows_per_tile & 0xffffu, d.rows_per_tile >> 16, ia, ib);
    // (the fields of axis xa by selects, the loop unrolled: no array is indexed at run time, so
    // a descriptor held in registers stays there)
    const uint32_t ext_xa = d.xa == 2u ? d.ext[2] : (d.xa == 1u ? d.ext[1] : d.ext[0]);
    const int64_t sstr_xa = d.xa == 2u ? d.sstr[2] : (d.xa == 1u ? d.sstr[1] : d.sstr[0]);
    const int64_t dstr_xa = d.xa == 2u ? d.dstr[2] : (d.xa == 1u ? d.dstr[1] : d.dstr[0]);
    int64_t s = 0, t = 0;
    VPS_UNROLL(3)
    for (int ax = 2; ax >= 0; --ax) {  // the two remaining axes, innermost first
        if ((uint32_t)ax == d.xa) continue;
        const uint32_t c = o % d.ext[ax];
        o /= d.ext[ax];
        s += (int64_t)c * d.sstr[ax];
        t += (int64_t)c * d.dstr[ax];
    }
    const uint32_t a0 = ia * XPOSE_T, b0 = ib * XPOSE_T;
    s += (int64_t)a0 * sstr_xa + (int64_t)b0 * d.sstr[3];
    t += (int64_t)a0 * dstr_xa + (int64_t)b0 * d.dstr[3];
    so = (uint64_t)(s * (int64_t)d.es);
    to = (uint64_t)(t * (int64_t)d.es);
    ta = ext_xa - a0 < (uint32_t)XPOSE_T ? ext_xa - a0 : (uint32_t)XPOSE_T;
    tb = d.ext[3] - b0 < (uint32_t)XPOSE_T ? d.ext[3] - b0 : (uint32_t)XPOSE_T;
}

// Tile q of descriptor `di`.  Chunks of a long run become direct tiles: chunk c covers the
// destination vectors [c*vec_window, (c+1)*vec_window) counted from the RUN_CUT_ALIGN boundary
// at or below the run's first destination byte (with a less aligned buffer base the tiles are
// still disjoint and complete, only less evenly cut).
VPS_HD TileRef make_run_tile(const CopyDesc& d, uint32_t q)   // (d.mode == MODE_RUN; no field of d is indexed at run time)
{
    TileRef t;
    t.src_pitch = 0; t.dst_pitch = 0;
    if (d.chunks_per_row) {
        const bool one_run = d.ext[0] == 1 && d.ext[1] == 1 && d.ext[2] == 1;   // (then every tile is a chunk of it)
        const uint32_t row = one_run ? 0u : q / d.chunks_per_row, c = q - row * d.chunks_per_row;
        uint64_t so, to;
        run_row_offsets(d, row, so, to);
        const uint64_t run_bytes = (uint64_t)d.ext[3] * d.es;
        // (the boundary is where it was when the descriptor was made: d.xa is the phase of dst_byte
        // at that time, so a descriptor that is later moved to another place, as the staged
        // exchange does with its pack descriptors, keeps its cuts and its number of tiles; the
        // windows are taken relative to the run's first byte, which may now lie anywhere)
        const uint64_t d0 = d.dst_byte + to;
        const int64_t pre = (int64_t)((d.xa + to) & (run_cut_align(d.vec_window) - 1)), win = 16ll * d.vec_window;
        int64_t rlo = (int64_t)c * win - pre, rhi = rlo + win;   // the chunk's window, relative to d0
        if (rlo < 0) rlo = 0;
        if (rhi > (int64_t)run_bytes) rhi = (int64_t)run_bytes;
        if (rhi < rlo) rhi = rlo;
        const uint64_t lo = d0 + (uint64_t)rlo, hi = d0 + (uint64_t)rhi;
        t.src = tile_pack_addr(d.src_slot, d.src_byte + so + (lo - d0));
        t.dst = tile_pack_addr(d.dst_slot, lo);
        t.alt_src = d.alt_src_slot >= 0 ? tile_pack_addr(d.alt_src_slot, d.alt_src_byte + so + (lo - d0)) : VPS_TILE_NO_ALT;
        t.nbytes = (uint32_t)(hi - lo);
        t.nruns_flags = (hi > lo ? 1u : 0u) << 8;
    } else {
        const uint32_t k = d.rows_per_tile;
        const uint32_t tps = (d.ext[2] + k - 1) / k;
        const uint32_t slab = q / tps, r0 = (q - slab * tps) * k;
        const uint32_t nruns = d.ext[2] - r0 < k ? d.ext[2] - r0 : k;
        uint64_t so, to;
        run_row_offsets(d, slab * d.ext[2] + r0, so, to);
        t.src = tile_pack_addr(d.src_slot, d.src_byte + so);
        t.dst = tile_pack_addr(d.dst_slot, d.dst_byte + to);
        t.alt_src = d.alt_src_slot >= 0 ? tile_pack_addr(d.alt_src_slot, d.alt_src_byte + so) : VPS_TILE_NO_ALT;
        t.src_pitch = d.sstr[2] * (int64_t)d.es;
        t.dst_pitch = d.dstr[2] * (int64_t)d.es;
        t.nbytes = d.ext[3] * d.es;
        t.nruns_flags = nruns << 8;
    }
    return t;
}

VPS_HD TileRef make_tile(const CopyDesc& d, uint32_t di, uint32_t q)
{
    if (d.mode == MODE_RUN) return make_run_tile(d, q);
    TileRef t;
    t.src_pitch = 0; t.dst_pitch = 0;
    if (d.mode == MODE_XPOSE) {
        uint64_t so, to;
        uint32_t ta, tb;
        xpose_tile_geometry(d, q, so, to, ta, tb);
        t.src = tile_pack_addr(d.src_slot, d.src_byte + so);
        t.dst = tile_pack_addr(d.dst_slot, d.dst_byte + to);
        t.alt_src = d.alt_src_slot >= 0 ? tile_pack_addr(d.alt_src_slot, d.alt_src_byte + so) : VPS_TILE_NO_ALT;
        t.src_pitch = d.sstr[3] * (int64_t)d.es;
        t.dst_pitch = (d.xa == 2u ? d.dstr[2] : (d.xa == 1u ? d.dstr[1] : d.dstr[0])) * (int64_t)d.es;
        t.nbytes = ta | tb << 16;
        t.nruns_flags = TILE_XPOSE | (d.es == 2 ? TILE_ES2 : 0u);
    } else {
        t.src = 0; t.dst = 0;
        t.alt_src = ((uint64_t)q << 32) | di;
        t.nbytes = 0;
        t.nruns_flags = TILE_INDIRECT;
    }
    return t;
}

// What the planner's last per-box step needs: where the statistics, the per-pair byte counts,
// the used-slot flags, the copy descriptors and their tile counts go.
struct FinishCtx {
    int32_t rank, wa, wb;
    bool through_buffers, routes_only;
    bool count_kinds;   // account_box also counts retained / sent / received boxes (else the caller has them)
    PtrLayout layout;
    uint32_t tile_bytes, xpose_shape;
    uint64_t* sum;      // summary block (SUM_* counters at its head)
    uint64_t* pairs;    // all ranks: [src*wb + dst]; one rank r: [src] = src -> r, [wa + dst] = r -> dst
    uint8_t* used;      // [op][slot]
    int64_t nslots;
    CopyDesc* descs;    // [3n]
    int64_t* ntiles;    // [3n + 1]
};

// Once per box: statistics and the payload bytes per (source, destination) pair.
VPS_HD void account_box(const FinishCtx& c, const vps_box& b)
{
    const uint64_t bytes = box_volume(b) * kind_bytes(b.kind);
    if (c.rank < 0) be_atomic_add_runs(c.pairs, (int64_t)b.src_rank * c.wb + b.dst_rank, bytes);
    else {
        if (b.dst_rank == c.rank) be_atomic_add(&c.pairs[b.src_rank], bytes);
        if (b.src_rank == c.rank) be_atomic_add(&c.pairs[c.wa + b.dst_rank], bytes);
    }
    if (!c.count_kinds) return;
    const bool retained = box_retained(b, c.through_buffers);
    be_atomic_count(&c.sum[SUM_NRETAIN], retained);
    be_atomic_count(&c.sum[SUM_NSEND], !retained && (c.rank < 0 || b.src_rank == c.rank));
    be_atomic_count(&c.sum[SUM_NRECV], !retained && (c.rank < 0 || b.dst_rank == c.rank));
}

// Copy descriptor `i` (operation op of box b) and its tile count.
VPS_HD void describe_box_op(const FinishCtx& c, const vps_box& b, int op, int64_t i)
{
    if (c.routes_only) { c.ntiles[i] = 0; return; }
    CopyDesc d;
    make_copy_desc(b, op, c.layout, c.rank, c.through_buffers, c.tile_bytes, c.xpose_shape, d);
    c.descs[i] = d;
    c.ntiles[i] = d.ntiles;
    if (d.ntiles) {
        c.used[op * c.nslots + d.src_slot] = 1;
        c.used[op * c.nslots + d.dst_slot] = 1;
    }
}

// Element k of an ELEM descriptor: byte offsets relative to the descriptor bases.
VPS_HD void elem_offsets(const CopyDesc& d, uint64_t k, int64_t& so, int64_t& to)
{
    const uint32_t c3 = (uint32_t)(k % d.ext[3]); k /= d.ext[3];
    const uint32_t c2 = (uint32_t)(k % d.ext[2]); k /= d.ext[2];
    const uint32_t c1 = (uint32_t)(k % d.ext[1]);
    const uint32_t c0 = (uint32_t)(k / d.ext[1]);
    so = ((int64_t)c0 * d.sstr[0] + (int64_t)c1 * d.sstr[1] + (int64_t)c2 * d.sstr[2] +
          (int64_t)c3 * d.sstr[3]) * (int64_t)d.es;
    to = ((int64_t)c0 * d.dstr[0] + (int64_t)c1 * d.dstr[1] + (int64_t)c2 * d.dstr[2] +
          (int64_t)c3 * d.dstr[3]) * (int64_t)d.es;
}

// ------------------------------------------------------------------------------------------
// Collective intent (Algorithm 1, OptimizePrimitives): per logical tensor and state kind, look
// at the routed boxes ("slices") that leave their rank.
// ------------------------------------------------------------------------------------------

enum { COLL_NONE = 0, COLL_P2P = 1, COLL_BROADCAST = 2, COLL_SCATTER = 3, COLL_GATHER = 4 };
enum : uint32_t { CF_ANY = 1, CF_MULTI_SRC = 2, CF_MULTI_DST = 4, CF_DIFFERENT = 8, CF_NONLINEAR = 16, CF_GAP = 32 };

// Is the box one contiguous range of the row-major flattening of its unsharded tensor?
VPS_HD bool box_is_linear_range(const vps_box& b, const TensorRec& x)
{
    int a = 0;
    while (a < 4 && b.ext[a] == 1) ++a;   // outermost axis that the box really spans
    for (int i = a + 1; i < 4; ++i)
        if (b.lo[i] != 0 || b.ext[i] != x.shape[i]) return false;
    return true;
}

VPS_HD int32_t classify_flags(uint32_t f)
{
    if (!(f & CF_ANY)) return COLL_NONE;
    const bool one_src = !(f & CF_MULTI_SRC), one_dst = !(f & CF_MULTI_DST);
    const bool identical = !(f & CF_DIFFERENT), cont = !(f & (CF_NONLINEAR | CF_GAP));
    if (one_src && !one_dst && identical) return COLL_BROADCAST;
    if (one_src && !one_dst && cont) return COLL_SCATTER;
    if (!one_src && one_dst && cont) return COLL_GATHER;
    return COLL_P2P;
}

template <class T>
VPS_HD int64_t upper_bound_idx(const T* a, int64_t n, T v)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) / 2;
        if (a[mid] <= v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <class T>
VPS_HD int64_t lower_bound_idx(const T* a, int64_t n, T v)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) / 2;
        if (a[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

}  // namespace vps

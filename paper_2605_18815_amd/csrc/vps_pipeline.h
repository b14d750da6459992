// vps_pipeline.h - the sequence of data-parallel steps that build a configuration's piece
// table (mapper) and a transition's routing plan (planner), written once over a small
// backend interface:
//
//   for_each(n, f)            run f(i) for i in [0, n)      -> one HIP kernel lane per item
//   exclusive_scan(in,out,n)  out[i] = sum in[0..i), n+1 long -> rocPRIM device scan
//   sort_pairs(keys,vals,n)   stable ascending by 64-bit key -> rocPRIM device radix sort
//
// The product library instantiates it with the HIP backend only.  The test-suite also
// instantiates it with a sequential CPU backend to exercise the per-item code under bounds
// checks without a GPU.
//
// Steps follow DynaTrain Section 4.1 (F_P), 4.2.1 (intersections, one source per
// destination element), 4.2.2 (flat ZeRO ranges as VPS sub-regions) and 4.3 (per-peer
// contiguous buffers).
#pragma once

#include <chrono>
#include <cstring>
#include <vector>

#include "vps_core.h"
#include "vps_inventory.h"

#if defined(__HIPCC__)
#define VPS_LAMBDA __host__ __device__
#else
#define VPS_LAMBDA
#endif

namespace vps {

// One tag per data-parallel step: it names the kernel in profiles.
namespace step {
struct map_tensor_class {};
struct map_shard_lengths {};
struct map_class_bounds {};
struct map_class_lengths {};
struct map_tensor_offsets {};
struct map_count_pieces {};
struct map_emit_pieces {};
struct plan_count_boxes {};
struct plan_emit_boxes {};
struct plan_key_lo {};
struct plan_key_send {};
struct plan_key_recv {};
struct plan_slot_sizes {};
struct plan_rank_bounds {};
struct plan_positions {};
struct plan_rank_bases {};
struct plan_pair_bytes {};
struct plan_copy_descs {};
struct plan_tile_table {};
struct plan_sorted_boxes {};
struct plan_recv_perm {};
}  // namespace step

struct ConfigData {
    vps_model_desc model;
    vps_parallel_desc par;
    ParConst P;
    int32_t rank_filter = -1;
    // backend memory
    TensorRec* T = nullptr;
    TensorLayout* TL = nullptr;
    ClassRec* C = nullptr;
    int64_t* piece_base = nullptr;  // map_num_items + 1
    vps_piece* pieces = nullptr;
    int64_t npieces = 0;
    // host copies
    std::vector<ClassRec> hC;
};

struct PlanData {
    ParConst A, B;
    int32_t rank = -1;
    uint32_t tile_bytes = 0;
    PtrLayout layout;
    int64_t nboxes = 0;
    // backend memory
    CopyDesc* descs = nullptr;  // 3*nboxes: retain | pack (send order), unpack (receive order)
    TileRef* tiles = nullptr;
    void** ptr_table = nullptr;  // all-ranks plans: device copy of the pointer table
    // host copies
    std::vector<vps_box> boxes_send_order;   // sorted by (src, dst, kind order, tensor, lo)
    std::vector<uint32_t> recv_perm;         // receive order -> index into boxes_send_order
    std::vector<int64_t> tile_base;          // 3*nboxes + 1
    std::vector<int64_t> first_send, first_recv;  // per rank: first box index, W+1 long
    std::vector<uint64_t> send_base, recv_base;   // per rank: offset of its buffer, W+1 long
    std::vector<uint64_t> pair_bytes;             // [src*WB + dst]
    std::vector<void*> host_ptrs;                 // staging for the pointer table
    vps_plan_stats_t stats;
};

template <class BE>
void free_config(BE& be, ConfigData& c)
{
    be.free(c.T); be.free(c.TL); be.free(c.C); be.free(c.piece_base); be.free(c.pieces);
    c.T = nullptr; c.TL = nullptr; c.C = nullptr; c.piece_base = nullptr; c.pieces = nullptr;
}

template <class BE>
void free_plan(BE& be, PlanData& p)
{
    be.free(p.descs); be.free(p.tiles); be.free(p.ptr_table);
    p.descs = nullptr; p.tiles = nullptr; p.ptr_table = nullptr;
}

// ---------------------------------------------------------------------------------- mapper

template <class BE>
void build_config(BE& be, const vps_model_desc& model, const vps_parallel_desc& par,
                  int32_t rank_filter, ConfigData& c)
{
    check_descs(model, par);
    std::vector<TensorRec> inv;
    build_inventory(model, inv);
    const int32_t nt = (int32_t)inv.size();
    c.model = model; c.par = par; c.rank_filter = rank_filter;
    c.P = make_par_const(model, par, nt);
    const ParConst P = c.P;
    if (rank_filter < -1 || rank_filter >= P.world) throw Error{ VPS_ERR_RANK_RANGE, "rank outside the configuration's world" };

    c.T = be.template alloc<TensorRec>(nt);
    c.TL = be.template alloc<TensorLayout>(nt);
    c.C = be.template alloc<ClassRec>(P.ncls);
    be.upload(c.T, inv.data(), sizeof(TensorRec) * (size_t)nt);

    // (1) class and shard length of every tensor; sort keys in flat-buffer order
    uint64_t* key = be.template alloc<uint64_t>(nt);
    uint32_t* val = be.template alloc<uint32_t>(nt);
    int64_t* len = be.template alloc<int64_t>(nt + 1);
    int64_t* ofs = be.template alloc<int64_t>(nt + 1);
    int64_t* cbeg = be.template alloc<int64_t>(P.ncls + 1);
    {
        const TensorRec* T = c.T; TensorLayout* TL = c.TL;
        be.for_each(step::map_tensor_class(), nt, [=] VPS_LAMBDA(int64_t q) {
            const int32_t t = P.flat_order ? nt - 1 - (int32_t)q : (int32_t)q;
            const TensorRec x = T[t];
            TensorLayout tl;
            tl.cls = class_of_tensor(P, x);
            tl.shard_len = shard_elems(P, x);
            tl.start = 0; tl.pad_ = 0;
            TL[t] = tl;
            key[q] = (uint64_t)tl.cls;
            val[q] = (uint32_t)t;
        });
    }
    // (2) group the tensors by class, keeping flat order inside a class
    be.sort_pairs(key, val, nt);
    {
        const TensorLayout* TL = c.TL;
        be.for_each(step::map_shard_lengths(), nt + 1, [=] VPS_LAMBDA(int64_t k) { len[k] = k < nt ? (int64_t)TL[val[k]].shard_len : 0; });
    }
    be.exclusive_scan(len, ofs, nt);
    // (3) class boundaries, lengths and padding
    {
        ClassRec* C = c.C;
        be.for_each(step::map_class_bounds(), P.ncls + 1, [=] VPS_LAMBDA(int64_t cls) { cbeg[cls] = lower_bound_idx(key, (int64_t)nt, (uint64_t)cls); });
        be.for_each(step::map_class_lengths(), P.ncls, [=] VPS_LAMBDA(int64_t cls) {
            ClassRec r;
            r.len = (uint64_t)(ofs[cbeg[cls + 1]] - ofs[cbeg[cls]]);
            const uint64_t quantum = 8ull * (uint64_t)(cls < P.pp ? P.ddp : P.dp);
            r.padded = (r.len + quantum - 1) / quantum * quantum;
            C[cls] = r;
        });
        TensorLayout* TL = c.TL;
        be.for_each(step::map_tensor_offsets(), nt, [=] VPS_LAMBDA(int64_t k) {
            TL[val[k]].start = (uint64_t)(ofs[k] - ofs[cbeg[key[k]]]);
        });
    }
    be.free(key); be.free(val); be.free(len); be.free(ofs); be.free(cbeg);

    // (4) pieces: count, scan, emit
    const int64_t nitems = map_num_items(P);
    int64_t* cnt = be.template alloc<int64_t>(nitems + 1);
    c.piece_base = be.template alloc<int64_t>(nitems + 1);
    MapCtx mc;
    mc.P = P; mc.T = c.T; mc.TL = c.TL; mc.C = c.C; mc.rank_filter = rank_filter;
    be.for_each(step::map_count_pieces(), nitems + 1, [=] VPS_LAMBDA(int64_t i) { cnt[i] = i < nitems ? map_item_pieces(mc, i, nullptr) : 0; });
    be.exclusive_scan(cnt, c.piece_base, nitems);
    be.download(&c.npieces, c.piece_base + nitems, sizeof(int64_t));
    c.pieces = be.template alloc<vps_piece>(c.npieces);
    {
        const int64_t* pb = c.piece_base; vps_piece* pieces = c.pieces;
        be.for_each(step::map_emit_pieces(), nitems, [=] VPS_LAMBDA(int64_t i) {
            if (pb[i + 1] > pb[i]) map_item_pieces(mc, i, pieces + pb[i]);
        });
    }
    be.free(cnt);
    c.hC.resize((size_t)P.ncls);
    be.download_later(c.hC.data(), c.C, sizeof(ClassRec) * (size_t)P.ncls);
    be.sync();
}

inline uint64_t config_buffer_elems(const ConfigData& c, int32_t rank, int32_t buf)
{
    const RankCoord rc = decode_rank(c.P, rank);
    const int group = buf / 4, kind = buf % 4;
    const ClassRec& cl = c.hC[(size_t)(group == 0 ? rc.pp : c.P.pp + rc.pp * c.P.ep + rc.ep)];
    const int D = group == 0 ? c.P.ddp : c.P.dp;
    return (c.P.zero == 1 && kind != 0) ? cl.padded / (uint64_t)D : cl.padded;
}

// --------------------------------------------------------------------------------- planner

template <class BE>
void build_plan(BE& be, const ConfigData& ca, const ConfigData& cb, int32_t rank,
                uint32_t tile_bytes, PlanData& p)
{
    const auto t_start = std::chrono::steady_clock::now();
    if (ca.rank_filter != -1 || cb.rank_filter != -1)
        throw Error{ VPS_ERR_INVALID_ARG, "planning needs configurations described with rank = -1" };
    if (memcmp(&ca.model, &cb.model, sizeof(vps_model_desc)) != 0)
        throw Error{ VPS_ERR_MODEL_MISMATCH, "source and destination describe different models" };
    const ParConst A = ca.P, B = cb.P;
    const int32_t WA = A.world, WB = B.world, W = WA > WB ? WA : WB;
    if (rank < -1 || rank >= W) throw Error{ VPS_ERR_RANK_RANGE, "rank outside both worlds" };
    p.A = A; p.B = B; p.rank = rank; p.tile_bytes = tile_bytes;
    p.layout.all_ranks = rank < 0; p.layout.wa = WA; p.layout.wb = WB;
    const PtrLayout layout = p.layout;

    // (1) intersections: one item per destination piece
    PlanCtx pc;
    pc.A = A; pc.B = B; pc.T = ca.T; pc.SP = ca.pieces; pc.DP = cb.pieces; pc.sbase = ca.piece_base;
    pc.rank = rank;
    const int64_t nd = cb.npieces;
    int64_t* cnt = be.template alloc<int64_t>(nd + 1);
    int64_t* bbase = be.template alloc<int64_t>(nd + 1);
    be.for_each(step::plan_count_boxes(), nd + 1, [=] VPS_LAMBDA(int64_t d) { cnt[d] = d < nd ? plan_item_boxes(pc, d, nullptr) : 0; });
    be.exclusive_scan(cnt, bbase, nd);
    int64_t n = 0;
    be.download(&n, bbase + nd, sizeof(int64_t));
    if (n >= (int64_t)1 << 31) throw Error{ VPS_ERR_OOM, "more than 2^31 boxes" };
    p.nboxes = n;
    vps_box* boxes = be.template alloc<vps_box>(n);
    be.for_each(step::plan_emit_boxes(), nd, [=] VPS_LAMBDA(int64_t d) {
        if (bbase[d + 1] > bbase[d]) plan_item_boxes(pc, d, boxes + bbase[d]);
    });
    be.free(cnt); be.free(bbase);

    // (2) order: by lo corner first, then stably by (owner rank, peer, kind order, tensor)
    uint64_t* kmin = be.template alloc<uint64_t>(n);
    uint64_t* kmaj = be.template alloc<uint64_t>(n);
    uint32_t* by_lo = be.template alloc<uint32_t>(n);
    uint32_t* ord_s = be.template alloc<uint32_t>(n);
    uint32_t* ord_r = be.template alloc<uint32_t>(n);
    {
        const TensorRec* T = ca.T;
        be.for_each(step::plan_key_lo(), n, [=] VPS_LAMBDA(int64_t k) { kmin[k] = box_minor_key(boxes[k], T[boxes[k].tensor]); by_lo[k] = (uint32_t)k; });
        be.sort_pairs(kmin, by_lo, n);
        be.for_each(step::plan_key_send(), n, [=] VPS_LAMBDA(int64_t k) { ord_s[k] = by_lo[k]; kmaj[k] = box_major_key(boxes[by_lo[k]], false); });
        be.sort_pairs(kmaj, ord_s, n);
        be.for_each(step::plan_key_recv(), n, [=] VPS_LAMBDA(int64_t k) { ord_r[k] = by_lo[k]; kmaj[k] = box_major_key(boxes[by_lo[k]], true); });
        be.sort_pairs(kmaj, ord_r, n);
    }
    be.free(kmin); be.free(kmaj); be.free(by_lo);

    // (3) buffer positions: exclusive scan of 16-byte aligned box sizes in each order
    int64_t* sz = be.template alloc<int64_t>(n + 1);
    int64_t* pos = be.template alloc<int64_t>(n + 1);
    int32_t* owner = be.template alloc<int32_t>(n);
    int64_t* first = be.template alloc<int64_t>(W + 1);
    uint64_t* rbase = be.template alloc<uint64_t>(2 * (W + 1));
    p.first_send.assign((size_t)W + 1, 0); p.first_recv.assign((size_t)W + 1, 0);
    p.send_base.assign((size_t)W + 1, 0); p.recv_base.assign((size_t)W + 1, 0);
    for (int side = 0; side < 2; ++side) {
        const uint32_t* ord = side == 0 ? ord_s : ord_r;
        be.for_each(step::plan_slot_sizes(), n + 1, [=] VPS_LAMBDA(int64_t k) {
            if (k == n) { sz[k] = 0; return; }
            const vps_box& b = boxes[ord[k]];
            const int32_t own = side == 0 ? b.src_rank : b.dst_rank;
            owner[k] = own;
            const bool resident = rank < 0 || own == rank;
            sz[k] = (b.src_rank != b.dst_rank && resident) ? (int64_t)box_slot_bytes(b) : 0;
        });
        be.exclusive_scan(sz, pos, n);
        be.for_each(step::plan_rank_bounds(), W + 1, [=] VPS_LAMBDA(int64_t r) { first[r] = lower_bound_idx(owner, n, (int32_t)r); });
        be.for_each(step::plan_positions(), n, [=] VPS_LAMBDA(int64_t k) {
            vps_box& b = boxes[ord[k]];
            if (sz[k] == 0) return;
            const uint64_t rel = (uint64_t)(pos[k] - pos[first[owner[k]]]);
            if (side == 0) b.send_pos = rel; else b.recv_pos = rel;
        });
        std::vector<int64_t>& hf = side == 0 ? p.first_send : p.first_recv;
        std::vector<uint64_t>& hb = side == 0 ? p.send_base : p.recv_base;
        be.for_each(step::plan_rank_bases(), W + 1, [=] VPS_LAMBDA(int64_t r) { rbase[side * (W + 1) + r] = (uint64_t)pos[first[r]]; });
        be.download_later(hf.data(), first, sizeof(int64_t) * (size_t)(W + 1));
        be.download_later(hb.data(), rbase + side * (W + 1), sizeof(uint64_t) * (size_t)(W + 1));
    }
    be.free(sz); be.free(pos); be.free(owner); be.free(first); be.free(rbase);

    // (4) payload bytes per (source, destination) pair
    uint64_t* pairs = be.template alloc<uint64_t>((int64_t)WA * WB);
    be.zero(pairs, sizeof(uint64_t) * (size_t)WA * (size_t)WB);
    be.for_each(step::plan_pair_bytes(), n, [=] VPS_LAMBDA(int64_t k) {
        const vps_box& b = boxes[k];
        be_atomic_add(&pairs[(int64_t)b.src_rank * WB + b.dst_rank], box_volume(b) * kind_bytes(b.kind));
    });
    p.pair_bytes.resize((size_t)WA * (size_t)WB);
    be.download_later(p.pair_bytes.data(), pairs, sizeof(uint64_t) * (size_t)WA * (size_t)WB);
    be.free(pairs);

    // (5) copy descriptors and tile table
    p.descs = be.template alloc<CopyDesc>(3 * n);
    int64_t* nt = be.template alloc<int64_t>(3 * n + 1);
    int64_t* tb = be.template alloc<int64_t>(3 * n + 1);
    {
        CopyDesc* descs = p.descs;
        be.for_each(step::plan_copy_descs(), 3 * n + 1, [=] VPS_LAMBDA(int64_t i) {
            if (i == 3 * n) { nt[i] = 0; return; }
            const int op = (int)(i / n);
            const int64_t k = i % n;
            const vps_box& b = boxes[op == OP_UNPACK ? ord_r[k] : ord_s[k]];
            CopyDesc d;
            make_copy_desc(b, op, layout, rank, tile_bytes, d);
            descs[i] = d;
            nt[i] = d.ntiles;
        });
    }
    be.exclusive_scan(nt, tb, 3 * n);
    p.tile_base.resize((size_t)(3 * n + 1));
    be.download(p.tile_base.data(), tb, sizeof(int64_t) * (size_t)(3 * n + 1));
    const int64_t ntiles = p.tile_base[(size_t)(3 * n)];
    if (ntiles >= (int64_t)1 << 31) throw Error{ VPS_ERR_OOM, "more than 2^31 tiles" };
    p.tiles = be.template alloc<TileRef>(ntiles);
    {
        TileRef* tiles = p.tiles;
        const CopyDesc* descs = p.descs;
        be.for_each(step::plan_tile_table(), ntiles, [=] VPS_LAMBDA(int64_t t) {
            const int64_t d = upper_bound_idx(tb, 3 * n + 1, t) - 1;
            tiles[t] = make_tile(descs[d], (uint32_t)d, (uint32_t)(t - tb[d]));
        });
    }
    be.free(nt); be.free(tb);

    // (6) host copies for queries
    {
        vps_box* sorted = be.template alloc<vps_box>(n);
        uint32_t* inv = be.template alloc<uint32_t>(n);
        uint32_t* rperm = be.template alloc<uint32_t>(n);
        be.for_each(step::plan_sorted_boxes(), n, [=] VPS_LAMBDA(int64_t k) { sorted[k] = boxes[ord_s[k]]; inv[ord_s[k]] = (uint32_t)k; });
        be.for_each(step::plan_recv_perm(), n, [=] VPS_LAMBDA(int64_t k) { rperm[k] = inv[ord_r[k]]; });
        p.boxes_send_order.resize((size_t)n);
        p.recv_perm.resize((size_t)n);
        be.download_later(p.boxes_send_order.data(), sorted, sizeof(vps_box) * (size_t)n);
        be.download_later(p.recv_perm.data(), rperm, sizeof(uint32_t) * (size_t)n);
        be.free(sorted); be.free(inv); be.free(rperm);
    }
    be.free(ord_s); be.free(ord_r); be.free(boxes);
    if (layout.all_ranks) p.ptr_table = be.template alloc<void*>(num_slots(layout));
    p.host_ptrs.assign((size_t)num_slots(layout), nullptr);
    be.sync();

    vps_plan_stats_t& st = p.stats;
    st = vps_plan_stats_t();
    st.num_boxes = n;
    std::vector<char> peer_out((size_t)W, 0), peer_in((size_t)W, 0);
    for (const vps_box& b : p.boxes_send_order) {
        if (b.src_rank == b.dst_rank) { st.num_retain_boxes++; continue; }
        if (rank < 0 || b.src_rank == rank) { st.num_send_boxes++; if (rank >= 0) peer_out[(size_t)b.dst_rank] = 1; }
        if (rank < 0 || b.dst_rank == rank) { st.num_recv_boxes++; if (rank >= 0) peer_in[(size_t)b.src_rank] = 1; }
    }
    for (int r = 0; r < W; ++r) { st.num_peers_out += peer_out[(size_t)r]; st.num_peers_in += peer_in[(size_t)r]; }
    st.num_retain_tiles = p.tile_base[(size_t)n] - p.tile_base[0];
    st.num_pack_tiles = p.tile_base[(size_t)(2 * n)] - p.tile_base[(size_t)n];
    st.num_unpack_tiles = p.tile_base[(size_t)(3 * n)] - p.tile_base[(size_t)(2 * n)];
    st.plan_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count();
}

// Tile range [begin, end) of operation `op` for `rank` (-1: every rank).
inline void plan_tile_range(const PlanData& p, int op, int32_t rank, int64_t& begin, int64_t& end)
{
    const int64_t n = p.nboxes;
    const std::vector<int64_t>& first = op == OP_UNPACK ? p.first_recv : p.first_send;
    const int64_t k0 = rank < 0 ? 0 : first[(size_t)rank];
    const int64_t k1 = rank < 0 ? n : first[(size_t)rank + 1];
    begin = p.tile_base[(size_t)(op * n + k0)];
    end = p.tile_base[(size_t)(op * n + k1)];
}

}  // namespace vps

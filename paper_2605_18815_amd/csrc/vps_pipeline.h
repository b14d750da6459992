// vps_pipeline.h - the sequence of data-parallel steps that build a configuration's piece
// table (mapper) and a transition's routing plan (planner), written once over a small
// backend interface:
//
//   for_each(n, f)            run f(i) for i in [0, n)      -> one HIP kernel lane per item
//   exclusive_scan(in,out,n)  out[i] = sum in[0..i), n+1 long -> workgroup scans (k_scan_*)
//   sort_pairs(keys,vals,n)   stable ascending by 64-bit key -> radix sort (k_sort_count, k_sort_scatter)
//
// The product library instantiates it with the HIP backend only.  The test-suite also
// instantiates it with a sequential CPU backend to exercise the per-item code under bounds
// checks without a GPU.
//
// Steps follow DynaTrain Section 4.1 (F_P), 4.2.1 (intersections, one source per
// destination element), 4.2.2 (flat ZeRO ranges as VPS sub-regions) and 4.3 (per-peer
// contiguous buffers).
#pragma once

#include <algorithm>
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
struct map_count_pieces {};
struct map_emit_pieces {};
struct plan_order_by_counting {};
struct plan_keys {};
struct plan_key_send {};
struct plan_key_recv {};
struct plan_slot_sizes {};
struct plan_positions {};
struct plan_sorted_boxes {};
struct plan_recv_perm {};
struct plan_pair_bytes {};
struct plan_pair_counts {};
struct plan_pair_sums {};
struct plan_pair_starts {};
struct plan_pair_scatter {};
struct plan_pair_rank {};
struct plan_pair_place {};
struct plan_copy_descs {};
struct plan_rank_tables {};
struct coll_keys {};
struct coll_group_key {};
struct coll_flags {};
struct coll_classes {};
struct stage_tile_keys {};
struct stage_tile_gather {};
struct stage_descs {};
struct stage_exchange_tiles {};
struct stage_bounds {};
}  // namespace step

struct ConfigData {
    vps_model_desc model;
    vps_parallel_desc par;
    ParConst P;
    ModelConst M;
    int32_t rank_filter = -1;
    // backend memory
    TensorRec* T = nullptr;
    TensorLayout* TL = nullptr;
    ClassRec* C = nullptr;
    // made on demand by the piece queries
    int64_t* piece_base = nullptr;  // map_num_items + 1
    vps_piece* pieces = nullptr;
    int64_t npieces = -1;
    // host copies
    bool host_ready = false;        // hC holds the class table
    std::vector<ClassRec> hC;
    uint64_t tensor_numel_max = 1;  // elements of the largest logical tensor
};

inline int bits_for(uint64_t max_value_exclusive)
{
    int b = 1;
    while (b < 64 && (1ull << b) < max_value_exclusive) ++b;
    return b;
}

// What the host keeps of a plan.  Everything here arrives with the one device-to-host copy of the
// plan's summary block; the boxes themselves stay on the device until a query asks for them.
struct PlanData {
    ParConst A, B;
    int32_t rank = -1;
    uint32_t tile_bytes = 0;
    bool routes_only = false;  // no copy descriptors and no tile table: queries only
    bool through_buffers = false;  // a rank is its own peer: nothing is copied directly
    PtrLayout layout;
    int64_t nboxes = 0;
    // backend memory
    CopyDesc* descs = nullptr;  // 3*nboxes: retain | pack (send order), unpack (receive order)
    TileRef* tiles = nullptr;
    int64_t* d_tile_base = nullptr;  // 3*nboxes + 1: first tile of every descriptor
    void** ptr_table = nullptr;  // all-ranks plans: device copy of the pointer table
    vps_box* d_boxes = nullptr;      // the boxes in send order: (src, dst, kind order, tensor, lo)
    uint32_t* d_recv_perm = nullptr; // receive order -> index into d_boxes
    // host copies, fetched on first use
    bool host_boxes_ready = false;
    std::vector<vps_box> boxes_send_order;
    std::vector<uint32_t> recv_perm;
    std::vector<int64_t> tile_base;
    // host copies that come with the plan
    std::vector<int64_t> first_send, first_recv;  // per rank: first box index, W+1 long
    std::vector<uint64_t> send_base, recv_base;   // per rank: offset of its buffer, W+1 long
    std::vector<int64_t> op_tile[3];              // per operation and rank: first tile, W+1 long
    std::vector<uint64_t> pair_bytes;             // all ranks: [src*WB + dst]; one rank r:
                                                  // [src] = src -> r for src < WA, [WA + dst] = r -> dst
    std::vector<uint8_t> used[3];                 // per operation: pointer-table slots it dereferences
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
    be.free(p.descs); be.free(p.tiles); be.free(p.ptr_table); be.free(p.d_boxes); be.free(p.d_recv_perm);
    be.free(p.d_tile_base);
    p.descs = nullptr; p.tiles = nullptr; p.ptr_table = nullptr; p.d_boxes = nullptr; p.d_recv_perm = nullptr;
    p.d_tile_base = nullptr;
}

// ---------------------------------------------------------------------------------- mapper

// F_P (Section 4.1, 4.2.2): the tensor table and, per flat-buffer class, the offsets of the
// tensors' shards.  Two launches on the null stream, nothing waits: the class table is copied
// to the host when the first size query asks for it.
template <class BE>
void build_config(BE& be, const vps_model_desc& model, const vps_parallel_desc& par,
                  int32_t rank_filter, ConfigData& c)
{
    check_descs(model, par);
    c.M = make_model_const(model);
    const ModelConst M = c.M;
    const int32_t nt = M.nt;
    c.model = model; c.par = par; c.rank_filter = rank_filter;
    c.P = make_par_const(model, par, nt);
    const ParConst P = c.P;
    if (rank_filter < -1 || rank_filter >= P.world) throw Error{ VPS_ERR_RANK_RANGE, "rank outside the configuration's world" };
    c.tensor_numel_max = model_numel_max(M);

    c.T = be.template alloc<TensorRec>(nt);
    c.TL = be.template alloc<TensorLayout>(nt);
    c.C = be.template alloc<ClassRec>(P.ncls);
    be.layout_classes(P, M, c.T, c.TL, c.C);   // tensor table and flat offsets in one launch
    c.hC.resize((size_t)P.ncls);
    c.host_ready = false;
}

// The class table on the host (buffer sizes), waiting for the mapping kernels if need be.
template <class BE>
void ensure_config_host(BE& be, ConfigData& c)
{
    if (c.host_ready) return;
    be.download(c.hC.data(), c.C, sizeof(ClassRec) * c.hC.size());
    c.host_ready = true;
}

// The piece table (Section 4.1, sub-VPS): only the piece queries need it; the planner derives
// the pieces of an item on the fly.
template <class BE>
void ensure_pieces(BE& be, ConfigData& c)
{
    if (c.npieces >= 0) return;
    const ParConst P = c.P;
    const int64_t nitems = map_num_items(P);
    int64_t* cnt = be.template alloc<int64_t>(nitems + 1);
    c.piece_base = be.template alloc<int64_t>(nitems + 1);
    MapCtx mc;
    mc.P = P; mc.T = c.T; mc.TL = c.TL; mc.C = c.C; mc.rank_filter = c.rank_filter;
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
    be.sync();
}

inline uint64_t config_buffer_elems(const ConfigData& c, int32_t rank, int32_t buf)
{
    const RankCoord rc = decode_rank(c.P, rank);
    const int group = buf / 4, kind = buf % 4;
    const ClassRec& cl = c.hC[(size_t)(group == 0 ? rc.pp : c.P.pp + rc.pp * c.P.ep + rc.ep)];
    const int D = group_dp(c.P, group);
    return (c.P.zero == 1 && kind != 0) ? cl.padded / (uint64_t)D : cl.padded;
}

// --------------------------------------------------------------------------------- planner

// Layout of a plan's summary block (64-bit words): counters, per-rank tables, pair bytes, then
// one byte per (operation, pointer-table slot).  It is cleared before planning, filled by the
// planning kernels and copied to the host once.
struct SummaryLayout {
    int64_t W, npairs, nslots;
    int64_t rank_tables() const { return SUM_HEADER; }
    int64_t pairs() const { return SUM_HEADER + 7 * (W + 1); }
    int64_t used() const { return pairs() + npairs; }
    int64_t words() const { return used() + (3 * nslots + 7) / 8; }
};

template <class BE>
void build_plan(BE& be, const ConfigData& ca, const ConfigData& cb, int32_t rank,
                uint32_t tile_bytes, uint32_t xpose_shape, uint32_t small_limit, bool routes_only,
                bool through_buffers, int64_t tile_hint, int64_t box_hint, PlanData& p, bool lane_list = true,
                int pair_work_log2 = PAIR_BUCKET_WORK_LOG2)
{
    const auto t_start = std::chrono::steady_clock::now();
    if (ca.rank_filter != -1 || cb.rank_filter != -1)
        throw Error{ VPS_ERR_INVALID_ARG, "planning needs configurations described with rank = -1" };
    if (memcmp(&ca.model, &cb.model, sizeof(vps_model_desc)) != 0)
        throw Error{ VPS_ERR_MODEL_MISMATCH, "source and destination describe different models" };
    const ParConst A = ca.P, B = cb.P;
    const int32_t WA = A.world, WB = B.world, W = WA > WB ? WA : WB;
    if (rank < -1 || rank >= W) throw Error{ VPS_ERR_RANK_RANGE, "rank outside both worlds" };
    if (rank < 0 && (int64_t)WA * WB > ((int64_t)1 << 26))
        throw Error{ VPS_ERR_OOM, "an all-ranks plan of this many ranks needs a byte matrix above 512 MiB" };
    p.A = A; p.B = B; p.rank = rank; p.tile_bytes = tile_bytes; p.routes_only = routes_only;
    p.through_buffers = through_buffers;
    p.layout.all_ranks = rank < 0; p.layout.wa = WA; p.layout.wb = WB;
    const PtrLayout layout = p.layout;
    be.after_null_stream();   // the configurations were mapped on the null stream

    PlanCtx pc;
    pc.A = A; pc.B = B; pc.rank = rank;
    pc.ma.P = A; pc.ma.T = ca.T; pc.ma.TL = ca.TL; pc.ma.C = ca.C; pc.ma.rank_filter = -1;
    pc.mb.P = B; pc.mb.T = cb.T; pc.mb.TL = cb.TL; pc.mb.C = cb.C; pc.mb.rank_filter = -1;
    plan_set_rank_ranges(pc);

    SummaryLayout SL;
    SL.W = W; SL.npairs = rank < 0 ? (int64_t)WA * WB : (int64_t)WA + WB; SL.nslots = num_slots(layout);
    uint64_t* sum = (uint64_t*)be.alloc_zeroed(sizeof(uint64_t) * (size_t)SL.words());
    uint64_t* pairs = sum + SL.pairs();
    uint8_t* used = (uint8_t*)(sum + SL.used());
    const int64_t nslots = SL.nslots;

    // (1) intersections: every lane walks the routed boxes of its item and writes each, with its
    // ordering keys, into the next free slot of the raw table (one atomic per wavefront and
    // step).  The table holds `cap` boxes; a plan with more is planned again with the exact size.
    // (a caller that has seen this transition before passes its box count, see the tile hint below)
    int64_t cap = box_hint > (int64_t)small_limit ? box_hint : (int64_t)small_limit;
    vps_box* raw = be.template alloc<vps_box>(cap);
    OrderRec* recs = be.template alloc<OrderRec>(cap);
    bool listed = false;
    // An all-ranks plan that is known to be large (the caller has seen the transition before) is
    // going to be ordered pair by pair: then the emission counts its boxes per pair as it makes
    // them, which saves that ordering its first pass over the box table.
    const bool pair_path = pair_work_log2 > 0 && rank < 0 && (int64_t)WA * WB <= PAIR_BUCKET_MAX_PAIRS;
    const int64_t np = (int64_t)WA * WB;
    uint64_t* pcount = nullptr;   // [4 np]: boxes per pair, buffer bytes per pair, scatter cursors, first places in the send order
    PairCounts counted;
    counted.count = counted.bytes = nullptr; counted.wb = WB;
    if (pair_path && box_hint > (int64_t)small_limit) {
        pcount = be.template alloc<uint64_t>(4 * np);
        be.zero(pcount, sizeof(uint64_t) * (size_t)(3 * np));
        counted.count = pcount; counted.bytes = pcount + np;
    }
    auto emit = [&](bool two_launches) {
        listed = be.plan_emit(pc, rank < 0 ? PLAN_ALL : PLAN_RANK, through_buffers, raw, recs, (uint64_t)cap, sum + SUM_NBOXES,
                              sum + SUM_NLISTED, two_launches, counted);
    };
    emit(lane_list);

    FinishCtx fc;
    fc.rank = rank; fc.wa = WA; fc.wb = WB; fc.through_buffers = through_buffers; fc.routes_only = routes_only;
    fc.count_kinds = true;
    fc.layout = layout; fc.tile_bytes = tile_bytes; fc.xpose_shape = xpose_shape;
    fc.sum = sum; fc.pairs = pairs; fc.used = used; fc.nslots = nslots;

    // (2) up to small_limit boxes: order and buffer positions by counting.  Box k's index in the
    // send order is the number of boxes with a smaller (src, dst, kind order, tensor, lo) key, its
    // position the bytes of the travelling ones among them that share its source; the same for
    // the receive order.  The lane then writes the box to its place and builds its copy
    // descriptors.  One launch, no sort, no scan.
    const int64_t ns = small_limit;          // bound of the optimistic path
    vps_box* sorted = be.template alloc<vps_box>(ns);
    uint32_t* rperm = be.template alloc<uint32_t>(ns);
    uint64_t* gs = be.template alloc<uint64_t>(ns + 1);
    uint64_t* gr = be.template alloc<uint64_t>(ns + 1);
    CopyDesc* descs = routes_only ? nullptr : be.template alloc<CopyDesc>(3 * ns);
    int64_t* ntl = be.template alloc<int64_t>(3 * ns + 1);
    int64_t* tb = be.template alloc<int64_t>(3 * ns + 1);
    const uint64_t* nbox = sum + SUM_NBOXES;
    fc.descs = descs; fc.ntiles = ntl;
    uint64_t* rank_rows = sum + SL.rank_tables();
    be.order_by_counting_each(step::plan_order_by_counting(), recs, nbox, ns, [=] VPS_LAMBDA(uint32_t k, uint32_t part) {
        return part > 2 ? vps_box() : raw[k];   // (the box itself, for the three lanes that go on)
    }, [=] VPS_LAMBDA(uint32_t k, const OrderPlace& o, uint32_t part, const vps_box& held) {
        if (part > 2) return;   // three lanes go on, one per copy operation
        const int64_t n = (int64_t)*nbox;
        vps_box b = held;
        const OrderRec rec = recs[k];
        if (rec.bytes_flags & ORD_SENDS) b.send_pos = o.gpos_s - o.base_s;
        if (rec.bytes_flags & ORD_RECEIVES) b.recv_pos = o.gpos_r - o.base_r;
        if (part == 0) {
            sorted[o.idx_s] = b;
            rperm[o.idx_r] = o.idx_s;
            gs[o.idx_s] = o.gpos_s; gr[o.idx_r] = o.gpos_r;
            // the last box of either order closes the cumulative positions
            if (o.idx_s == n - 1) gs[n] = o.gpos_s + order_send_bytes(rec);
            if (o.idx_r == n - 1) gr[n] = o.gpos_r + order_recv_bytes(rec);
            if (k == 0) ntl[3 * n] = 0;
            account_box(fc, b);
            // boxes per source and per destination rank, in the first two rows of the rank
            // tables: their prefix sums are every rank's first box in the two orders
            be_atomic_add(rank_rows + b.src_rank, 1);
            be_atomic_add(rank_rows + (W + 1) + b.dst_rank, 1);
        }
        describe_box_op(fc, b, (int)part, part * n + (part == OP_UNPACK ? o.idx_r : o.idx_s));
    });
    // (3) tile bases by a prefix sum, and per rank: first box, buffer offset and first tile of
    // every operation
    int64_t* rt = (int64_t*)(sum + SL.rank_tables());
    // (rows 0 and 1 of the tables, the first box of every rank in the two orders, are there before)
    auto rank_row = [=] VPS_LAMBDA(int64_t r, int64_t n, const uint64_t* gsend, const uint64_t* grecv, const int64_t* tbase) {
        if (n == 0) {   // nothing is routed at all: no box has written the cumulative positions
            for (int c = 2; c < 7; ++c) rt[c * (W + 1) + r] = 0;
            return;
        }
        const int64_t fs = rt[0 * (W + 1) + r], fr = rt[1 * (W + 1) + r];
        rt[2 * (W + 1) + r] = (int64_t)gsend[fs];
        rt[3 * (W + 1) + r] = (int64_t)grecv[fr];
        rt[4 * (W + 1) + r] = tbase[fs];
        rt[5 * (W + 1) + r] = tbase[n + fs];
        rt[6 * (W + 1) + r] = tbase[2 * n + fr];
    };
    // (the same launch leaves a copy of the summary block in pinned host memory, unless the block
    // is large, i.e. holds the byte matrix of an all-ranks plan: one workgroup would take longer
    // over that than a copy command)
    std::vector<uint64_t> hsum((size_t)SL.words());
    const bool mirrored = SL.words() <= 4096;
    uint64_t* hmirror = mirrored ? (uint64_t*)be.host_mirror(hsum.data(), sizeof(uint64_t) * hsum.size()) : nullptr;
    be.exclusive_scan_counted_then_each(step::plan_rank_tables(), ntl, tb, 3 * ns + 1, nbox, 3, rt, W + 1, 2, W + 1, [=] VPS_LAMBDA(int64_t r) {
        // (rows 0 and 1 hold the first boxes by now: the counts of the ordering pass, summed)
        rank_row(r, (int64_t)*nbox, gs, gr, tb);
    }, sum, hmirror, mirrored ? SL.words() : 0);

    // (4) the tile table.  Its size is only known on the device so far; when the caller has seen
    // this transition before it passes the size as a hint and the table is built before the host
    // looks at anything, so that the whole plan needs one synchronisation.
    TileRef* tiles = nullptr;
    int64_t tiles_cap = 0;
    if (!routes_only && tile_hint > 0) {
        tiles_cap = tile_hint;
        tiles = be.template alloc<TileRef>(tiles_cap);
        be.tile_table(tb, descs, nbox, 0, ns, tiles, tiles_cap, tiles_cap);
    }

    if (mirrored) be.sync();   // the one synchronisation
    else be.download(hsum.data(), sum, sizeof(uint64_t) * hsum.size());
    if (listed && hsum[SUM_NLISTED] > BE::PLAN_LIST_CAP) {
        // more busy lanes than the list holds: nothing was emitted, so plan again without the list
        be.free(sum); be.free(raw); be.free(recs); be.free(sorted); be.free(rperm); be.free(gs); be.free(gr);
        be.free(descs); be.free(ntl); be.free(tb); be.free(tiles); be.free(pcount);
        build_plan(be, ca, cb, rank, tile_bytes, xpose_shape, small_limit, routes_only, through_buffers, tile_hint, box_hint, p, false,
                   pair_work_log2);
        return;
    }
    int64_t n = (int64_t)hsum[SUM_NBOXES];
    if (n >= (int64_t)1 << 31) throw Error{ VPS_ERR_OOM, "more than 2^31 boxes" };
    p.nboxes = n;

    if (n > ns) {
        // ---- more boxes than the counting path takes: sort them (a stable radix sort by lo
        // corner, then by (owner, peer, kind order, tensor)), positions by scans
        be.free(sorted); be.free(rperm); be.free(gs); be.free(gr); be.free(descs); be.free(ntl); be.free(tb);
        be.free(tiles);
        tiles = nullptr; tiles_cap = 0;
        if (n > cap) {
            be.free(raw); be.free(recs);
            cap = n;
            raw = be.template alloc<vps_box>(cap);
            recs = be.template alloc<OrderRec>(cap);
            be.zero(sum, sizeof(uint64_t) * (size_t)SL.words());
            if (pcount) be.zero(pcount, sizeof(uint64_t) * (size_t)(3 * np));
            emit(lane_list);
        } else {
            be.zero(sum + 1, sizeof(uint64_t) * (size_t)(SL.words() - 1));
        }
        // ---- all ranks: order pair by pair.  Both orders keep the boxes of a (source, destination)
        // pair together, in the same order inside; so the boxes are counted and scattered into one
        // bucket per pair, ranked inside their bucket by counting, and the places of the buckets
        // in the two orders and in the peer buffers come from sums over the rows and the columns
        // of the pair matrix.  No sort; the work is the sum of the squared bucket sizes, and when
        // that is out of proportion (or the matrix too large) the radix path below takes over.
        bool ordered = false;
        const uint64_t pair_work_max = pair_work_log2 > 0 ? (uint64_t)1 << pair_work_log2 : 0;
        if (pair_path) {
            const bool counted_already = pcount != nullptr;
            if (!pcount) pcount = be.template alloc<uint64_t>(4 * np);  // boxes per pair
            uint64_t* pbytes = pcount + np;                               // buffer bytes per pair
            uint64_t* pcur = pbytes + np;                                 // scatter cursors
            uint64_t* pstart_s = pcur + np;                               // first place of the pair in the send order
            uint64_t* pstart_r = be.template alloc<uint64_t>(3 * np);   // ... in the receive order
            uint64_t* poff_s = pstart_r + np;                             // offset of the pair's segment in the send buffer
            uint64_t* poff_r = poff_s + np;                               // ... in the receive buffer
            int64_t* edge = be.template alloc<int64_t>(8 * ((int64_t)W + 1));
            int64_t* rows_n = edge, *cols_n = edge + (W + 1), *rows_b = edge + 2 * (W + 1), *cols_b = edge + 3 * (W + 1);
            int64_t* rows_n0 = edge + 4 * (W + 1), *cols_n0 = edge + 5 * (W + 1), *rows_b0 = edge + 6 * (W + 1), *cols_b0 = edge + 7 * (W + 1);
            PairRec* bucket = be.template alloc<PairRec>(n);
            uint64_t* work = sum + SUM_PAIR_WORK;
            be.zero(edge, sizeof(int64_t) * (size_t)(4 * (W + 1)));
            if (!counted_already) {
                be.zero(pcount, sizeof(uint64_t) * (size_t)(3 * np));
                be.for_each(step::plan_pair_counts(), n, [=] VPS_LAMBDA(int64_t k) {
                    const vps_box& b = raw[k];
                    const int64_t pr = (int64_t)b.src_rank * WB + b.dst_rank;
                    be_atomic_add_runs(pcount, pr, 1);
                    const uint64_t bf = recs[k].bytes_flags;
                    be_atomic_add_runs(pbytes, pr, (bf & ORD_SENDS) ? (bf & ~(uint64_t)15) : 0);
                });
            }
            // sums of the rows (one source rank each) and of the columns (one destination rank each)
            be.for_each(step::plan_pair_sums(), (int64_t)WA + WB, [=] VPS_LAMBDA(int64_t i) {
                uint64_t cn = 0, cb = 0, sq = 0;
                if (i < WA) {
                    VPS_UNROLL(8)
                    for (int64_t d = 0; d < WB; ++d) { const uint64_t c = pcount[i * WB + d]; cn += c; cb += pbytes[i * WB + d]; sq += c * c; }
                    rows_n[i] = (int64_t)cn; rows_b[i] = (int64_t)cb;
                    if (sq) be_atomic_add(work, sq);
                    // the statistics by kind of box fall out of the row: what a rank sends to itself
                    // is retained, everything else is sent by it and received by a resident rank
                    // (three counters in one memory line, bumped once per wavefront of boxes, were
                    // the longest wait of the pass over the boxes)
                    const uint64_t own = (!through_buffers && i < WB) ? pcount[i * WB + i] : 0;
                    if (own) be_atomic_add(sum + SUM_NRETAIN, own);
                    if (cn - own) { be_atomic_add(sum + SUM_NSEND, cn - own); be_atomic_add(sum + SUM_NRECV, cn - own); }
                } else {
                    const int64_t d = i - WA;
                    VPS_UNROLL(8)
                    for (int64_t r = 0; r < WA; ++r) { cn += pcount[r * WB + d]; cb += pbytes[r * WB + d]; }
                    cols_n[d] = (int64_t)cn; cols_b[d] = (int64_t)cb;
                }
            });
            be.exclusive_scan_rows(edge, edge + 4 * (W + 1), W, W + 1, 4);   // rows_n0, cols_n0, rows_b0, cols_b0
            if (W <= 256) {
                // one lane per pair: it adds up its row to the left of it and its column above it
                be.for_each(step::plan_pair_starts(), np, [=] VPS_LAMBDA(int64_t pr) {
                    const int64_t i = pr / WB, d = pr - i * WB;
                    uint64_t at = (uint64_t)rows_n0[i], off = 0;
                    VPS_UNROLL(8)
                    for (int64_t q = 0; q < d; ++q) { at += pcount[i * WB + q]; off += pbytes[i * WB + q]; }
                    pstart_s[pr] = at; poff_s[pr] = off;
                    at = (uint64_t)cols_n0[d]; off = 0;
                    VPS_UNROLL(8)
                    for (int64_t q = 0; q < i; ++q) { at += pcount[q * WB + d]; off += pbytes[q * WB + d]; }
                    pstart_r[pr] = at; poff_r[pr] = off;
                });
            } else {
                be.for_each(step::plan_pair_starts(), (int64_t)WA + WB, [=] VPS_LAMBDA(int64_t i) {
                    if (i < WA) {
                        uint64_t at = (uint64_t)rows_n0[i], off = 0;
                        VPS_UNROLL(8)
                        for (int64_t d = 0; d < WB; ++d) { pstart_s[i * WB + d] = at; poff_s[i * WB + d] = off; at += pcount[i * WB + d]; off += pbytes[i * WB + d]; }
                    } else {
                        const int64_t d = i - WA;
                        uint64_t at = (uint64_t)cols_n0[d], off = 0;
                        VPS_UNROLL(8)
                        for (int64_t r = 0; r < WA; ++r) { pstart_r[r * WB + d] = at; poff_r[r * WB + d] = off; at += pcount[r * WB + d]; off += pbytes[r * WB + d]; }
                    }
                });
            }
            be.for_each(step::plan_pair_scatter(), n, [=] VPS_LAMBDA(int64_t k) {
                const vps_box& b = raw[k];
                const int64_t pr = (int64_t)b.src_rank * WB + b.dst_rank;
                const OrderRec r = recs[k];
                PairRec q;
                q.key = pair_rec_key(r, pr); q.klo = r.klo; q.bytes_flags = r.bytes_flags; q.box = (uint64_t)k;
                bucket[pstart_s[pr] + be_atomic_fetch_add(&pcur[pr], 1)] = q;
            });
            sorted = be.template alloc<vps_box>(n);
            rperm = be.template alloc<uint32_t>(n);
            gs = be.template alloc<uint64_t>(n + 1);
            gr = be.template alloc<uint64_t>(n + 1);
            uint64_t* before_of = be.template alloc<uint64_t>(2 * n);
            uint64_t* bytes_of = before_of + n;
            be.pair_rank_each(step::plan_pair_rank(), bucket, pstart_s, pcount, n, work, pair_work_max,
                              [=] VPS_LAMBDA(int64_t j, uint64_t before, uint64_t bytes) { before_of[j] = before; bytes_of[j] = bytes; });
            be.for_each(step::plan_pair_place(), n, [=] VPS_LAMBDA(int64_t j) {
                const PairRec me = bucket[j];
                const int64_t pr = (int64_t)(me.key >> 26);
                const uint64_t before = before_of[j], bytes = bytes_of[j];
                const vps_box* in = raw + me.box;
                const uint64_t is = pstart_s[pr] + before, ir = pstart_r[pr] + before;
                const uint64_t ps = poff_s[pr] + bytes, pq = poff_r[pr] + bytes;
                // (copied as it is, then the two positions: a box changed in a local copy and
                // stored whole would pass through scratch memory)
                vps_box* out = sorted + is;
                *out = *in;
                if (me.bytes_flags & ORD_SENDS) out->send_pos = ps;
                if (me.bytes_flags & ORD_RECEIVES) out->recv_pos = pq;
                rperm[ir] = (uint32_t)is;
                gs[is] = (uint64_t)rows_b0[in->src_rank] + ps;
                gr[ir] = (uint64_t)cols_b0[in->dst_rank] + pq;
                if (j == 0) { gs[n] = (uint64_t)rows_b0[W]; gr[n] = (uint64_t)cols_b0[W]; }
            });
            be.free(before_of);
            be.free(pcount); be.free(pstart_r); be.free(edge); be.free(bucket);
            pcount = nullptr;
            ordered = true;
        }
        const bool pair_ordered = ordered;
        fc.count_kinds = !pair_ordered;
        if (!ordered) {
            uint64_t* kmin = be.template alloc<uint64_t>(n);
            uint64_t* kmaj = be.template alloc<uint64_t>(n);
            uint32_t* by_lo = be.template alloc<uint32_t>(n);
            uint32_t* ord_s = be.template alloc<uint32_t>(n);
            uint32_t* ord_r = be.template alloc<uint32_t>(n);
            const int lo_bits = bits_for(ca.tensor_numel_max);
            be.for_each(step::plan_keys(), n, [=] VPS_LAMBDA(int64_t k) { kmin[k] = recs[k].klo; by_lo[k] = (uint32_t)k; });
            be.sort_pairs(kmin, by_lo, n, lo_bits);
            // (keys cut to the bits this transition needs: every bit less is work the sort does not do)
            const int rank_bits = bits_for((uint64_t)W), tensor_bits = bits_for((uint64_t)A.nt);
            const int major_bits = 2 * rank_bits + 2 + tensor_bits;
            be.for_each(step::plan_key_send(), n, [=] VPS_LAMBDA(int64_t k) {
                ord_s[k] = by_lo[k];
                kmaj[k] = compact_major_key(recs[by_lo[k]].key_s, rank_bits, tensor_bits);
            });
            be.sort_pairs(kmaj, ord_s, n, major_bits);
            be.for_each(step::plan_key_recv(), n, [=] VPS_LAMBDA(int64_t k) {
                ord_r[k] = by_lo[k];
                kmaj[k] = compact_major_key(recs[by_lo[k]].key_r, rank_bits, tensor_bits);
            });
            be.sort_pairs(kmaj, ord_r, n, major_bits);
            be.free(kmin); be.free(kmaj); be.free(by_lo);
            int64_t* sz = be.template alloc<int64_t>(n + 1);
            gs = be.template alloc<uint64_t>(n + 1);
            gr = be.template alloc<uint64_t>(n + 1);
            for (int side = 0; side < 2; ++side) {
                const uint32_t* ord = side == 0 ? ord_s : ord_r;
                uint64_t* g = side == 0 ? gs : gr;
                be.for_each(step::plan_slot_sizes(), n + 1, [=] VPS_LAMBDA(int64_t k) {
                    if (k == n) { sz[k] = 0; return; }
                    const uint64_t bf = recs[ord[k]].bytes_flags;
                    sz[k] = (bf & (side == 0 ? ORD_SENDS : ORD_RECEIVES)) ? (int64_t)(bf & ~(uint64_t)15) : 0;
                });
                be.exclusive_scan(sz, (int64_t*)g, n);
                // position inside the owner's buffer: cumulative bytes minus those of the ranks before
                be.for_each(step::plan_positions(), n, [=] VPS_LAMBDA(int64_t k) {
                    vps_box& b = raw[ord[k]];
                    if (!(recs[ord[k]].bytes_flags & (side == 0 ? ORD_SENDS : ORD_RECEIVES))) return;
                    const int32_t own = side == 0 ? b.src_rank : b.dst_rank;
                    int64_t lo = 0, hi = k;   // first box of the owner in this order
                    while (lo < hi) {
                        const int64_t mid = (lo + hi) / 2;
                        const vps_box& m = raw[ord[mid]];
                        if ((side == 0 ? m.src_rank : m.dst_rank) < own) lo = mid + 1; else hi = mid;
                    }
                    const uint64_t rel = g[k] - g[lo];
                    if (side == 0) b.send_pos = rel; else b.recv_pos = rel;
                });
            }
            be.free(sz);
            sorted = be.template alloc<vps_box>(n);
            rperm = be.template alloc<uint32_t>(n);
            uint32_t* inv = be.template alloc<uint32_t>(n);
            be.for_each(step::plan_sorted_boxes(), n, [=] VPS_LAMBDA(int64_t k) { sorted[k] = raw[ord_s[k]]; inv[ord_s[k]] = (uint32_t)k; });
            be.for_each(step::plan_recv_perm(), n, [=] VPS_LAMBDA(int64_t k) { rperm[k] = inv[ord_r[k]]; });
            be.free(inv); be.free(ord_s); be.free(ord_r);
        }
        descs = routes_only ? nullptr : be.template alloc<CopyDesc>(3 * n);
        ntl = be.template alloc<int64_t>(3 * n + 1);
        tb = be.template alloc<int64_t>(3 * n + 1);
        fc.descs = descs; fc.ntiles = ntl;
        // Every rank's first box in the two orders: position k is the first box of the ranks
        // after its predecessor's up to its own (boxes ascend by rank in either order; k = n
        // closes the tables).  One lane per position instead of a search per rank, whose
        // dependent loads would take longer than all positions together.
        auto first_boxes_at = [=] VPS_LAMBDA(int64_t k) {
            const int32_t ps = k ? sorted[k - 1].src_rank : -1, cs = k < n ? sorted[k].src_rank : W;
            for (int32_t r = ps + 1; r <= cs; ++r) rt[0 * (W + 1) + r] = k;
            const int32_t pd = k ? sorted[rperm[k - 1]].dst_rank : -1, cd = k < n ? sorted[rperm[k]].dst_rank : W;
            for (int32_t r = pd + 1; r <= cd; ++r) rt[1 * (W + 1) + r] = k;
        };
        if (routes_only) {
            // no copy descriptors, no tiles: statistics and first boxes only
            be.zero(tb, sizeof(int64_t) * (size_t)(3 * n + 1));
            be.for_each(step::plan_copy_descs(), n + 1, [=] VPS_LAMBDA(int64_t k) {
                if (k < n) account_box(fc, sorted[k]);
                first_boxes_at(k);
            });
        } else {
            be.for_each(step::plan_copy_descs(), 3 * n + 1, [=] VPS_LAMBDA(int64_t i) {
                if (i == 3 * n) { ntl[i] = 0; first_boxes_at(n); return; }
                const int op = (int)(i / n);
                const int64_t k = i - op * n;
                const vps_box& b = sorted[op == OP_UNPACK ? rperm[k] : k];
                if (op == OP_RETAIN) { account_box(fc, b); first_boxes_at(k); }
                describe_box_op(fc, b, op, i);
            });
            be.exclusive_scan(ntl, tb, 3 * n);
        }
        be.for_each(step::plan_rank_tables(), W + 1, [=] VPS_LAMBDA(int64_t r) { rank_row(r, n, gs, gr, tb); });
        be.download(hsum.data(), sum, sizeof(uint64_t) * hsum.size());
        if ((int64_t)hsum[SUM_NBOXES] != n) throw Error{ VPS_ERR_HIP, "planning passes disagree on the number of boxes" };
        if (pair_ordered && hsum[SUM_PAIR_WORK] > pair_work_max) {
            // a few pairs hold nearly all boxes: the ranking inside the buckets was skipped, so
            // plan again with the radix sort
            be.free(sum); be.free(raw); be.free(recs); be.free(sorted); be.free(rperm); be.free(gs); be.free(gr);
            be.free(descs); be.free(ntl); be.free(tb);
            build_plan(be, ca, cb, rank, tile_bytes, xpose_shape, small_limit, routes_only, through_buffers, tile_hint, box_hint, p,
                       lane_list, 0);
            return;
        }
    }
    be.free(raw); be.free(recs); be.free(gs); be.free(gr); be.free(ntl);
    be.free(pcount);   // (counted for nothing when the plan turned out small)

    // (5) the host's view of the plan
    {
        const int64_t* rt = (const int64_t*)(hsum.data() + SL.rank_tables());
        auto col = [&](int c, std::vector<int64_t>& v) { v.assign(rt + c * (W + 1), rt + (c + 1) * (W + 1)); };
        std::vector<int64_t> sb, rb;
        col(0, p.first_send); col(1, p.first_recv); col(2, sb); col(3, rb);
        p.send_base.assign(sb.begin(), sb.end());
        p.recv_base.assign(rb.begin(), rb.end());
        for (int op = 0; op < 3; ++op) col(4 + op, p.op_tile[op]);
        p.pair_bytes.assign(hsum.begin() + SL.pairs(), hsum.begin() + SL.pairs() + SL.npairs);
        const uint8_t* hu = (const uint8_t*)(hsum.data() + SL.used());
        for (int op = 0; op < 3; ++op) p.used[op].assign(hu + op * nslots, hu + (op + 1) * nslots);
    }
    const int64_t ntiles = routes_only ? 0 : p.op_tile[OP_UNPACK][(size_t)W];
    if (ntiles >= (int64_t)1 << 31) throw Error{ VPS_ERR_OOM, "more than 2^31 tiles" };
    p.d_boxes = sorted;
    p.d_recv_perm = rperm;
    p.descs = descs;
    p.d_tile_base = tb;
    p.host_boxes_ready = false;
    be.free(sum);

    // (6) the tile table, unless the hinted one above already holds it
    if (!routes_only && ntiles > tiles_cap) {
        be.free(tiles);
        tiles = be.template alloc<TileRef>(ntiles);
        be.tile_table(tb, descs, nullptr, n, 0, tiles, ntiles, ntiles);
        be.sync();
    }
    p.tiles = tiles;
    if (layout.all_ranks) p.ptr_table = be.template alloc<void*>(num_slots(layout));

    vps_plan_stats_t& st = p.stats;
    st = vps_plan_stats_t();
    st.num_boxes = n;
    st.num_retain_boxes = (int64_t)hsum[SUM_NRETAIN];
    st.num_send_boxes = (int64_t)hsum[SUM_NSEND];
    st.num_recv_boxes = (int64_t)hsum[SUM_NRECV];
    if (rank >= 0)
        for (int32_t q = 0; q < W; ++q) {
            if (q == rank && !through_buffers) continue;
            if (q < WB && p.pair_bytes[(size_t)WA + (size_t)q]) st.num_peers_out++;
            if (q < WA && p.pair_bytes[(size_t)q]) st.num_peers_in++;
        }
    st.num_retain_tiles = p.op_tile[0][(size_t)W] - p.op_tile[0][0];
    st.num_pack_tiles = p.op_tile[1][(size_t)W] - p.op_tile[1][0];
    st.num_unpack_tiles = p.op_tile[2][(size_t)W] - p.op_tile[2][0];
    st.plan_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count();
}

// The host copies of the boxes and of the tile bases, fetched on first use.
template <class BE>
void ensure_host_boxes(BE& be, PlanData& p)
{
    if (p.host_boxes_ready) return;
    p.boxes_send_order.resize((size_t)p.nboxes);
    p.recv_perm.resize((size_t)p.nboxes);
    p.tile_base.assign((size_t)(3 * p.nboxes + 1), 0);
    be.download_later(p.boxes_send_order.data(), p.d_boxes, sizeof(vps_box) * (size_t)p.nboxes);
    be.download_later(p.recv_perm.data(), p.d_recv_perm, sizeof(uint32_t) * (size_t)p.nboxes);
    if (!p.routes_only)
        be.download_later(p.tile_base.data(), p.d_tile_base, sizeof(int64_t) * (size_t)(3 * p.nboxes + 1));
    be.sync();
    p.host_boxes_ready = true;
}

// Payload bytes src -> dst known to the plan (0 for pairs outside a single-rank plan).
inline uint64_t plan_pair_bytes(const PlanData& p, int32_t src, int32_t dst)
{
    if (src < 0 || dst < 0 || src >= p.A.world || dst >= p.B.world) return 0;
    if (p.rank < 0) return p.pair_bytes[(size_t)src * (size_t)p.B.world + (size_t)dst];
    if (dst == p.rank) return p.pair_bytes[(size_t)src];
    if (src == p.rank) return p.pair_bytes[(size_t)p.A.world + (size_t)dst];
    return 0;
}

// Tile range [begin, end) of operation `op` for `rank` (-1: every rank).
inline void plan_tile_range(const PlanData& p, int op, int32_t rank, int64_t& begin, int64_t& end)
{
    const std::vector<int64_t>& t = p.op_tile[op];
    begin = rank < 0 ? t.front() : t[(size_t)rank];
    end = rank < 0 ? t.back() : t[(size_t)rank + 1];
}

// ------------------------------------------------------------------- staged XOR exchange

// DynaTrain Algorithm 1 (MemoryAwareChunk and the step loop) for resident virtual ranks: the
// XOR steps are grouped into stages whose per-rank buffers fit a budget; every stage packs,
// exchanges (send segment -> peer's receive segment, a device copy here) and unpacks, reusing
// one scratch area.
struct StageData {
    int32_t nsteps = 0, nstages = 0;
    std::vector<int32_t> stage_of_step;   // [nsteps + 1], -1 = no traffic in that step
    std::vector<uint64_t> step_cost;      // [nsteps + 1], max over ranks of send + receive bytes
    std::vector<uint64_t> send_base, recv_base;  // [stage][rank]: region offsets in scratch
    std::vector<uint64_t> stage_scratch;  // [stage]
    uint64_t scratch_needed = 0;
    std::vector<int64_t> pack_begin, exch_begin, unpack_begin;  // [stage + 1] tile ranges
    // backend memory
    CopyDesc* descs = nullptr;   // 2n: pack and unpack descriptors with per-stage positions
    TileRef* tiles = nullptr;    // [pack by stage | exchange by stage | unpack by stage]
    void** ptr_table = nullptr;
    int64_t n = 0;
};

template <class BE>
void free_stage(BE& be, StageData& sd)
{
    be.free(sd.descs); be.free(sd.tiles); be.free(sd.ptr_table);
    sd.descs = nullptr; sd.tiles = nullptr; sd.ptr_table = nullptr;
}

// The greedy of Algorithm 1 (MemoryAwareChunk) over steps 1..nsteps: a step joins the current
// stage unless that would exceed the budget; steps without traffic belong to no stage, and no
// empty stage is emitted (a step that alone exceeds the budget becomes a stage of its own).
inline int32_t chunk_steps(const std::vector<uint64_t>& cost, uint64_t budget, std::vector<int32_t>& stage_of_step)
{
    const int32_t nsteps = (int32_t)cost.size() - 1;
    stage_of_step.assign(cost.size(), -1);
    int32_t nstages = 0;
    uint64_t cur = 0;
    bool open = false;
    for (int32_t s = 1; s <= nsteps; ++s) {
        if (cost[(size_t)s] == 0) continue;
        if (open && cur + cost[(size_t)s] > budget) { ++nstages; cur = 0; open = false; }
        stage_of_step[(size_t)s] = nstages;
        cur += cost[(size_t)s];
        open = true;
    }
    if (open) ++nstages;
    return nstages;
}

template <class BE>
void build_stage_plan(BE& be, const PlanData& p, uint64_t budget, uint32_t tile_bytes, StageData& sd)
{
    if (!p.layout.all_ranks) throw Error{ VPS_ERR_INVALID_ARG, "staged exchange needs an all-ranks plan" };
    if (p.routes_only) throw Error{ VPS_ERR_INVALID_ARG, "staged exchange needs a plan with copy tables" };
    if (p.through_buffers) throw Error{ VPS_ERR_INVALID_ARG, "staged exchange does not take a plan in which a rank is its own peer" };
    const int32_t WA = p.A.world, WB = p.B.world, W = WA > WB ? WA : WB;
    const int64_t n = p.nboxes;
    sd.n = n;
    const size_t npair = (size_t)WA * (size_t)WB;
    // (1) peer segments from the host copy of the boxes (sorted by source, destination)
    std::vector<uint64_t> seg_bytes(npair, 0), seg_send(npair, 0), seg_recv(npair, 0);
    for (const vps_box& b : p.boxes_send_order) {
        if (b.src_rank == b.dst_rank) continue;
        const size_t pr = (size_t)b.src_rank * (size_t)WB + (size_t)b.dst_rank;
        if (seg_bytes[pr] == 0) { seg_send[pr] = b.send_pos; seg_recv[pr] = b.recv_pos; }
        seg_bytes[pr] = b.send_pos + box_slot_bytes(b) - seg_send[pr];
    }
    // (2) XOR steps: in step s rank i is paired with i ^ s
    int32_t pow2 = 1;
    while (pow2 < W) pow2 <<= 1;
    sd.nsteps = pow2 - 1;
    sd.step_cost.assign((size_t)sd.nsteps + 1, 0);
    auto seg = [&](int32_t i, int32_t j) -> uint64_t { return (i < WA && j < WB) ? seg_bytes[(size_t)i * (size_t)WB + (size_t)j] : 0; };
    for (int32_t s = 1; s <= sd.nsteps; ++s)
        for (int32_t r = 0; r < W; ++r) {
            const uint64_t c = seg(r, r ^ s) + seg(r ^ s, r);
            if (c > sd.step_cost[(size_t)s]) sd.step_cost[(size_t)s] = c;
        }
    sd.nstages = chunk_steps(sd.step_cost, budget, sd.stage_of_step);
    const int32_t G = sd.nstages;
    // (3) per stage: regions of every rank and positions of every segment inside them
    std::vector<int32_t> stage_of_pair(npair, -1);
    std::vector<int64_t> delta_send(npair, 0), delta_recv(npair, 0);
    std::vector<uint64_t> st_send_off(npair, 0), st_recv_off(npair, 0);
    sd.send_base.assign((size_t)G * (size_t)WA, 0);
    sd.recv_base.assign((size_t)G * (size_t)WB, 0);
    sd.stage_scratch.assign((size_t)G, 0);
    for (int32_t g = 0; g < G; ++g) {
        uint64_t off = 0;
        for (int32_t i = 0; i < WA; ++i) {   // send regions, peers ascending inside
            sd.send_base[(size_t)g * (size_t)WA + (size_t)i] = off;
            uint64_t in = 0;
            for (int32_t j = 0; j < WB; ++j) {
                const int32_t s = i ^ j;
                const size_t pr = (size_t)i * (size_t)WB + (size_t)j;
                if (s == 0 || s > sd.nsteps || sd.stage_of_step[(size_t)s] != g || !seg_bytes[pr]) continue;
                stage_of_pair[pr] = g;
                st_send_off[pr] = in;
                delta_send[pr] = (int64_t)in - (int64_t)seg_send[pr];
                in += seg_bytes[pr];
            }
            off += (in + 255) & ~255ull;
        }
        for (int32_t j = 0; j < WB; ++j) {   // receive regions, sources ascending inside
            sd.recv_base[(size_t)g * (size_t)WB + (size_t)j] = off;
            uint64_t in = 0;
            for (int32_t i = 0; i < WA; ++i) {
                const size_t pr = (size_t)i * (size_t)WB + (size_t)j;
                if (stage_of_pair[pr] != g) continue;
                st_recv_off[pr] = in;
                delta_recv[pr] = (int64_t)in - (int64_t)seg_recv[pr];
                in += seg_bytes[pr];
            }
            off += (in + 255) & ~255ull;
        }
        sd.stage_scratch[(size_t)g] = off;
        if (off > sd.scratch_needed) sd.scratch_needed = off;
    }
    // (4) device: descriptors with stage positions, tiles regrouped by stage
    std::vector<int32_t> pair_send((size_t)n), pair_recv((size_t)n);
    for (int64_t k = 0; k < n; ++k) {
        const vps_box& b = p.boxes_send_order[(size_t)k];
        pair_send[(size_t)k] = b.src_rank * WB + b.dst_rank;
    }
    for (int64_t k = 0; k < n; ++k) pair_recv[(size_t)k] = pair_send[(size_t)p.recv_perm[(size_t)k]];
    int32_t* d_pair = be.template alloc<int32_t>(2 * n);       // pair of pack desc k, unpack desc k
    int32_t* d_stage = be.template alloc<int32_t>((int64_t)npair);
    int64_t* d_dsend = be.template alloc<int64_t>((int64_t)npair);
    int64_t* d_drecv = be.template alloc<int64_t>((int64_t)npair);
    be.upload(d_pair, pair_send.data(), sizeof(int32_t) * (size_t)n);
    be.upload(d_pair + n, pair_recv.data(), sizeof(int32_t) * (size_t)n);
    be.upload(d_stage, stage_of_pair.data(), sizeof(int32_t) * npair);
    be.upload(d_dsend, delta_send.data(), sizeof(int64_t) * npair);
    be.upload(d_drecv, delta_recv.data(), sizeof(int64_t) * npair);
    sd.descs = be.template alloc<CopyDesc>(2 * n);
    {
        CopyDesc* out = sd.descs;
        const CopyDesc* in = p.descs + n;   // the plan's pack and unpack descriptors
        be.for_each(step::stage_descs(), 2 * n, [=] VPS_LAMBDA(int64_t i) {
            CopyDesc d = in[i];
            if (d.ntiles) {
                const int32_t pr = d_pair[i];
                if (i < n) d.dst_byte = (uint64_t)((int64_t)d.dst_byte + d_dsend[pr]);
                else { d.src_byte = (uint64_t)((int64_t)d.src_byte + d_drecv[pr]); d.alt_src_slot = -1; }
            }
            out[i] = d;
        });
    }
    // pack and unpack tiles of the plan, keyed by stage (stable sort keeps their order)
    const int64_t t_pack0 = p.tile_base[(size_t)n], t_unpack0 = p.tile_base[(size_t)(2 * n)], t_end = p.tile_base[(size_t)(3 * n)];
    const int64_t nmove = t_end - t_pack0;
    int64_t* tb = be.template alloc<int64_t>(3 * n + 1);
    be.upload(tb, p.tile_base.data(), sizeof(int64_t) * (size_t)(3 * n + 1));
    uint64_t* key = be.template alloc<uint64_t>(nmove);
    uint32_t* idx = be.template alloc<uint32_t>(nmove);
    be.for_each(step::stage_tile_keys(), nmove, [=] VPS_LAMBDA(int64_t k) {
        const int64_t t = t_pack0 + k;
        const int64_t d = upper_bound_idx(tb, 3 * n + 1, t) - 1;   // descriptor index in [n, 3n)
        const uint64_t op = d < 2 * n ? 0 : 1;
        key[k] = op << 32 | (uint32_t)d_stage[d_pair[d - n]];
        idx[k] = (uint32_t)k;
    });
    be.sort_pairs(key, idx, nmove, 33);
    // exchange tiles: every segment cut into tile_bytes pieces, stages ascending
    std::vector<int64_t> seg_tile_base;
    std::vector<uint64_t> seg_src, seg_dst, seg_len;
    sd.exch_begin.assign((size_t)G + 1, 0);
    int64_t nexch = 0;
    for (int32_t g = 0; g < G; ++g) {
        sd.exch_begin[(size_t)g] = nexch;
        for (int32_t i = 0; i < WA; ++i)
            for (int32_t j = 0; j < WB; ++j) {
                const size_t pr = (size_t)i * (size_t)WB + (size_t)j;
                if (stage_of_pair[pr] != g) continue;
                seg_tile_base.push_back(nexch);
                seg_src.push_back(tile_pack_addr(slot_send(p.layout, i), st_send_off[pr]));
                seg_dst.push_back(tile_pack_addr(slot_recv(p.layout, j), st_recv_off[pr]));
                seg_len.push_back(seg_bytes[pr]);
                nexch += (int64_t)((seg_bytes[pr] + tile_bytes - 1) / tile_bytes);
            }
    }
    sd.exch_begin[(size_t)G] = nexch;
    seg_tile_base.push_back(nexch);
    const int64_t nseg = (int64_t)seg_len.size();
    int64_t* d_stb = be.template alloc<int64_t>(nseg + 1);
    uint64_t* d_ssrc = be.template alloc<uint64_t>(nseg);
    uint64_t* d_sdst = be.template alloc<uint64_t>(nseg);
    uint64_t* d_slen = be.template alloc<uint64_t>(nseg);
    be.upload(d_stb, seg_tile_base.data(), sizeof(int64_t) * (size_t)(nseg + 1));
    be.upload(d_ssrc, seg_src.data(), sizeof(uint64_t) * (size_t)nseg);
    be.upload(d_sdst, seg_dst.data(), sizeof(uint64_t) * (size_t)nseg);
    be.upload(d_slen, seg_len.data(), sizeof(uint64_t) * (size_t)nseg);
    if (nmove + nexch >= (int64_t)1 << 31) throw Error{ VPS_ERR_OOM, "more than 2^31 tiles" };
    sd.tiles = be.template alloc<TileRef>(nmove + nexch);
    {
        // layout of the new table: [pack tiles by stage | exchange tiles by stage | unpack tiles by stage]
        const int64_t npack = t_unpack0 - t_pack0;
        TileRef* out = sd.tiles;
        const CopyDesc* sdescs = sd.descs;
        be.for_each(step::stage_tile_gather(), nmove, [=] VPS_LAMBDA(int64_t k) {
            const int64_t t = t_pack0 + idx[k];
            const int64_t d = upper_bound_idx(tb, 3 * n + 1, t) - 1;
            // rebuilt from the stage descriptor: same geometry, stage positions
            out[k < npack ? k : k + nexch] = make_tile(sdescs[d - n], (uint32_t)(d - n), (uint32_t)(t - tb[d]));
        });
        be.for_each(step::stage_exchange_tiles(), nexch, [=] VPS_LAMBDA(int64_t t) {
            const int64_t sg = upper_bound_idx(d_stb, nseg + 1, t) - 1;
            const uint64_t o = (uint64_t)(t - d_stb[sg]) * tile_bytes;
            TileRef r;
            r.src = d_ssrc[sg] + o;
            r.dst = d_sdst[sg] + o;
            r.alt_src = VPS_TILE_NO_ALT;
            r.src_pitch = 0; r.dst_pitch = 0;
            r.nbytes = (uint32_t)(d_slen[sg] - o < tile_bytes ? d_slen[sg] - o : tile_bytes);
            r.nruns_flags = 1u << 8;
            out[npack + t] = r;
        });
    }
    // per-stage tile ranges of pack and unpack from the sorted keys
    sd.pack_begin.assign((size_t)G + 1, 0);
    sd.unpack_begin.assign((size_t)G + 1, 0);
    {
        int64_t* bounds = be.template alloc<int64_t>(2 * ((int64_t)G + 1));
        be.for_each(step::stage_bounds(), 2 * ((int64_t)G + 1), [=] VPS_LAMBDA(int64_t i) {
            const uint64_t op = i > G ? 1 : 0, g = (uint64_t)(i > G ? i - (G + 1) : i);
            bounds[i] = lower_bound_idx(key, nmove, op << 32 | g);
        });
        std::vector<int64_t> hb(2 * ((size_t)G + 1));
        be.download(hb.data(), bounds, sizeof(int64_t) * hb.size());
        be.free(bounds);
        const int64_t npack = t_unpack0 - t_pack0;
        for (int32_t g = 0; g <= G; ++g) {
            sd.pack_begin[(size_t)g] = hb[(size_t)g] < npack ? hb[(size_t)g] : npack;
            sd.unpack_begin[(size_t)g] = hb[(size_t)G + 1 + (size_t)g] + nexch;
            sd.exch_begin[(size_t)g] += npack;
        }
    }
    sd.ptr_table = be.template alloc<void*>(num_slots(p.layout));
    be.free(d_pair); be.free(d_stage); be.free(d_dsend); be.free(d_drecv); be.free(tb); be.free(key); be.free(idx);
    be.free(d_stb); be.free(d_ssrc); be.free(d_sdst); be.free(d_slen);
    be.sync();
}

// --------------------------------------------------------------------- collective intent

// Algorithm 1 (OptimizePrimitives, GroupByLogicalTensor ... Broadcast / Scatter / Gather): the
// boxes that leave their rank are grouped by (tensor, kind); a group with one source, several
// destinations and identical slices is a broadcast; with one source, several destinations and
// slices that tile one contiguous range of the flattened tensor a scatter; with several
// sources, one destination and such slices a gather; anything else stays point-to-point.
// classes[tensor*4 + kind] receives the COLL_* code.
template <class BE>
void classify_collectives(BE& be, const PlanData& p, const ConfigData& ca, std::vector<int32_t>& classes)
{
    const int64_t n = p.nboxes;
    const int32_t ngroups = p.A.nt * 4;
    classes.assign((size_t)ngroups, COLL_NONE);
    const vps_box* boxes = p.d_boxes;
    uint64_t* key = be.template alloc<uint64_t>(n);
    uint64_t* gk = be.template alloc<uint64_t>(n);
    uint32_t* ord = be.template alloc<uint32_t>(n);
    uint32_t* flags = be.template alloc<uint32_t>(ngroups);
    int32_t* out = be.template alloc<int32_t>(ngroups);
    be.zero(flags, sizeof(uint32_t) * (size_t)ngroups);
    const TensorRec* T = ca.T;
    // order: group, then first element of the slice
    be.for_each(step::coll_keys(), n, [=] VPS_LAMBDA(int64_t k) { key[k] = box_minor_key(boxes[k], T[boxes[k].tensor]); ord[k] = (uint32_t)k; });
    be.sort_pairs(key, ord, n);
    be.for_each(step::coll_group_key(), n, [=] VPS_LAMBDA(int64_t k) {
        const vps_box& b = boxes[ord[k]];
        gk[k] = b.src_rank == b.dst_rank ? ~0ull : (uint64_t)(b.tensor * 4 + b.kind);   // retained boxes last
    });
    be.sort_pairs(gk, ord, n);
    be.for_each(step::coll_flags(), n, [=] VPS_LAMBDA(int64_t k) {
        if (gk[k] == ~0ull) return;
        const vps_box& b = boxes[ord[k]];
        const TensorRec x = T[b.tensor];
        const int64_t g0 = lower_bound_idx(gk, n, gk[k]);
        const vps_box& f = boxes[ord[g0]];
        uint32_t fl = CF_ANY;
        if (b.src_rank != f.src_rank) fl |= CF_MULTI_SRC;
        if (b.dst_rank != f.dst_rank) fl |= CF_MULTI_DST;
        for (int a = 0; a < 4; ++a)
            if (b.lo[a] != f.lo[a] || b.ext[a] != f.ext[a]) fl |= CF_DIFFERENT;
        if (!box_is_linear_range(b, x)) fl |= CF_NONLINEAR;
        if (k > g0) {
            const vps_box& pv = boxes[ord[k - 1]];
            if (box_minor_key(pv, x) + box_volume(pv) != box_minor_key(b, x)) fl |= CF_GAP;
        }
        be_atomic_or(&flags[gk[k]], fl);
    });
    be.for_each(step::coll_classes(), ngroups, [=] VPS_LAMBDA(int64_t g) { out[g] = classify_flags(flags[g]); });
    be.download(classes.data(), out, sizeof(int32_t) * (size_t)ngroups);
    be.free(key); be.free(gk); be.free(ord); be.free(flags); be.free(out);
    be.sync();
}

}  // namespace vps

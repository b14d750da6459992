// vps_api_impl.h - the C entry points of include/vps.h, written over the backend interface.
// Included exactly once by a translation unit that defines VPS_BACKEND (the backend class) and
// VPS_FN(name) (the exported symbol name).  The product library uses the HIP backend and the
// names of include/vps.h.
#pragma once

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>

#include "vps_pipeline.h"

namespace vps {

static thread_local std::string g_last_error;

// Settings that apply to plans created afterwards (vps_set_option).  Plain atomics: a plan reads
// them once, when it is made.
static std::atomic<uint32_t> g_tile_bytes{ 8u << 10 };
static std::atomic<uint32_t> g_small_plan_boxes{ 8192u };   // boxes ordered by counting, without a sort
static std::atomic<uint32_t> g_pair_work_log2{ (uint32_t)PAIR_BUCKET_WORK_LOG2 };   // 0: all-ranks plans are always sorted
static std::atomic<uint32_t> g_xpose_shape{ 0u };           // 0 = chosen per box from the pitches

// Number of tiles and boxes of the plans made so far, by what determines them (model, both
// configurations, rank, flags, tile size).  A repeated transition then sizes its tables without
// waiting for the device.  Only sizes: every plan computes all of its tables anew.
struct TileHints {
    struct Sizes {
        int64_t tiles, boxes;
    };
    std::mutex m;
    std::unordered_map<uint64_t, Sizes> tiles;
    static uint64_t key(const vps_model_desc& model, const vps_parallel_desc& a, const vps_parallel_desc& b, int32_t rank,
                        uint32_t flags, uint32_t tile_bytes, uint32_t xpose_shape)
    {
        uint64_t h = 0xcbf29ce484222325ull;
        auto mix = [&](const void* p, size_t n) {
            for (size_t i = 0; i < n; ++i) h = (h ^ ((const unsigned char*)p)[i]) * 0x100000001b3ull;   // FNV-1a
        };
        mix(&model, sizeof model); mix(&a, sizeof a); mix(&b, sizeof b); mix(&rank, sizeof rank);
        mix(&flags, sizeof flags); mix(&tile_bytes, sizeof tile_bytes); mix(&xpose_shape, sizeof xpose_shape);
        return h;
    }
    Sizes get(uint64_t k)
    {
        std::lock_guard<std::mutex> g(m);
        auto it = tiles.find(k);
        return it == tiles.end() ? Sizes{ 0, 0 } : it->second;
    }
    void put(uint64_t k, Sizes n)
    {
        std::lock_guard<std::mutex> g(m);
        if (tiles.size() > 4096) tiles.clear();
        tiles[k] = n;
    }
};
static TileHints g_tile_hints;

inline int fail(int code, const std::string& msg)
{
    g_last_error = msg;
    return code;
}

}  // namespace vps

struct vps_config {
    vps::ConfigData d;
    std::mutex host_copy;   // guards the on-demand host copies (class table, piece table)
};

struct vps_plan {
    vps::PlanData d;
    std::mutex host_copy;   // guards the on-demand host copy of the boxes and the stream list
    std::vector<void*> streams;   // streams that copy kernels of this plan were queued on
};

namespace vps {

// Size queries need the class table on the host; piece queries need the piece table.
inline vps::ConfigData& with_host_config(const vps_config* cfg, bool pieces)
{
    vps_config* mc = const_cast<vps_config*>(cfg);
    std::lock_guard<std::mutex> g(mc->host_copy);
    VPS_BACKEND be(nullptr);
    try {
        ensure_config_host(be, mc->d);
        if (pieces) ensure_pieces(be, mc->d);
    } catch (...) {
        // the backend takes back what it allocated: the configuration must not keep pointers to it
        mc->d.piece_base = nullptr; mc->d.pieces = nullptr; mc->d.npieces = -1;
        be.release_all();
        throw;
    }
    be.commit();   // the piece table now belongs to the configuration
    return mc->d;
}

// Queries that read the boxes on the host fetch them first if the plan left them on the device.
inline const PlanData& with_host_boxes(const vps_plan* plan)
{
    vps_plan* mp = const_cast<vps_plan*>(plan);
    std::lock_guard<std::mutex> g(mp->host_copy);
    if (!mp->d.host_boxes_ready) {
        VPS_BACKEND be(nullptr);
        ensure_host_boxes(be, mp->d);
    }
    return mp->d;
}

}  // namespace vps

struct vps_stage_plan {
    vps::StageData d;
    const vps_plan* plan;
    std::mutex guard;
    std::vector<void*> streams;   // streams that copy kernels of this stage plan were queued on
};

#define VPS_TRY try {
#define VPS_CATCH                                                            \
    }                                                                        \
    catch (const vps::Error& e) { return vps::fail(e.code, e.msg); }         \
    catch (const std::bad_alloc&) { return vps::fail(VPS_ERR_OOM, "host allocation failed"); } \
    catch (...) { return vps::fail(VPS_ERR_INVALID_ARG, "unexpected failure"); }

extern "C" {

const char* VPS_FN(last_error)(void) { return vps::g_last_error.c_str(); }

int VPS_FN(set_tile_bytes)(uint32_t bytes)
{
    if (bytes < 4096 || bytes > (1u << 20) || (bytes & (bytes - 1)))
        return vps::fail(VPS_ERR_INVALID_ARG, "tile bytes must be a power of two in [4 KiB, 1 MiB]");
    vps::g_tile_bytes = bytes;
    return VPS_OK;
}

int VPS_FN(set_option)(int32_t option, uint32_t value)
{
    if (option == VPS_OPT_TILE_BYTES) return VPS_FN(set_tile_bytes)(value);
    if (option == VPS_OPT_SMALL_PLAN_BOXES) {
        if (value < 1 || value > (1u << 16)) return vps::fail(VPS_ERR_INVALID_ARG, "small-plan limit must be in [1, 65536]");
        vps::g_small_plan_boxes = value;
        return VPS_OK;
    }
    if (option == VPS_OPT_XPOSE_SHAPE) {
        const uint32_t sa = value & 0xffffu, sb = value >> 16;
        if (value && (sa < 1 || sb < 1 || sa > 64 || sb > 64)) return vps::fail(VPS_ERR_INVALID_ARG, "super-block edges must be in [1, 64]");
        vps::g_xpose_shape = value;
        return VPS_OK;
    }
    if (option == VPS_OPT_PAIR_ORDER_WORK) {
        if (value > 40) return vps::fail(VPS_ERR_INVALID_ARG, "log2 of the pair-ordering work bound must be at most 40");
        vps::g_pair_work_log2 = value;
        return VPS_OK;
    }
    if (option == VPS_OPT_XCD_RUN) {
        if (value > 4096) return vps::fail(VPS_ERR_INVALID_ARG, "XCD run length must be at most 4096 tiles");
        VPS_BACKEND::set_xcd_chunk(value);
        return VPS_OK;
    }
    return vps::fail(VPS_ERR_INVALID_ARG, "unknown option");
}

int VPS_FN(plain_copy)(void* dst, const void* src, uint64_t bytes, void* stream)
{
    if (!bytes) return VPS_OK;
    if (!dst || !src) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t)dst | (uintptr_t)src | bytes) & 15)
        return vps::fail(VPS_ERR_INVALID_ARG, "plain copy needs 16-byte aligned pointers and a multiple of 16 bytes");
    const char* s = (const char*)src;
    const char* d = (const char*)dst;
    if (s < d + bytes && d < s + bytes) return vps::fail(VPS_ERR_INVALID_ARG, "plain copy ranges overlap");
    VPS_TRY
    VPS_BACKEND be(stream);
    be.launch_plain_copy(dst, src, bytes);
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(plain_read)(const void* src, uint64_t bytes, void* sink, void* stream)
{
    if (!bytes) return VPS_OK;
    if (!src || !sink) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t)src | bytes) & 15) return vps::fail(VPS_ERR_INVALID_ARG, "plain read needs a 16-byte aligned pointer and a multiple of 16 bytes");
    VPS_TRY
    VPS_BACKEND be(stream);
    be.launch_plain_half(0, nullptr, src, bytes, sink);
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(plain_fill)(void* dst, uint64_t bytes, void* stream)
{
    if (!bytes) return VPS_OK;
    if (!dst) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t)dst | bytes) & 15) return vps::fail(VPS_ERR_INVALID_ARG, "plain fill needs a 16-byte aligned pointer and a multiple of 16 bytes");
    VPS_TRY
    VPS_BACKEND be(stream);
    be.launch_plain_half(1, dst, nullptr, bytes, nullptr);
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(describe_config)(const vps_model_desc* model, const vps_parallel_desc* par, int32_t rank,
                            vps_config** out)
{
    if (!model || !par || !out) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    VPS_TRY
    vps_config* c = new vps_config();
    VPS_BACKEND be(nullptr);
    try {
        vps::build_config(be, *model, *par, rank, c->d);
    } catch (...) {
        be.release_all();
        delete c;
        throw;
    }
    be.commit();
    *out = c;
    return VPS_OK;
    VPS_CATCH
}

void VPS_FN(config_destroy)(vps_config* c)
{
    if (!c) return;
    VPS_BACKEND be(nullptr);
    vps::free_config(be, c->d);
    delete c;
}

int VPS_FN(plan_intersections_ex)(const vps_config* src, const vps_config* dst, int32_t rank, uint32_t flags,
                                  void* stream, vps_plan** out);

int VPS_FN(plan_intersections)(const vps_config* src, const vps_config* dst, int32_t rank, void* stream,
                               vps_plan** out)
{
    return VPS_FN(plan_intersections_ex)(src, dst, rank, 0, stream, out);
}

int VPS_FN(plan_intersections_ex)(const vps_config* src, const vps_config* dst, int32_t rank, uint32_t flags,
                                  void* stream, vps_plan** out)
{
    if (!src || !dst || !out) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    VPS_TRY
    vps_plan* p = new vps_plan();
    VPS_BACKEND be(stream);
    try {
        if (flags & ~(uint32_t)(VPS_PLAN_ROUTES_ONLY | VPS_PLAN_THROUGH_BUFFERS))
            throw vps::Error{ VPS_ERR_INVALID_ARG, "unknown plan flag" };
        const uint32_t tile_bytes = vps::g_tile_bytes.load(), xpose_shape = vps::g_xpose_shape.load();
        const uint64_t hk = vps::TileHints::key(src->d.model, src->d.par, dst->d.par, rank, flags, tile_bytes, xpose_shape);
        vps::build_plan(be, src->d, dst->d, rank, tile_bytes, xpose_shape,
                        vps::g_small_plan_boxes.load(), (flags & VPS_PLAN_ROUTES_ONLY) != 0,
                        (flags & VPS_PLAN_THROUGH_BUFFERS) != 0, vps::g_tile_hints.get(hk).tiles,
                        vps::g_tile_hints.get(hk).boxes, p->d, true, (int)vps::g_pair_work_log2.load());
        const vps_plan_stats_t& st = p->d.stats;
        vps::g_tile_hints.put(hk, { st.num_retain_tiles + st.num_pack_tiles + st.num_unpack_tiles, st.num_boxes });
    } catch (...) {
        be.release_all();
        delete p;
        throw;
    }
    be.commit();
    *out = p;
    return VPS_OK;
    VPS_CATCH
}

void VPS_FN(plan_destroy)(vps_plan* p)
{
    if (!p) return;
    VPS_BACKEND be(nullptr);
    // copy kernels that are still queued read the plan's tables: wait for the streams they are on
    for (void* s : p->streams) be.wait_stream(s);
    vps::free_plan(be, p->d);
    delete p;
}

}  // extern "C"

namespace vps {

// Launch the tiles [t0, t1) with the given pointers.  ptrs has num_slots entries (host).
template <class BE>
int launch_ops(BE& be, const vps_plan* plan, int64_t t0, int64_t t1, const std::vector<void*>& ptrs,
               int alias)
{
    const PlanData& p = plan->d;
    if (p.routes_only) return fail(VPS_ERR_INVALID_ARG, "the plan was made with VPS_PLAN_ROUTES_ONLY and has no copy tables");
    if (t1 <= t0) return VPS_OK;
    {
        vps_plan* mp = const_cast<vps_plan*>(plan);
        std::lock_guard<std::mutex> g(mp->host_copy);
        void* s = (void*)be.stream();
        if (std::find(mp->streams.begin(), mp->streams.end(), s) == mp->streams.end()) mp->streams.push_back(s);
    }
    PtrArgs pa;
    memset(&pa, 0, sizeof(pa));
    if (p.layout.all_ranks) {
        be.set_ptr_table(p.ptr_table, ptrs.data(), (int)ptrs.size());
        pa.tbl = (char* const*)p.ptr_table;
    } else {
        for (int s = 0; s < PT_INLINE; ++s) pa.inl[s] = (char*)ptrs[(size_t)s];
    }
    be.launch_copy(p.descs, p.tiles, t0, t1 - t0, pa, alias);
    return VPS_OK;
}

inline int check_used(const vps_plan* plan, int op, int32_t rank, const std::vector<void*>& ptrs,
                      bool alias)
{
    const PlanData& p = plan->d;
    const std::vector<uint8_t>& u = p.used[op];
    for (size_t s = 0; s < u.size(); ++s) {
        if (!u[s] || ptrs[s]) continue;
        // a slot of another rank does not matter when only `rank` is launched
        if (p.layout.all_ranks && rank >= 0) {
            const int32_t nb = (p.layout.wa + p.layout.wb) * 8;
            int32_t owner;
            if ((int32_t)s < p.layout.wa * 8) owner = (int32_t)s / 8;
            else if ((int32_t)s < nb) owner = ((int32_t)s - p.layout.wa * 8) / 8;
            else if ((int32_t)s < nb + p.layout.wa) owner = (int32_t)s - nb;
            else owner = (int32_t)s - nb - p.layout.wa;
            if (owner != rank) continue;
        }
        if (alias && op == OP_UNPACK && (int32_t)s >= (p.layout.wa + p.layout.wb) * 8 + p.layout.wa) continue;
        return fail(VPS_ERR_INVALID_ARG, "a buffer that the plan reads or writes is NULL (slot " + std::to_string(s) + ")");
    }
    return VPS_OK;
}

inline int check_rank_arg(const PlanData& p, int32_t rank, int32_t world, bool allow_all)
{
    if (p.rank >= 0) {
        if (rank != p.rank) return fail(VPS_ERR_RANK_RANGE, "plan was made for another rank");
        return VPS_OK;
    }
    if (rank == -1 && allow_all) return VPS_OK;
    if (rank < 0 || rank >= world) return fail(VPS_ERR_RANK_RANGE, "rank outside the world");
    return VPS_OK;
}

}  // namespace vps

extern "C" {

int VPS_FN(pack)(const vps_plan* plan, int32_t rank, const void* const* src_bufs, void* send_buf, void* stream)
{
    if (!plan || !src_bufs) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    const vps::PlanData& p = plan->d;
    if (int rc = vps::check_rank_arg(p, rank, p.A.world, false)) return rc;
    if ((uintptr_t)send_buf & 15) return vps::fail(VPS_ERR_INVALID_ARG, "send_buf must be 16-byte aligned");
    std::vector<void*> ptrs((size_t)vps::num_slots(p.layout), nullptr);
    if (rank < p.A.world) {
        for (int b = 0; b < 8; ++b) ptrs[(size_t)vps::slot_src(p.layout, rank, b)] = (void*)src_bufs[b];
        ptrs[(size_t)vps::slot_send(p.layout, rank)] = send_buf;
    }
    if (int rc = vps::check_used(plan, vps::OP_PACK, rank, ptrs, false)) return rc;
    int64_t t0, t1;
    vps::plan_tile_range(p, vps::OP_PACK, p.rank >= 0 ? -1 : rank, t0, t1);
    VPS_BACKEND be(stream);
    return vps::launch_ops(be, plan, t0, t1, ptrs, 0);
    VPS_CATCH
}

int VPS_FN(unpack)(const vps_plan* plan, int32_t rank, const void* recv_buf, void* const* dst_bufs, void* stream)
{
    if (!plan || !dst_bufs) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    const vps::PlanData& p = plan->d;
    if (int rc = vps::check_rank_arg(p, rank, p.B.world, false)) return rc;
    if ((uintptr_t)recv_buf & 15) return vps::fail(VPS_ERR_INVALID_ARG, "recv_buf must be 16-byte aligned");
    std::vector<void*> ptrs((size_t)vps::num_slots(p.layout), nullptr);
    if (rank < p.B.world) {
        for (int b = 0; b < 8; ++b) ptrs[(size_t)vps::slot_dst(p.layout, rank, b)] = dst_bufs[b];
        ptrs[(size_t)vps::slot_recv(p.layout, rank)] = (void*)recv_buf;
    }
    if (int rc = vps::check_used(plan, vps::OP_UNPACK, rank, ptrs, false)) return rc;
    int64_t t0, t1;
    vps::plan_tile_range(p, vps::OP_UNPACK, p.rank >= 0 ? -1 : rank, t0, t1);
    VPS_BACKEND be(stream);
    return vps::launch_ops(be, plan, t0, t1, ptrs, 0);
    VPS_CATCH
}

int VPS_FN(plan_buffer_bytes)(const vps_plan* plan, int32_t rank, uint64_t* send_total, uint64_t* recv_total,
                              uint64_t* retain_total, uint64_t* scratch_needed, uint64_t* recv_offset)
{
    if (!plan) return vps::fail(VPS_ERR_INVALID_ARG, "null plan");
    const vps::PlanData& p = plan->d;
    const int32_t W = p.A.world > p.B.world ? p.A.world : p.B.world;
    if (rank < -1 || rank >= W) return vps::fail(VPS_ERR_RANK_RANGE, "rank outside both worlds");
    if (p.rank >= 0 && rank != p.rank) return vps::fail(VPS_ERR_RANK_RANGE, "plan was made for another rank");
    uint64_t s = 0, r = 0, k = 0, need = 0, roff = 0;
    if (rank >= 0) {
        s = p.send_base[(size_t)rank + 1] - p.send_base[(size_t)rank];
        r = p.recv_base[(size_t)rank + 1] - p.recv_base[(size_t)rank];
        k = p.through_buffers ? 0 : vps::plan_pair_bytes(p, rank, rank);
        roff = (s + 255) & ~255ull;
        need = roff + r;
    } else {
        s = p.send_base[(size_t)W];
        r = p.recv_base[(size_t)W];
        for (int32_t q = 0; q < p.A.world && q < p.B.world && !p.through_buffers; ++q) k += vps::plan_pair_bytes(p, q, q);
        need = s;
    }
    if (send_total) *send_total = s;
    if (recv_total) *recv_total = r;
    if (retain_total) *retain_total = k;
    if (scratch_needed) *scratch_needed = need;
    if (recv_offset) *recv_offset = roff;
    return VPS_OK;
}

int VPS_FN(apply_transition)(const vps_plan* plan, int32_t rank, const void* const* src_bufs,
                             void* const* dst_bufs, void* scratch, uint64_t scratch_bytes, void* stream)
{
    if (!plan || !src_bufs || !dst_bufs) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    const vps::PlanData& p = plan->d;
    if (p.rank >= 0 ? rank != p.rank : rank != -1)
        return vps::fail(VPS_ERR_RANK_RANGE, "rank must be the planned rank (or -1 for an all-ranks plan)");
    uint64_t s, r, k, need, roff;
    VPS_FN(plan_buffer_bytes)(plan, rank, &s, &r, &k, &need, &roff);
    if (scratch_bytes < need) return vps::fail(VPS_ERR_SCRATCH_TOO_SMALL, "scratch smaller than scratch_needed");
    if (need && (!scratch || ((uintptr_t)scratch & 15))) return vps::fail(VPS_ERR_INVALID_ARG, "scratch must be a 16-byte aligned device pointer");
    const vps::PtrLayout& L = p.layout;
    std::vector<void*> ptrs((size_t)vps::num_slots(L), nullptr);
    // the table holds the retain tiles, then the pack tiles, then the unpack tiles
    const int64_t t_retain = p.op_tile[vps::OP_RETAIN].front(), t_unpack = p.op_tile[vps::OP_UNPACK].front();
    const int64_t t_end = p.op_tile[vps::OP_UNPACK].back();
    {
        const size_t ns = (size_t)(p.rank >= 0 ? 1 : p.A.world) * 8, nd = (size_t)(p.rank >= 0 ? 1 : p.B.world) * 8;
        for (size_t i = 0; i < ns; ++i)
            for (size_t j = 0; j < nd; ++j)
                if (src_bufs[i] && src_bufs[i] == dst_bufs[j])
                    return vps::fail(VPS_ERR_INVALID_ARG, "a source buffer is also passed as a destination buffer");
    }
    VPS_BACKEND be(stream);
    if (p.rank >= 0) {
        for (int b = 0; b < 8; ++b) {
            ptrs[(size_t)vps::slot_src(L, rank, b)] = (void*)src_bufs[b];
            ptrs[(size_t)vps::slot_dst(L, rank, b)] = dst_bufs[b];
        }
        ptrs[(size_t)vps::slot_send(L, rank)] = scratch;
        ptrs[(size_t)vps::slot_recv(L, rank)] = (char*)scratch + roff;
        for (int op = 0; op < 3; ++op)
            if (int rc = vps::check_used(plan, op, rank, ptrs, false)) return rc;
        // the three operations touch disjoint destinations: one launch over every tile
        if (!p.through_buffers)
            return vps::launch_ops(be, plan, t_retain, t_end, ptrs, 0);
        // the rank is its own peer: its segment is unpacked straight out of the send buffer, after
        // the pack launch has written it
        if (int rc = vps::launch_ops(be, plan, t_retain, t_unpack, ptrs, 0)) return rc;
        return vps::launch_ops(be, plan, t_unpack, t_end, ptrs, 1);
    }
    for (int32_t q = 0; q < p.A.world; ++q) {
        for (int b = 0; b < 8; ++b) ptrs[(size_t)vps::slot_src(L, q, b)] = (void*)src_bufs[(size_t)q * 8 + b];
        ptrs[(size_t)vps::slot_send(L, q)] = (char*)scratch + p.send_base[(size_t)q];
    }
    for (int32_t q = 0; q < p.B.world; ++q)
        for (int b = 0; b < 8; ++b) ptrs[(size_t)vps::slot_dst(L, q, b)] = dst_bufs[(size_t)q * 8 + b];
    for (int op = 0; op < 3; ++op)
        if (int rc = vps::check_used(plan, op, -1, ptrs, true)) return rc;
    // retain + pack for every rank, then unpack straight out of the senders' segments
    if (int rc = vps::launch_ops(be, plan, t_retain, t_unpack, ptrs, 0)) return rc;
    return vps::launch_ops(be, plan, t_unpack, t_end, ptrs, 1);
    VPS_CATCH
}

int VPS_FN(config_world)(const vps_config* c, int32_t* world)
{
    if (!c || !world) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *world = c->d.P.world;
    return VPS_OK;
}

int VPS_FN(config_num_buffers)(const vps_config* c, int32_t rank, int32_t* n)
{
    if (!c || !n) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    if (rank < 0 || rank >= c->d.P.world) return vps::fail(VPS_ERR_RANK_RANGE, "rank outside the world");
    *n = VPS_NUM_BUFFERS;
    return VPS_OK;
}

int VPS_FN(config_num_tensors)(const vps_config* c, int32_t* n)
{
    if (!c || !n) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *n = c->d.P.nt;
    return VPS_OK;
}

int VPS_FN(config_buffer_bytes)(const vps_config* c, int32_t rank, int32_t buf, uint64_t* bytes)
{
    if (!c || !bytes) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    if (rank < 0 || rank >= c->d.P.world) return vps::fail(VPS_ERR_RANK_RANGE, "rank outside the world");
    if (buf < 0 || buf >= 8) return vps::fail(VPS_ERR_INVALID_ARG, "buffer index must be 0..7");
    VPS_TRY
    *bytes = vps::config_buffer_elems(vps::with_host_config(c, false), rank, buf) * vps::kind_bytes(buf % 4);
    return VPS_OK;
    VPS_CATCH
    return VPS_OK;
}

int VPS_FN(config_num_pieces)(const vps_config* c, int64_t* n)
{
    if (!c || !n) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    *n = vps::with_host_config(c, true).npieces;
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(config_get_pieces)(const vps_config* c, vps_piece* out, int64_t max)
{
    if (!c || (!out && max > 0)) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    const vps::ConfigData& d = vps::with_host_config(c, true);
    VPS_BACKEND be(nullptr);
    const int64_t n = max < d.npieces ? max : d.npieces;
    if (n > 0) be.download(out, d.pieces, sizeof(vps_piece) * (size_t)n);
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(plan_pair_bytes)(const vps_plan* plan, int32_t src_rank, int32_t dst_rank, uint64_t* bytes)
{
    if (!plan || !bytes) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    const vps::PlanData& p = plan->d;
    if (src_rank < 0 || src_rank >= p.A.world || dst_rank < 0 || dst_rank >= p.B.world)
        return vps::fail(VPS_ERR_RANK_RANGE, "rank outside the world");
    *bytes = vps::plan_pair_bytes(p, src_rank, dst_rank);
    return VPS_OK;
}

int VPS_FN(plan_peer_bytes)(const vps_plan* plan, int32_t rank, int32_t peer, uint64_t* send, uint64_t* recv)
{
    if (!plan) return vps::fail(VPS_ERR_INVALID_ARG, "null plan");
    const vps::PlanData& p = plan->d;
    const int32_t W = p.A.world > p.B.world ? p.A.world : p.B.world;
    if (rank < 0 || rank >= W || peer < 0 || peer >= W) return vps::fail(VPS_ERR_RANK_RANGE, "rank outside both worlds");
    uint64_t s = 0, r = 0;
    s = vps::plan_pair_bytes(p, rank, peer);
    r = vps::plan_pair_bytes(p, peer, rank);
    if (send) *send = s;
    if (recv) *recv = r;
    return VPS_OK;
}

int VPS_FN(plan_peer_segment)(const vps_plan* plan, int32_t src_rank, int32_t dst_rank, uint64_t* send_off,
                              uint64_t* recv_off, uint64_t* bytes)
{
    if (!plan) return vps::fail(VPS_ERR_INVALID_ARG, "null plan");
    VPS_TRY
    const vps::PlanData& p = vps::with_host_boxes(plan);
    if (src_rank < 0 || src_rank >= p.A.world || dst_rank < 0 || dst_rank >= p.B.world)
        return vps::fail(VPS_ERR_RANK_RANGE, "rank outside the world");
    uint64_t so = UINT64_MAX, ro = UINT64_MAX, nb = 0;
    if (src_rank != dst_rank || p.through_buffers) {
        // boxes are sorted by (src, dst, ...): binary search the pair's range
        const std::vector<vps_box>& bx = p.boxes_send_order;
        auto key = [](const vps_box& b) { return ((uint64_t)b.src_rank << 32) | (uint32_t)b.dst_rank; };
        const uint64_t want = ((uint64_t)src_rank << 32) | (uint32_t)dst_rank;
        size_t lo = 0, hi = bx.size();
        while (lo < hi) { size_t mid = (lo + hi) / 2; if (key(bx[mid]) < want) lo = mid + 1; else hi = mid; }
        size_t end = lo;
        while (end < bx.size() && key(bx[end]) == want) ++end;
        if (end > lo) {
            const vps_box& f = bx[lo];
            const vps_box& l = bx[end - 1];
            so = f.send_pos; ro = f.recv_pos;
            if (f.send_pos != UINT64_MAX) nb = l.send_pos + vps::box_slot_bytes(l) - f.send_pos;
            else if (f.recv_pos != UINT64_MAX) nb = l.recv_pos + vps::box_slot_bytes(l) - f.recv_pos;
        }
    }
    if (send_off) *send_off = so;
    if (recv_off) *recv_off = ro;
    if (bytes) *bytes = nb;
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(plan_num_boxes)(const vps_plan* plan, int64_t* n)
{
    if (!plan || !n) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *n = plan->d.nboxes;
    return VPS_OK;
}

int VPS_FN(plan_get_boxes)(const vps_plan* plan, vps_box* out, int64_t max)
{
    if (!plan || (!out && max > 0)) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    const vps::PlanData& p = vps::with_host_boxes(plan);
    const int64_t n = max < p.nboxes ? max : p.nboxes;
    if (n > 0) memcpy(out, p.boxes_send_order.data(), sizeof(vps_box) * (size_t)n);
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(plan_stats)(const vps_plan* plan, vps_plan_stats_t* out)
{
    if (!plan || !out) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *out = plan->d.stats;
    return VPS_OK;
}

int VPS_FN(stage_exchange)(const vps_plan* plan, uint64_t budget, void* stream, vps_stage_plan** out)
{
    if (!plan || !out) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    VPS_TRY
    vps_stage_plan* sp = new vps_stage_plan();
    sp->plan = plan;
    VPS_BACKEND be(stream);
    try {
        vps::build_stage_plan(be, vps::with_host_boxes(plan), budget, plan->d.tile_bytes, sp->d);
    } catch (...) {
        be.release_all();
        delete sp;
        throw;
    }
    be.commit();
    *out = sp;
    return VPS_OK;
    VPS_CATCH
}

void VPS_FN(stage_plan_destroy)(vps_stage_plan* sp)
{
    if (!sp) return;
    VPS_BACKEND be(nullptr);
    for (void* s : sp->streams) be.wait_stream(s);
    vps::free_stage(be, sp->d);
    delete sp;
}

int VPS_FN(stage_info)(const vps_stage_plan* sp, int32_t* num_steps, int32_t* num_stages, uint64_t* scratch_needed)
{
    if (!sp) return vps::fail(VPS_ERR_INVALID_ARG, "null stage plan");
    if (num_steps) *num_steps = sp->d.nsteps;
    if (num_stages) *num_stages = sp->d.nstages;
    if (scratch_needed) *scratch_needed = sp->d.scratch_needed;
    return VPS_OK;
}

int VPS_FN(stage_steps)(const vps_stage_plan* sp, int32_t* stage_of_step, uint64_t* step_cost, int32_t max_entries)
{
    if (!sp) return vps::fail(VPS_ERR_INVALID_ARG, "null stage plan");
    for (int32_t s = 0; s <= sp->d.nsteps && s < max_entries; ++s) {
        if (stage_of_step) stage_of_step[s] = sp->d.stage_of_step[(size_t)s];
        if (step_cost) step_cost[s] = sp->d.step_cost[(size_t)s];
    }
    return VPS_OK;
}

int VPS_FN(apply_transition_staged)(const vps_stage_plan* sp, const void* const* src_bufs, void* const* dst_bufs,
                                    void* scratch, uint64_t scratch_bytes, void* stream)
{
    if (!sp || !src_bufs || !dst_bufs) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    const vps::StageData& sd = sp->d;
    const vps::PlanData& p = sp->plan->d;
    if (scratch_bytes < sd.scratch_needed) return vps::fail(VPS_ERR_SCRATCH_TOO_SMALL, "scratch smaller than scratch_needed");
    if (sd.scratch_needed && (!scratch || ((uintptr_t)scratch & 15))) return vps::fail(VPS_ERR_INVALID_ARG, "scratch must be a 16-byte aligned device pointer");
    const vps::PtrLayout& L = p.layout;
    std::vector<void*> ptrs((size_t)vps::num_slots(L), nullptr);
    for (int32_t q = 0; q < p.A.world; ++q)
        for (int b = 0; b < 8; ++b) ptrs[(size_t)vps::slot_src(L, q, b)] = (void*)src_bufs[(size_t)q * 8 + b];
    for (int32_t q = 0; q < p.B.world; ++q)
        for (int b = 0; b < 8; ++b) ptrs[(size_t)vps::slot_dst(L, q, b)] = dst_bufs[(size_t)q * 8 + b];
    for (int op = 0; op < 3; ++op) {
        // send / receive slots are filled per stage below
        std::vector<void*> chk = ptrs;
        for (int32_t q = 0; q < p.A.world; ++q) chk[(size_t)vps::slot_send(L, q)] = scratch;
        for (int32_t q = 0; q < p.B.world; ++q) chk[(size_t)vps::slot_recv(L, q)] = scratch;
        if (int rc = vps::check_used(sp->plan, op, -1, chk, false)) return rc;
    }
    VPS_BACKEND be(stream);
    {
        vps_stage_plan* msp = const_cast<vps_stage_plan*>(sp);
        std::lock_guard<std::mutex> g(msp->guard);
        if (std::find(msp->streams.begin(), msp->streams.end(), stream) == msp->streams.end()) msp->streams.push_back(stream);
        vps_plan* mp = const_cast<vps_plan*>(sp->plan);
        std::lock_guard<std::mutex> g2(mp->host_copy);
        if (std::find(mp->streams.begin(), mp->streams.end(), stream) == mp->streams.end()) mp->streams.push_back(stream);
    }
    vps::PtrArgs pa;
    memset(&pa, 0, sizeof(pa));
    pa.tbl = (char* const*)sd.ptr_table;
    // retained boxes: old local -> new local, once
    be.set_ptr_table(sd.ptr_table, ptrs.data(), (int)ptrs.size());
    be.launch_copy(p.descs, p.tiles, p.op_tile[vps::OP_RETAIN].front(),
                   p.op_tile[vps::OP_RETAIN].back() - p.op_tile[vps::OP_RETAIN].front(), pa, 0);
    for (int32_t g = 0; g < sd.nstages; ++g) {
        for (int32_t q = 0; q < p.A.world; ++q)
            ptrs[(size_t)vps::slot_send(L, q)] = (char*)scratch + sd.send_base[(size_t)g * (size_t)p.A.world + (size_t)q];
        for (int32_t q = 0; q < p.B.world; ++q)
            ptrs[(size_t)vps::slot_recv(L, q)] = (char*)scratch + sd.recv_base[(size_t)g * (size_t)p.B.world + (size_t)q];
        be.set_ptr_table(sd.ptr_table, ptrs.data(), (int)ptrs.size());
        be.launch_copy(sd.descs, sd.tiles, sd.pack_begin[(size_t)g], sd.pack_begin[(size_t)g + 1] - sd.pack_begin[(size_t)g], pa, 0);
        be.launch_copy(sd.descs, sd.tiles, sd.exch_begin[(size_t)g], sd.exch_begin[(size_t)g + 1] - sd.exch_begin[(size_t)g], pa, 0);
        be.launch_copy(sd.descs, sd.tiles, sd.unpack_begin[(size_t)g], sd.unpack_begin[(size_t)g + 1] - sd.unpack_begin[(size_t)g], pa, 0);
    }
    return VPS_OK;
    VPS_CATCH
}

int VPS_FN(plan_classify_collectives)(const vps_plan* plan, const vps_config* src, void* stream, int32_t* classes,
                                      int64_t max_entries)
{
    if (!plan || !src || !classes) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    VPS_TRY
    if (memcmp(&src->d.P, &plan->d.A, sizeof(vps::ParConst)) != 0)
        return vps::fail(VPS_ERR_MODEL_MISMATCH, "src must be the source configuration of the plan");
    std::vector<int32_t> cls;
    VPS_BACKEND be(stream);
    try {
        vps::classify_collectives(be, plan->d, src->d, cls);
    } catch (...) {
        be.release_all();
        throw;
    }
    be.commit();
    for (size_t i = 0; i < cls.size() && (int64_t)i < max_entries; ++i) classes[i] = cls[i];
    return VPS_OK;
    VPS_CATCH
}

}  // extern "C"

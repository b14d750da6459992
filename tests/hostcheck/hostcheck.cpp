// hostcheck.cpp - TEST INFRASTRUCTURE: a CPU build of the library's per-item code.
//
// The mapper, planner and tile-geometry functions of paper_2605_18815_amd/csrc are written so
// that they also compile as plain C++.  This file instantiates the same pipeline with a
// sequential backend (one loop iteration per kernel lane, std::stable_sort, a serial scan) and
// exports it as vpsh_* so that the test-suite can check index arithmetic and buffer bounds
// against the CPU oracle on a machine without a GPU.  Every access of the copy step is bounds
// checked against the buffer sizes registered with vpsh_set_bounds.  It is never linked into,
// or loaded by, the product library.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <vector>

#include "../../paper_2605_18815_amd/csrc/vps_core.h"
#include "../../paper_2605_18815_amd/csrc/vps_inventory.h"

namespace vps {

struct Bounds {
    const char* lo;
    const char* hi;
};
static std::vector<Bounds> g_bounds;
static long g_violations = 0;

// Dry run: the copy step checks bounds and records every destination write as an interval, but
// moves nothing, so that shares far larger than host memory can be walked with made-up buffer
// addresses.
struct Interval {
    uint64_t lo, hi;
};
static bool g_dry_run = false;
// Tiles seen by the copy step since the last vpsh_tile_histogram call, by kind: count and bytes.
enum { TK_FULL_RUN = 0, TK_PART_RUN = 1, TK_FEW_RUNS = 2, TK_MANY_RUNS = 3, TK_XPOSE = 4, TK_ELEM = 5, TK_EMPTY = 6, TK_KINDS = 7 };
static uint64_t g_hist_count[TK_KINDS], g_hist_bytes[TK_KINDS];
static uint64_t g_unaligned_run_tiles = 0;
static std::vector<Interval> g_dry_writes;

static bool in_bounds(const void* p, size_t n)
{
    const char* c = (const char*)p;
    for (const Bounds& b : g_bounds)
        if (c >= b.lo && c + n <= b.hi) return true;
    return false;
}

uint32_t g_tile_bytes_setting();

class HostBackend {
public:
    explicit HostBackend(void*) {}
    ~HostBackend() { release_all(); }
    // Ownership as in the device backend: what a build allocates belongs to the backend until
    // commit() hands it to the handle; a backend that goes away without commit() takes its
    // allocations with it (so a handle that kept a pointer reads freed memory, which the
    // sanitizer build reports).
    template <class T> T* alloc(int64_t n)
    {
        // filled with a pattern, not zeros: pooled device memory holds whatever the last user left
        const size_t bytes = (size_t)(n > 0 ? n : 1) * sizeof(T);
        void* p = malloc(bytes);
        memset(p, 0xCD, bytes);
        live_.push_back(p);
        return (T*)p;
    }
    void free(void* p)
    {
        if (!p) return;
        auto it = std::find(live_.begin(), live_.end(), p);
        if (it != live_.end()) live_.erase(it);
        ::free(p);
    }
    void commit() { live_.clear(); }
    void release_all()
    {
        for (void* p : live_) ::free(p);
        live_.clear();
    }
    std::vector<void*> live_;
    template <class Step, class F> void for_each(Step, int64_t n, F f) { for (int64_t i = 0; i < n; ++i) f(i); }
    void exclusive_scan(const int64_t* in, int64_t* out, int64_t n)
    {
        int64_t acc = 0;
        for (int64_t i = 0; i <= n; ++i) { out[i] = acc; acc += in[i]; }
    }
    void exclusive_scan_rows(const int64_t* in, int64_t* out, int64_t n, int64_t stride, int rows)
    {
        for (int r = 0; r < rows; ++r) exclusive_scan(in + r * stride, out + r * stride, n);
    }
    void sort_pairs(uint64_t*& keys, uint32_t*& vals, int64_t n, int bits = 64)
    {
        for (int64_t i = 0; bits < 64 && i < n; ++i)
            if (keys[i] >> bits) { fprintf(stderr, "sort key wider than %d bits\n", bits); abort(); }
        if (n <= 1) return;
        std::vector<int64_t> idx((size_t)n);
        std::iota(idx.begin(), idx.end(), 0);
        std::stable_sort(idx.begin(), idx.end(), [&](int64_t a, int64_t b) { return keys[a] < keys[b]; });
        std::vector<uint64_t> k2((size_t)n);
        std::vector<uint32_t> v2((size_t)n);
        for (int64_t i = 0; i < n; ++i) { k2[(size_t)i] = keys[idx[(size_t)i]]; v2[(size_t)i] = vals[idx[(size_t)i]]; }
        memcpy(keys, k2.data(), sizeof(uint64_t) * (size_t)n);
        memcpy(vals, v2.data(), sizeof(uint32_t) * (size_t)n);
    }
    void upload(void* d, const void* h, size_t b) { if (b) memcpy(d, h, b); }
    void download(void* h, const void* d, size_t b) { if (b) memcpy(h, d, b); }
    void download_later(void* h, const void* d, size_t b) { if (b) memcpy(h, d, b); }
    void zero(void* d, size_t b) { if (b) memset(d, 0, b); }
    void* host_mirror(void* host, size_t) { return host; }
    void* alloc_zeroed(size_t bytes) { void* p = alloc<uint8_t>((int64_t)bytes); memset(p, 0, bytes); return p; }
    void sync() {}
    void wait_stream(void*) {}
    void* stream() const { return nullptr; }
    static void set_xcd_chunk(uint32_t) {}
    void after_null_stream() {}

    // The same per-item code as the device kernels, one item after the other.
    void layout_classes(const ParConst& P, const ModelConst& M, TensorRec* T, TensorLayout* TL, ClassRec* C)
    {
        for (int32_t t = 0; t < P.nt; ++t) T[t] = inventory_rec(M, t);
        for (int32_t cls = 0; cls < P.ncls; ++cls) {
            uint64_t running = 0;
            for (int32_t q = 0; q < P.nt; ++q) {
                const int32_t t = P.flat_order ? P.nt - 1 - q : q;
                if (class_of_tensor(P, T[t]) != cls) continue;
                TensorLayout tl;
                tl.start = running; tl.shard_len = shard_elems(P, T[t]); tl.cls = cls; tl.stage = cls < P.pp ? cls : (cls - P.pp) / P.ep;
                TL[t] = tl;
                running += tl.shard_len;
            }
            C[cls] = make_class_rec(P, cls, running);
        }
    }

    static constexpr uint64_t PLAN_LIST_CAP = 1ull << 22;
    bool plan_emit(const PlanCtx& pc, int mode, bool through, vps_box* raw, OrderRec* recs, uint64_t cap, uint64_t* counter,
                   uint64_t*, bool, const PairCounts& pairs)
    {
        const int pb = plan_part_bits(mode);
        const int64_t callers = plan_num_lanes(pc, mode) << pb;
        for (int64_t e = 0; e < callers; ++e)
            plan_lane_boxes(pc, mode, e >> pb, [&](const vps_box& b) {
                const uint64_t k = (*counter)++;
                emit_box(b, make_order_rec(b, pc.ma.T[b.tensor], pc.rank, through), k, raw, recs, cap, pairs);
            }, (int)(e & ((1 << pb) - 1)), 1 << pb);
        return false;
    }

    template <class Step, class F>
    void exclusive_scan_counted_then_each(Step, const int64_t* in, int64_t* out, int64_t bound, const uint64_t* count,
                                          int mult, int64_t* rows, int64_t row_len, int nrows, int64_t m, F f,
                                          const uint64_t* blk, uint64_t* mirror, int64_t words)
    {
        const int64_t len = (int64_t)*count * mult + 1;
        if (len <= bound) {
            exclusive_scan(in, out, len - 1);
            for (int r = 0; r < nrows; ++r) {
                int64_t run = 0;
                for (int64_t i = 0; i < row_len; ++i) { const int64_t v = rows[r * row_len + i]; rows[r * row_len + i] = run; run += v; }
            }
            for (int64_t i = 0; i < m; ++i) f(i);
        }
        for (int64_t i = 0; i < words; ++i) mirror[i] = blk[i];
    }

    void tile_table(const int64_t* tile_base, const CopyDesc* descs, const uint64_t* nbox, int64_t n_host, int64_t bound,
                    TileRef* tiles, int64_t cap, int64_t)
    {
        const int64_t n = nbox ? (int64_t)*nbox : n_host;
        if (nbox && n > bound) return;
        const int64_t total = tile_base[3 * n] < cap ? tile_base[3 * n] : cap;
        int64_t d = 0;
        for (int64_t t = 0; t < total; ++t) {
            while (t >= tile_base[d + 1]) ++d;   // (descriptors without tiles are stepped over)
            tiles[t] = make_tile(descs[d], (uint32_t)d, (uint32_t)(t - tile_base[d]));
        }
    }

    template <class Step, class F>
    void pair_rank_each(Step, const PairRec* bucket, const uint64_t* pstart, const uint64_t* pcount, int64_t n,
                        const uint64_t* work, uint64_t work_max, F f)
    {
        for (int64_t j = 0; j < n; ++j) {
            const PairRec me = bucket[j];
            const uint64_t pr = me.key >> 26, lo = pstart[pr], cnt = pcount[pr];
            uint64_t before = (uint64_t)j - lo, bytes = 0;
            if (*work <= work_max) {
                before = 0;
                for (uint64_t q = lo; q < lo + cnt; ++q) {
                    const PairRec o = bucket[q];
                    const bool less = pair_rec_less(o, me);
                    before += less ? 1 : 0;
                    bytes += (less && (o.bytes_flags & ORD_SENDS)) ? (o.bytes_flags & ~(uint64_t)15) : 0;
                }
            }
            f(j, before, bytes);
        }
    }

    template <class Step, class P, class F>
    void order_by_counting_each(Step, const OrderRec* recs, const uint64_t* nbox, int64_t bound, P pre, F f)
    {
        const uint64_t n = *nbox;
        if (n > (uint64_t)bound) return;
        for (uint64_t k = 0; k < n; ++k) {
            const OrderPlace o = order_by_counting(recs, (uint32_t)n, (uint32_t)k);
            for (uint32_t part = 0; part < 16; ++part) f((uint32_t)k, o, part, pre((uint32_t)k, part));
        }
    }
    void set_ptr_table(void** table, void* const* host_ptrs, int n) { memcpy(table, host_ptrs, sizeof(void*) * (size_t)n); }

    void launch_plain_copy(void* dst, const void* src, uint64_t bytes)
    {
        if (!in_bounds((const char*)src, bytes) || !in_bounds((char*)dst, bytes)) { ++g_violations; return; }
        memcpy(dst, src, bytes);
    }

    void launch_plain_half(int mode, void* dst, const void* src, uint64_t bytes, void* sink)
    {
        if (mode == 0) { if (!in_bounds((const char*)src, bytes) || !in_bounds((char*)sink, 4)) ++g_violations; return; }
        if (!in_bounds((char*)dst, bytes)) { ++g_violations; return; }
        memset(dst, 0xA5, bytes);
    }

    // Same slot walk as the device kernel, one lane at a time, with bounds checks.
    void launch_copy(const CopyDesc* descs, const TileRef* tiles, int64_t tile0, int64_t ntiles,
                     const PtrArgs& pa, int alias_exchange)
    {
        auto slot_ptr = [&](int32_t s) { return pa.tbl ? pa.tbl[s] : pa.inl[s]; };
        auto note_write = [&](const char* t, size_t n) {
            const uint64_t lo = (uint64_t)(uintptr_t)t;
            if (!g_dry_writes.empty() && g_dry_writes.back().hi == lo) g_dry_writes.back().hi = lo + n;
            else g_dry_writes.push_back({ lo, lo + n });
        };
        auto move = [&](const char* s, char* t, size_t n) {
            if (!in_bounds(s, n) || !in_bounds(t, n)) { ++g_violations; return; }
            if (g_dry_run) { note_write(t, n); return; }
            memcpy(t, s, n);
        };
        for (int64_t ti = 0; ti < ntiles; ++ti) {
            const TileRef tr = tiles[tile0 + ti];
            if (!(tr.nruns_flags & TILE_INDIRECT)) {
                const uint32_t nruns = tr.nruns_flags >> 8;
                {
                    int kind;
                    uint64_t bytes = (uint64_t)nruns * tr.nbytes;
                    if (tr.nruns_flags & TILE_XPOSE) {
                        kind = TK_XPOSE;
                        bytes = (uint64_t)(tr.nbytes & 0xffffu) * (tr.nbytes >> 16) * ((tr.nruns_flags & TILE_ES2) ? 2 : 4);
                    } else if (nruns == 0) kind = TK_EMPTY;
                    else if (nruns == 1) kind = 2 * tr.nbytes >= g_tile_bytes_setting() ? TK_FULL_RUN : TK_PART_RUN;
                    else kind = nruns < 4 ? TK_FEW_RUNS : TK_MANY_RUNS;
                    g_hist_count[kind]++;
                    g_hist_bytes[kind] += bytes;
                }
                const uint64_t sa = (alias_exchange && tr.alt_src != VPS_TILE_NO_ALT) ? tr.alt_src : tr.src;
                const uint64_t s0 = (uint64_t)(uintptr_t)slot_ptr(tile_slot(sa)) + tile_offset(sa);
                const uint64_t d0 = (uint64_t)(uintptr_t)slot_ptr(tile_slot(tr.dst)) + tile_offset(tr.dst);
                if (!(tr.nruns_flags & TILE_XPOSE) && nruns == 1 && (d0 & 255)) ++g_unaligned_run_tiles;
                if (tr.nruns_flags & TILE_XPOSE) {
                    const uint32_t ta = tr.nbytes & 0xffffu, tb = tr.nbytes >> 16;
                    const uint32_t es = (tr.nruns_flags & TILE_ES2) ? 2 : 4;
                    if (ta == 0 || tb == 0 || ta > XPOSE_T || tb > XPOSE_T) ++g_violations;
                    for (uint32_t a = 0; a < ta; ++a) {
                        if (g_dry_run) {   // one destination row of the block per recorded write
                            const char* trow = (const char*)(uintptr_t)(d0 + (uint64_t)((int64_t)a * tr.dst_pitch));
                            if (!in_bounds(trow, (size_t)tb * es)) ++g_violations;
                            else note_write(trow, (size_t)tb * es);
                            for (uint32_t b = 0; b < tb; b += tb > 1 ? tb - 1 : 1)   // first and last source element of the row
                                if (!in_bounds((const char*)(uintptr_t)(s0 + (uint64_t)a * es + (uint64_t)((int64_t)b * tr.src_pitch)), es)) ++g_violations;
                            continue;
                        }
                        for (uint32_t b = 0; b < tb; ++b)
                            move((const char*)(uintptr_t)(s0 + (uint64_t)a * es + (uint64_t)((int64_t)b * tr.src_pitch)),
                                 (char*)(uintptr_t)(d0 + (uint64_t)((int64_t)a * tr.dst_pitch) + (uint64_t)b * es), es);
                    }
                    continue;
                }
                for (uint32_t r = 0; r < nruns; ++r) {
                    const uint64_t srow = s0 + r * (uint64_t)tr.src_pitch, drow = d0 + r * (uint64_t)tr.dst_pitch;
                    const RunWindow g = run_window(srow, drow, tr.nbytes, 0, (tr.nbytes + 30) >> 4);
                    if (g.head_bytes) move((const char*)(uintptr_t)srow, (char*)(uintptr_t)drow, g.head_bytes);
                    if (g.dvec & 15) ++g_violations;
                    if (g_dry_run && g.wbeg < g.wend)
                        move((const char*)(uintptr_t)(g.svec + 16ull * g.wbeg), (char*)(uintptr_t)(g.dvec + 16ull * g.wbeg),
                             16ull * (g.wend - g.wbeg));
                    for (uint32_t w = g.wbeg; w < g.wend && !g_dry_run; ++w)
                        move((const char*)(uintptr_t)(g.svec + 16ull * w), (char*)(uintptr_t)(g.dvec + 16ull * w), 16);
                    if (g.tail_bytes) move((const char*)(uintptr_t)(g.svec + g.tail_off), (char*)(uintptr_t)(g.dvec + g.tail_off), g.tail_bytes);
                }
                continue;
            }
            const uint32_t tq = (uint32_t)(tr.alt_src >> 32);
            const CopyDesc d = descs[(uint32_t)tr.alt_src];
            g_hist_count[TK_ELEM]++;
            g_hist_bytes[TK_ELEM] += (uint64_t)d.rows_per_tile * d.es;
            const bool alias = alias_exchange && d.alt_src_slot >= 0;
            const char* sbase = alias ? slot_ptr(d.alt_src_slot) + d.alt_src_byte : slot_ptr(d.src_slot) + d.src_byte;
            char* dbase = slot_ptr(d.dst_slot) + d.dst_byte;
            {
                const uint64_t vol = (uint64_t)d.ext[0] * d.ext[1] * d.ext[2] * d.ext[3];
                const uint64_t k0 = (uint64_t)tq * d.rows_per_tile;
                const uint64_t k1 = k0 + d.rows_per_tile < vol ? k0 + d.rows_per_tile : vol;
                for (uint64_t k = k0; k < k1; ++k) {
                    int64_t so, to;
                    elem_offsets(d, k, so, to);
                    move(sbase + so, dbase + to, d.es);
                }
            }
        }
    }
};

}  // namespace vps

#define VPS_BACKEND vps::HostBackend
#define VPS_FN(name) vpsh_##name
#include "../../paper_2605_18815_amd/csrc/vps_api_impl.h"

namespace vps {
uint32_t g_tile_bytes_setting() { return g_tile_bytes; }
}

extern "C" {

// Register the address ranges the copy step may touch (pairs of lo, hi); clears the counter.
void vpsh_set_bounds(const void* const* lo_hi, int n)
{
    vps::g_bounds.clear();
    for (int i = 0; i < n; ++i) vps::g_bounds.push_back({ (const char*)lo_hi[2 * i], (const char*)lo_hi[2 * i + 1] });
    vps::g_violations = 0;
}

long vpsh_bounds_violations(void) { return vps::g_violations; }

// Tiles walked since the previous call, by kind (full single run: at least half a tile of
// payload; partial single run; 2-3 runs; 4 or more runs; transpose; element-wise; empty):
// counts and payload bytes, 7 entries each.  Resets the counters.
void vpsh_tile_histogram(uint64_t* counts, uint64_t* bytes)
{
    for (int i = 0; i < vps::TK_KINDS; ++i) {
        counts[i] = vps::g_hist_count[i];
        bytes[i] = vps::g_hist_bytes[i];
        vps::g_hist_count[i] = vps::g_hist_bytes[i] = 0;
    }
}

// Dry-run mode of the copy step (see g_dry_run).  Switching it on clears the recorded writes.
void vpsh_set_dry_run(int on)
{
    vps::g_dry_run = on != 0;
    vps::g_dry_writes.clear();
}

// Bytes written into the address window [lo, hi) since the dry run was switched on; *overlaps =
// number of recorded writes in the window that share a byte with an earlier one.
uint64_t vpsh_dry_run_written(uint64_t lo, uint64_t hi, int64_t* overlaps)
{
    std::vector<vps::Interval> w;
    for (const vps::Interval& i : vps::g_dry_writes)
        if (i.lo >= lo && i.hi <= hi) w.push_back(i);
    std::sort(w.begin(), w.end(), [](const vps::Interval& a, const vps::Interval& b) { return a.lo < b.lo; });
    uint64_t total = 0, reach = 0;
    int64_t bad = 0;
    for (const vps::Interval& i : w) {
        total += i.hi - i.lo;
        if (i.lo < reach) ++bad;
        if (i.hi > reach) reach = i.hi;
    }
    if (overlaps) *overlaps = bad;
    return total;
}

// Single-run tiles walked since the previous call whose destination does not start on a
// multiple of 256 bytes (the buffers of the caller are assumed to).  Resets the counter.
uint64_t vpsh_unaligned_run_tiles(void)
{
    const uint64_t n = vps::g_unaligned_run_tiles;
    vps::g_unaligned_run_tiles = 0;
    return n;
}

// The tensor ids of one group as the planner's per-group lane ranges enumerate them; returns
// their number (ids beyond `max` are not written), or -1 for an illegal description.
int vpsh_group_tensors(const vps_model_desc* m, const vps_parallel_desc* p, int group, int32_t* out, int max)
{
    try {
        vps::check_descs(*m, *p);
    } catch (const vps::Error&) {
        return -1;
    }
    const vps::ParConst P = vps::make_par_const(*m, *p, vps::make_model_const(*m).nt);
    const int n = vps::group_tensor_count(P, group);
    for (int i = 0; i < n && i < max; ++i) out[i] = vps::group_tensor_id(P, group, i);
    return n;
}

// Split a linear range of a row-major array: writes (start, axis, count) triples, returns n.
int vpsh_split_linear_range(const int64_t* dims, uint64_t v0, uint64_t v1, int64_t* out, int max)
{
    int k = 0;
    return vps::split_linear_range(dims, v0, v1, [&](uint64_t start, int axis, uint64_t cnt) {
        if (k < max) { out[3 * k] = (int64_t)start; out[3 * k + 1] = axis; out[3 * k + 2] = (int64_t)cnt; }
        ++k;
    });
}

}  // extern "C"

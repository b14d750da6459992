// vps_backend_hip.h - device backend of the mapper/planner pipeline: one kernel lane per item,
// wavefront ballots and prefix sums for compaction, scans and the radix sort.  No library
// routines: everything that runs on the device is in these headers.
#pragma once

#include <cstdlib>
#include <cstring>

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "vps_copy_kernel.h"
#include "vps_inventory.h"

namespace vps {

#define VPS_HIP_CHECK(expr)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            throw Error{ e_ == hipErrorOutOfMemory ? VPS_ERR_OOM : VPS_ERR_HIP,               \
                         std::string(#expr) + ": " + hipGetErrorString(e_) };                 \
    } while (0)

template <class Step, class F>
__global__ __launch_bounds__(256) void k_for_each(F f, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) f(i);
}

// ---- wavefront and workgroup prefix sums (all 64 lanes of a wavefront must call) ----

template <class V>
__device__ __forceinline__ V wave_exclusive_scan(V v, V& total)
{
    const unsigned lane = threadIdx.x & 63u;
    V x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const V y = __shfl_up(x, d, 64);
        if (lane >= (unsigned)d) x += y;
    }
    total = __shfl(x, 63, 64);
    return x - v;
}

// Exclusive prefix sum over the 256 lanes of a workgroup; `carry` (4 entries of LDS) is scratch.
template <class V>
__device__ __forceinline__ V group_exclusive_scan(V v, V& total, V* carry)
{
    V wtot;
    const V in_wave = wave_exclusive_scan(v, wtot);
    const unsigned wave = threadIdx.x >> 6;
    __syncthreads();   // carry may still be read from the previous round
    if ((threadIdx.x & 63u) == 63u) carry[wave] = wtot;
    __syncthreads();
    V before = 0;
    total = 0;
#pragma unroll
    for (unsigned w = 0; w < 4; ++w) {
        const V c = carry[w];
        if (w < wave) before += c;
        total += c;
    }
    return before + in_wave;
}

// F_P, tensor table and flat offsets: workgroup `cls` walks the tensors of its pipeline stage in
// flat-buffer order, takes each from the closed form of the inventory, and gives every tensor of
// its class its record and the running sum of the shard lengths before it (a workgroup-wide
// prefix sum per 1024 tensors, four consecutive ones per lane); the class length and its padded
// size fall out at the end.  Every tensor belongs to exactly one class, so the table is complete.
__global__ __launch_bounds__(256) void k_layout_classes(ParConst P, ModelConst M, TensorRec* __restrict__ T,
                                                        TensorLayout* __restrict__ TL, ClassRec* __restrict__ C)
{
    __shared__ uint64_t carry[4];
    const int32_t cls = (int32_t)blockIdx.x;
    int32_t lo, hi;
    const int32_t stage = cls < P.pp ? cls : (cls - P.pp) / P.ep;
    stage_tensor_range(P, stage, lo, hi);
    const int32_t count = hi - lo;
    uint64_t running = 0;
    for (int32_t q0 = 0; q0 < count; q0 += 1024) {
        int32_t t[4];
        uint64_t len[4], mine = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int32_t q = q0 + (int32_t)threadIdx.x * 4 + k;
            t[k] = -1;
            len[k] = 0;
            if (q < count) {
                const int32_t id = P.flat_order ? hi - 1 - q : lo + q;
                const TensorRec x = inventory_rec(M, id);
                if (class_of_tensor(P, x) == cls) { t[k] = id; len[k] = shard_elems(P, x); T[id] = x; }
            }
            mine += len[k];
        }
        uint64_t total;
        uint64_t before = running + group_exclusive_scan(mine, total, carry);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (t[k] >= 0) {
                TensorLayout tl;
                tl.start = before; tl.shard_len = len[k]; tl.cls = cls; tl.stage = stage;
                TL[t[k]] = tl;
            }
            before += len[k];
        }
        running += total;
    }
    if (threadIdx.x == 0) C[cls] = make_class_rec(P, cls, running);
}

// A slot of the box table for every lane that is emitting a box right now: a ballot names the
// lanes, the first of them takes the wavefront's share with one atomic, and each lane's slot is
// that base plus the number of emitting lanes below it.
__device__ __forceinline__ uint64_t take_box_slot(unsigned long long* counter)
{
    const uint64_t mask = __ballot(1);
    const unsigned lane = threadIdx.x & 63u;
    const int leader = __ffsll((unsigned long long)mask) - 1;
    const unsigned below = (unsigned)__popcll(mask & ((1ull << lane) - 1ull));
    unsigned long long base = 0;
    if ((int)lane == leader) base = atomicAdd(counter, (unsigned long long)__popcll(mask));
    const unsigned lo = (unsigned)__shfl((int)(unsigned)base, leader, 64);
    const unsigned hi = (unsigned)__shfl((int)(unsigned)(base >> 32), leader, 64);
    return (((uint64_t)hi << 32) | lo) + below;
}

// Intersections with wavefront compaction: every lane walks the routed boxes of its item and
// writes each into the next free slot of the box table, together with its ordering record.
// Boxes beyond the table's capacity are counted but not written.
__global__ __launch_bounds__(256) void k_plan_emit(PlanCtx pc, int mode, int through, int64_t lanes,
                                                   vps_box* __restrict__ raw, OrderRec* __restrict__ recs,
                                                   uint64_t cap, unsigned long long* counter, PairCounts pairs)
{
    // a workgroup walks many lanes: millions of short-lived workgroups would be bound by the rate
    // at which the hardware starts them
    // (`lanes` counts the callers: 2^plan_part_bits(mode) per item lane)
    const int pb = plan_part_bits(mode);
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < lanes; e += (int64_t)gridDim.x * 256)
        plan_lane_boxes(pc, mode, e >> pb, [&](const vps_box& b) {
            const uint64_t k = take_box_slot(counter);
            emit_box(b, make_order_rec(b, pc.ma.T[b.tensor], pc.rank, through != 0), k, raw, recs, cap, pairs);
        }, (int)(e & ((1 << pb) - 1)), 1 << pb);
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask)
{
    const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, mask, 64);
    const unsigned hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), mask, 64);
    return ((uint64_t)hi << 32) | lo;
}

// The same in two launches, for item grids of millions of lanes of which few have work: the
// first writes the indices of the lanes that pass the cheap tests into a list, the second walks
// the list with every lane busy.
//
// Appending to the list: every wavefront collects its entries in LDS and moves them to the list 64
// at a time; what is left at the end goes out with one reservation for the whole workgroup.  The
// list's counter is one address, and atomics on one address are served one after the other (a
// few ns each): an atomic per ballot, or per wavefront at the end of tens of thousands of
// wavefronts, would take longer than the tests themselves.
struct LaneListAppender {
    uint64_t (*staged)[128];
    uint32_t* left;               // [4] entries the wavefronts hold at the end
    unsigned long long* wg_base;
    uint64_t* list;
    uint64_t cap;
    unsigned long long* count;
    uint32_t held = 0;            // entries of staged[wave], the same in every lane

    __device__ void add(bool pass, uint64_t value)
    {
        const unsigned wave = threadIdx.x >> 6, lid = threadIdx.x & 63u;
        const uint64_t mask = __ballot(pass ? 1 : 0);
        if (pass) staged[wave][held + (uint32_t)__popcll(mask & ((1ull << lid) - 1ull))] = value;
        held += (uint32_t)__popcll(mask);
        if (held >= 64) {
            unsigned long long base = 0;
            if (lid == 0) base = atomicAdd(count, 64ull);
            const unsigned lo = (unsigned)__shfl((int)(unsigned)base, 0, 64), hi = (unsigned)__shfl((int)(unsigned)(base >> 32), 0, 64);
            const uint64_t k = (((uint64_t)hi << 32) | lo) + lid;
            if (k < cap) list[k] = staged[wave][lid];
            const uint64_t moved = lid < held - 64 ? staged[wave][64 + lid] : 0;
            if (lid < held - 64) staged[wave][lid] = moved;
            held -= 64;
        }
    }
    // every lane of the workgroup calls this once, after its last add
    __device__ void finish()
    {
        const unsigned wave = threadIdx.x >> 6, lid = threadIdx.x & 63u;
        if (lid == 0) left[wave] = held;
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t total = left[0] + left[1] + left[2] + left[3];
            *wg_base = total ? atomicAdd(count, (unsigned long long)total) : 0ull;
        }
        __syncthreads();
        uint64_t k = *wg_base + lid;
        for (unsigned w = 0; w < wave; ++w) k += left[w];
        if (lid < held && k < cap) list[k] = staged[wave][lid];
    }
};

#define VPS_LANE_LIST_APPENDER(name, list, cap, count)         \
    __shared__ uint64_t name##_staged[4][128];                   \
    __shared__ uint32_t name##_left[4];                          \
    __shared__ unsigned long long name##_base;                   \
    LaneListAppender name;                                       \
    name.staged = name##_staged; name.left = name##_left; name.wg_base = &name##_base; \
    name.list = list; name.cap = cap; name.count = count

__global__ __launch_bounds__(256) void k_plan_filter(PlanCtx pc, int mode, int64_t lanes, uint64_t* __restrict__ list,
                                                     uint64_t cap, unsigned long long* count)
{
    VPS_LANE_LIST_APPENDER(app, list, cap, count);
    for (int64_t first = (int64_t)blockIdx.x * 256; first < lanes; first += (int64_t)gridDim.x * 256) {
        const int64_t lane = first + threadIdx.x;
        LaneItem it;
        app.add(lane < lanes && plan_lane_decode(pc, mode, lane, it), (uint64_t)lane);
    }
    app.finish();
}

// The filter for all-ranks plans.  A lane index there has power-of-two fields sized for the
// largest group, and a tensor with few destination items and source slots (an expert held by two
// ranks on each side, beside dense state sharded 32 ways) would leave nearly all of its lanes
// idle.  Here the dense tensors and the expert tensors have lane ranges of their own, with
// fields sized for their group (PlanGroupLanes); the entries of the list are the same lane
// indices as k_plan_filter's.
__global__ __launch_bounds__(256) void k_plan_filter_groups(PlanCtx pc, PlanGroupLanes gl, uint64_t* __restrict__ list,
                                                            uint64_t cap, unsigned long long* count)
{
    VPS_LANE_LIST_APPENDER(app, list, cap, count);
    const int64_t lanes = gl.lanes[0] + gl.lanes[1];
    for (int64_t first = (int64_t)blockIdx.x * 256; first < lanes; first += (int64_t)gridDim.x * 256) {
        const int64_t gl_lane = first + threadIdx.x;
        int64_t lane = 0;
        const bool pass = gl_lane < lanes && plan_group_lane_check(pc, gl, gl_lane, lane);
        app.add(pass, (uint64_t)lane);
    }
    app.finish();
}

__global__ __launch_bounds__(256) void k_plan_emit_listed(PlanCtx pc, int mode, int through, const uint64_t* __restrict__ list,
                                                          uint64_t list_cap, const unsigned long long* __restrict__ count,
                                                          vps_box* __restrict__ raw, OrderRec* __restrict__ recs,
                                                          uint64_t cap, unsigned long long* counter, PairCounts pairs)
{
    uint64_t n = *count;
    if (n > list_cap) return;   // the list overflowed: the caller plans again in one launch
    const int pb = plan_part_bits(mode);
    n <<= pb;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256)
        plan_lane_boxes(pc, mode, (int64_t)list[i >> pb], [&](const vps_box& b) {
            const uint64_t k = take_box_slot(counter);
            emit_box(b, make_order_rec(b, pc.ma.T[b.tensor], pc.rank, through != 0), k, raw, recs, cap, pairs);
        }, (int)(i & ((1u << pb) - 1)), 1 << pb);
}

// Place of every box in the send and in the receive order by counting (order_by_counting).  A
// group of 16 lanes shares one box: the ordering records are staged through LDS 256 at a time,
// every lane of the group counts a sixteenth of them, and a butterfly over the group adds the
// counts up.  f(k, place, part) continues with box k on the group's lanes part = 0 .. 15.
constexpr unsigned ORDER_GROUP = 16;

template <class Step, class P, class F>
__global__ __launch_bounds__(256) void k_order_by_counting(const OrderRec* __restrict__ recs, const uint64_t* __restrict__ nbox,
                                                           uint32_t bound, P pre, F f)
{
    constexpr unsigned BOXES = 256 / ORDER_GROUP;
    __shared__ OrderRec tile[512];
    const uint64_t n64 = *nbox;
    if (n64 > bound || (uint64_t)blockIdx.x * BOXES >= n64) return;   // uniform over the workgroup
    const uint32_t n = (uint32_t)n64, part = threadIdx.x % ORDER_GROUP, k = blockIdx.x * BOXES + threadIdx.x / ORDER_GROUP;
    const uint32_t kk = k < n ? k : n - 1;
    const OrderRec me = recs[kk];
    // what f needs of box k besides its place is asked for now: it arrives while the counting runs
    const auto held = pre(kk, part);
    const uint64_t floor_s = order_owner_floor(me.key_s), floor_r = order_owner_floor(me.key_r);
    OrderPlace o = order_place_zero();
    for (uint32_t q0 = 0; q0 < n; q0 += 512) {
        __syncthreads();
        // (two records per lane, both loads in flight together)
        const uint32_t i0 = q0 + threadIdx.x, i1 = i0 + 256;
        OrderRec r0 = me, r1 = me;
        if (i0 < n) r0 = recs[i0];
        if (i1 < n) r1 = recs[i1];
        if (i0 < n) tile[threadIdx.x] = r0;
        if (i1 < n) tile[threadIdx.x + 256] = r1;
        __syncthreads();
        const uint32_t m = n - q0 < 512u ? n - q0 : 512u;
        for (uint32_t q = part; q < m; q += ORDER_GROUP) order_count_one(tile[q], me, floor_s, floor_r, o);
    }
#pragma unroll
    for (int d = ORDER_GROUP / 2; d >= 1; d >>= 1) {
        o.idx_s += (uint32_t)__shfl_xor((int)o.idx_s, d, 64);
        o.idx_r += (uint32_t)__shfl_xor((int)o.idx_r, d, 64);
        o.gpos_s += shfl_xor_u64(o.gpos_s, d);
        o.gpos_r += shfl_xor_u64(o.gpos_r, d);
        o.base_s += shfl_xor_u64(o.base_s, d);
        o.base_r += shfl_xor_u64(o.base_r, d);
    }
    if (k < n) f(k, o, part, held);
}

// Rank of every record inside its pair's bucket (pair-by-pair ordering of large all-ranks plans):
// the number of records of the bucket that come before it and the buffer bytes of the travelling
// ones among them.  A group of 16 lanes shares one record and walks the bucket 16 records at a
// time; f(j, before, bytes) continues on the group's first lane.  When *work exceeds work_max the
// walk is skipped and a record keeps its place in the bucket (the caller plans again).
template <class Step, class F>
__global__ __launch_bounds__(256) void k_pair_rank(const PairRec* __restrict__ bucket, const uint64_t* __restrict__ pstart,
                                                   const uint64_t* __restrict__ pcount, int64_t n, const uint64_t* work,
                                                   uint64_t work_max, F f)
{
    const unsigned part = threadIdx.x % ORDER_GROUP;
    const int64_t j = (int64_t)blockIdx.x * (256 / ORDER_GROUP) + threadIdx.x / ORDER_GROUP;
    if (j >= n) return;   // whole groups leave together
    const PairRec me = bucket[j];
    const uint64_t pr = me.key >> 26, lo = pstart[pr], cnt = pcount[pr];
    uint32_t before = (uint32_t)((uint64_t)j - lo);
    uint64_t bytes = 0;
    if (*work <= work_max) {
        before = 0;
        for (uint64_t q = lo + part; q < lo + cnt; q += ORDER_GROUP) {
            const PairRec o = bucket[q];
            const bool less = pair_rec_less(o, me);
            before += less ? 1u : 0u;
            bytes += (less && (o.bytes_flags & ORD_SENDS)) ? (o.bytes_flags & ~(uint64_t)15) : 0;
        }
#pragma unroll
        for (int d = ORDER_GROUP / 2; d >= 1; d >>= 1) {
            before += (uint32_t)__shfl_xor((int)before, d, 64);
            bytes += shfl_xor_u64(bytes, d);
        }
    }
    if (part == 0) f(j, (uint64_t)before, bytes);
}

// ---- stable least-significant-digit radix sort of (64-bit key, 32-bit value) pairs, 8 bits per
// pass.  A workgroup owns a tile of SORT_TILE consecutive pairs.  Pass = three launches: digit
// counts per tile (k_sort_count) -> exclusive scan of the table laid out digit-major (all tiles'
// counts of digit 0, then of digit 1, ...: the scanned entry is where the tile's first pair with
// that digit goes) -> k_sort_scatter, which gives every pair its rank among the tile's pairs of
// the same digit.  The rank keeps the input order: the tile is taken in rounds of 256 pairs; in a
// round the lanes of a wavefront find the lanes with their digit by eight ballots (one per bit)
// and count those below them, the wavefronts' counts per digit are added up in wavefront order
// through LDS, and a per-digit counter carries on from round to round.
constexpr int SORT_ROUNDS = 8;
constexpr int SORT_TILE = 256 * SORT_ROUNDS;

__global__ __launch_bounds__(256) void k_sort_count(const uint64_t* __restrict__ keys, int64_t n, int shift, int64_t ntiles,
                                                    int64_t* __restrict__ table)
{
    __shared__ uint32_t hist[256];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SORT_TILE;
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        const int64_t i = base + r * 256 + threadIdx.x;
        if (i < n) atomicAdd(&hist[(uint32_t)(keys[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    table[(int64_t)threadIdx.x * ntiles + blockIdx.x] = hist[threadIdx.x];
    if (blockIdx.x == 0 && threadIdx.x == 0) table[256 * ntiles] = 0;   // the scan's closing entry
}

__global__ __launch_bounds__(256) void k_sort_scatter(const uint64_t* __restrict__ keys, const uint32_t* __restrict__ vals,
                                                      int64_t n, int shift, int64_t ntiles, const int64_t* __restrict__ start,
                                                      uint64_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out)
{
    __shared__ uint32_t seen[256];        // pairs of the tile with this digit in the rounds so far
    __shared__ uint32_t wave_cnt[4][256]; // this round: pairs with this digit per wavefront
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    seen[threadIdx.x] = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) wave_cnt[w][threadIdx.x] = 0;
    __syncthreads();
    const int64_t first = start[(int64_t)threadIdx.x * ntiles + blockIdx.x];   // thread d: where digit d of this tile starts
    __shared__ int64_t digit_start[256];
    digit_start[threadIdx.x] = first;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SORT_TILE;
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        const int64_t i = base + r * 256 + threadIdx.x;
        const bool valid = i < n;
        const uint64_t key = valid ? keys[i] : 0;
        const uint32_t digit = (uint32_t)(key >> shift) & 255u;
        // lanes of this wavefront with the same digit
        uint64_t peers = __ballot(valid ? 1 : 0);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t m = __ballot((digit >> b) & 1u);
            peers &= ((digit >> b) & 1u) ? m : ~m;
        }
        const uint32_t below = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        if (valid && below == 0) wave_cnt[wave][digit] = (uint32_t)__popcll(peers);   // the first lane of its digit
        __syncthreads();
        if (valid) {
            uint32_t rank = seen[digit] + below;
            for (unsigned w = 0; w < wave; ++w) rank += wave_cnt[w][digit];
            const int64_t to = digit_start[digit] + rank;
            keys_out[to] = key;
            vals_out[to] = vals[i];
        }
        __syncthreads();
        {   // thread d closes digit d of this round
            uint32_t add = 0;
#pragma unroll
            for (int w = 0; w < 4; ++w) { add += wave_cnt[w][threadIdx.x]; wave_cnt[w][threadIdx.x] = 0; }
            seen[threadIdx.x] += add;
        }
        __syncthreads();
    }
}

// The tile table: one lane per tile builds its record from the tile's descriptor.  Finding the
// descriptor is a search in the table of tile bases; a workgroup's consecutive tiles lie
// between the descriptors of its first and of its last tile, which are the same for the whole
// workgroup: those two searches run on the scalar unit (the bases are read through the constant
// address space; ten dependent loads from the scalar cache instead of from L2), and a lane then
// only searches between them, which mostly is no step at all.  nbox < 0: the number of boxes is
// n_host; else it is read from *nbox and the kernel leaves when it exceeds `bound`.
// (kept out of line: inlined beside the call with the descriptor in registers, the two would be
// merged into one body that reads its descriptor through a pointer, i.e. from scratch memory)
__device__ __noinline__ TileRef make_tile_from_table(const CopyDesc* descs, uint32_t di, uint32_t q)
{
    return make_tile(descs[di], di, q);
}

constexpr int TILE_TABLE_ROUNDS = 4;   // a workgroup writes this many stretches of 256 records
__global__ __launch_bounds__(256) void k_tile_table(const int64_t* __restrict__ tbase, const CopyDesc* __restrict__ descs,
                                                    const uint64_t* nbox, int64_t n_host, int64_t bound, TileRef* __restrict__ tiles,
                                                    int64_t cap)
{
    typedef const __attribute__((address_space(4))) int64_t* cbase_t;
    const int64_t n = nbox ? (int64_t)*(const __attribute__((address_space(4))) uint64_t*)(uintptr_t)nbox : n_host;
    if (nbox && n > bound) return;
    const cbase_t tb = (cbase_t)(uintptr_t)tbase;
    const int64_t nd = 3 * n;
    const int64_t total = tb[nd] < cap ? tb[nd] : cap;
    const int64_t g0 = (int64_t)blockIdx.x * (256 * TILE_TABLE_ROUNDS);
    if (g0 >= total) return;
    const int64_t g1 = g0 + 256 * TILE_TABLE_ROUNDS - 1 < total ? g0 + 256 * TILE_TABLE_ROUNDS - 1 : total - 1;
    auto last_not_above = [&](int64_t t, int64_t lo) {   // the descriptor that holds tile t: last d >= lo - 1 with tb[d] <= t
        int64_t hi = nd + 1;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (tb[mid] <= t) lo = mid + 1; else hi = mid;
        }
        return lo - 1;
    };
    // (a descriptor of a long run has thousands of tiles: mostly the workgroup's last tile lies in
    // the same one, which a single load shows)
    const int64_t d_first = last_not_above(g0, 0);
    const int64_t d_last = tb[d_first + 1] > g1 ? d_first : last_not_above(g1, d_first + 2);
    // The 48-byte records of the workgroup go through LDS so that the table is written in whole
    // lines: a lane storing its own record would touch every third 16-byte piece, and each of its
    // three stores would open every line of the wavefront's stretch again.
    static_assert(sizeof(TileRef) == 48, "three 16-byte vectors per record");
    __shared__ __attribute__((aligned(16))) TileRef staged[256];
    // One descriptor of runs for the whole workgroup (the usual case): it is read once, with scalar
    // loads, instead of by every lane.
    CopyDesc one = CopyDesc();
    const int64_t first_base = tb[d_first];
    bool one_of_runs = false;
    if (d_first == d_last) {
        // (field by field, and only what make_run_tile reads: a struct assignment would go through
        // scratch memory)
        const __attribute__((address_space(4))) CopyDesc* c = (const __attribute__((address_space(4))) CopyDesc*)(uintptr_t)(descs + d_first);
        one.mode = c->mode;
        one_of_runs = one.mode == MODE_RUN;
        one.src_byte = c->src_byte; one.dst_byte = c->dst_byte;
#pragma unroll
        for (int a = 0; a < 4; ++a) { one.sstr[a] = c->sstr[a]; one.dstr[a] = c->dstr[a]; one.ext[a] = c->ext[a]; }
        one.src_slot = c->src_slot; one.dst_slot = c->dst_slot; one.alt_src_slot = c->alt_src_slot;
        one.es = c->es; one.alt_src_byte = c->alt_src_byte;
        one.rows_per_tile = c->rows_per_tile; one.vec_window = c->vec_window;
        one.chunks_per_row = c->chunks_per_row; one.xa = c->xa;
    }
    for (int64_t t0 = g0; t0 <= g1; t0 += 256) {
        const int64_t t = t0 + threadIdx.x;
        if (t0 > g0) __syncthreads();   // the stretch before has left the staging area
        if (t < total) {
            if (one_of_runs) {
                staged[threadIdx.x] = make_run_tile(one, (uint32_t)(t - first_base));
            } else {
                int64_t lo = d_first, hi = d_last + 1;    // the lane's own descriptor lies in [d_first, d_last]
                while (hi - lo > 1) {
                    const int64_t mid = (lo + hi) >> 1;
                    if (tbase[mid] <= t) lo = mid; else hi = mid;
                }
                staged[threadIdx.x] = make_tile_from_table(descs, (uint32_t)lo, (uint32_t)(t - tbase[lo]));
            }
        }
        __syncthreads();
        const uint32_t nvec = 3u * (uint32_t)(total - t0 < 256 ? total - t0 : 256);
        const u32x4* from = reinterpret_cast<const u32x4*>(staged);
        u32x4* to = reinterpret_cast<u32x4*>(tiles + t0);
        for (uint32_t v = threadIdx.x; v < nvec; v += 256) to[v] = from[v];
    }
}

// ---- exclusive prefix sum of n int64 values: out[i] = in[0] + ... + in[i-1] ----
constexpr int SCAN_PER_LANE = 8;
constexpr int SCAN_PER_GROUP = 256 * SCAN_PER_LANE;

// One workgroup walks the whole array (small inputs, and the table of workgroup sums).
__device__ __forceinline__ void scan_by_one_group(const int64_t* in, int64_t* out, int64_t n)
{
    __shared__ int64_t carry[4];
    int64_t running = 0;
    for (int64_t base = 0; base < n; base += SCAN_PER_GROUP) {
        const int64_t i0 = base + (int64_t)threadIdx.x * SCAN_PER_LANE;
        int64_t v[SCAN_PER_LANE], mine = 0;
#pragma unroll
        for (int k = 0; k < SCAN_PER_LANE; ++k) { v[k] = i0 + k < n ? in[i0 + k] : 0; mine += v[k]; }
        int64_t total;
        int64_t acc = running + group_exclusive_scan(mine, total, carry);
#pragma unroll
        for (int k = 0; k < SCAN_PER_LANE; ++k) { if (i0 + k < n) out[i0 + k] = acc; acc += v[k]; }
        running += total;
    }
}

__global__ __launch_bounds__(256) void k_scan_one_group(const int64_t* in, int64_t* out, int64_t n)
{
    scan_by_one_group(in, out, n);
}

__global__ __launch_bounds__(256) void k_zero_words(uint64_t* __restrict__ p, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) p[i] = 0;
}

// Several short arrays at a constant distance from each other, one workgroup each.
__global__ __launch_bounds__(256) void k_scan_rows(const int64_t* in, int64_t* out, int64_t n, int64_t stride)
{
    scan_by_one_group(in + (int64_t)blockIdx.x * stride, out + (int64_t)blockIdx.x * stride, n);
}

// The same over the first mult * (*count) + 1 entries (at most n; no sums beyond); then the nrows
// rows of row_len counters at `rows` become their own exclusive prefix sums, in place; then, in
// the same workgroup, f(i) for i in [0, m): the per-rank tables that read the sums.  At the end
// the `words` 64-bit words at `blk` (the plan's summary block) are copied to `mirror`, which is
// pinned host memory: the host reads them after its wait, without a copy command of its own; and
// as many words at `clear` (if not null) are set to zero: the summary block of the next plan.
template <class Step, class F>
__global__ __launch_bounds__(256) void k_scan_counted_then_each(const int64_t* in, int64_t* out, int64_t n,
                                                                const uint64_t* count, int mult, int64_t* rows,
                                                                int64_t row_len, int nrows, int64_t m, F f,
                                                                const uint64_t* blk, uint64_t* mirror, int64_t words,
                                                                uint64_t* clear)
{
    if (clear)
        for (int64_t i = threadIdx.x; i < words; i += 256) clear[i] = 0;
    const int64_t len = (int64_t)*count * mult + 1;
    if (len <= n) {   // (uniform over the workgroup)
        scan_by_one_group(in, out, len);
        for (int r = 0; r < nrows; ++r) {
            __syncthreads();   // the carries of the scan before are free again
            scan_by_one_group(rows + r * row_len, rows + r * row_len, row_len);
        }
        __syncthreads();   // the sums are in memory for every lane of the workgroup
        for (int64_t i = threadIdx.x; i < m; i += 256) f(i);
        __syncthreads();   // and so is what f wrote into the block
    }
    for (int64_t i = threadIdx.x; i < words; i += 256) mirror[i] = blk[i];
}

__global__ __launch_bounds__(256) void k_scan_group_sums(const int64_t* in, int64_t* sums, int64_t n)
{
    __shared__ int64_t carry[4];
    const int64_t i0 = (int64_t)blockIdx.x * SCAN_PER_GROUP + (int64_t)threadIdx.x * SCAN_PER_LANE;
    int64_t mine = 0;
#pragma unroll
    for (int k = 0; k < SCAN_PER_LANE; ++k) mine += i0 + k < n ? in[i0 + k] : 0;
    int64_t total;
    group_exclusive_scan(mine, total, carry);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void k_scan_with_offsets(const int64_t* in, int64_t* out, const int64_t* offsets, int64_t n)
{
    __shared__ int64_t carry[4];
    const int64_t i0 = (int64_t)blockIdx.x * SCAN_PER_GROUP + (int64_t)threadIdx.x * SCAN_PER_LANE;
    int64_t v[SCAN_PER_LANE], mine = 0;
#pragma unroll
    for (int k = 0; k < SCAN_PER_LANE; ++k) { v[k] = i0 + k < n ? in[i0 + k] : 0; mine += v[k]; }
    int64_t total;
    int64_t acc = offsets[blockIdx.x] + group_exclusive_scan(mine, total, carry);
#pragma unroll
    for (int k = 0; k < SCAN_PER_LANE; ++k) { if (i0 + k < n) out[i0 + k] = acc; acc += v[k]; }
}

// Pointer tables travel as kernel arguments: the launch copies them, so the host array can be
// reused at once and nothing waits on the stream.
struct PtrChunk {
    char* p[384];
};

__global__ void k_set_ptrs(char** table, int offset, int count, PtrChunk chunk)
{
    const int i = threadIdx.x + blockIdx.x * blockDim.x;
    if (i < count) table[offset + i] = chunk.p[i];
}

// Device memory for the library's own tables (never payload).  hipMalloc/hipFree cost tens of
// microseconds and hipFree waits for the device, so freed blocks are kept in power-of-two size
// classes and handed out again.  Every mapper/planner step runs on one stream and the builders
// synchronise that stream before they return, so a block is only ever reused after the work
// that touched it has finished.  Blocks still referenced by queued copy kernels are returned by
// vps_plan_destroy, which waits for the device first.
struct DeviceAlloc {
    static hipError_t alloc(void** p, size_t n) { return hipMalloc(p, n); }
    static void release(void* p) { (void)hipFree(p); }
};
// Pinned host memory: device-to-host copies into it are truly asynchronous.
struct PinnedAlloc {
    static hipError_t alloc(void** p, size_t n) { return hipHostMalloc(p, n, hipHostMallocDefault); }
    static void release(void* p) { (void)hipHostFree(p); }
};

template <class Alloc>
class BlockPool {
public:
    static BlockPool& get()
    {
        static BlockPool pool;
        return pool;
    }

    void* take(size_t bytes, size_t& cls_bytes)
    {
        int cls = 8;  // 256 bytes
        while (((size_t)1 << cls) < bytes) ++cls;
        cls_bytes = (size_t)1 << cls;
        {
            std::lock_guard<std::mutex> g(m_);
            if (!free_[cls].empty()) {
                void* p = free_[cls].back();
                free_[cls].pop_back();
                cached_bytes_ -= cls_bytes;
                return p;
            }
        }
        void* p = nullptr;
        hipError_t e = Alloc::alloc(&p, cls_bytes);
        if (e != hipSuccess) {
            trim();  // give cached blocks back and retry once
            e = Alloc::alloc(&p, cls_bytes);
        }
        if (e != hipSuccess)
            throw Error{ e == hipErrorOutOfMemory ? VPS_ERR_OOM : VPS_ERR_HIP,
                         std::string("allocation of library tables: ") + hipGetErrorString(e) };
        std::lock_guard<std::mutex> g(m_);
        size_of_[p] = cls;
        return p;
    }

    void give(void* p)
    {
        std::lock_guard<std::mutex> g(m_);
        auto it = size_of_.find(p);
        if (it == size_of_.end()) return;
        const int cls = it->second;
        // keep at most 1 GiB of idle blocks
        if (cached_bytes_ + ((size_t)1 << cls) > ((size_t)1 << 30)) {
            size_of_.erase(it);
            Alloc::release(p);
            return;
        }
        free_[cls].push_back(p);
        cached_bytes_ += (size_t)1 << cls;
    }

    void trim()
    {
        std::lock_guard<std::mutex> g(m_);
        for (int c = 0; c < 48; ++c) {
            for (void* p : free_[c]) { size_of_.erase(p); Alloc::release(p); }
            free_[c].clear();
        }
        cached_bytes_ = 0;
    }

private:
    std::mutex m_;
    std::vector<void*> free_[48];
    std::unordered_map<void*, int> size_of_;
    size_t cached_bytes_ = 0;
};

typedef BlockPool<DeviceAlloc> DevicePool;
typedef BlockPool<PinnedAlloc> PinnedPool;

class HipBackend {
public:
    explicit HipBackend(void* s) : stream_((hipStream_t)s) {}
    ~HipBackend() { release_all(); }

    template <class T>
    T* alloc(int64_t n)
    {
        size_t got = 0;
        void* p = DevicePool::get().take(sizeof(T) * (size_t)(n > 0 ? n : 1), got);
        live_.push_back(p);
        return (T*)p;
    }

    // Temporaries of a build: the stream still has work queued on them, so they go back to the
    // pool only when the build ends (commit / release_all, after a stream synchronisation).
    void free(void* p)
    {
        if (!p) return;
        auto it = std::find(live_.begin(), live_.end(), p);
        if (it != live_.end()) {
            live_.erase(it);
            dead_.push_back(p);
        } else {
            // a block owned by a handle that is being destroyed
            DevicePool::get().give(p);
        }
    }

    // Hand the remaining allocations over to the caller (the handle now owns them).
    void commit()
    {
        live_.clear();
        recycle_dead();
    }

    void release_all()
    {
        if (live_.empty() && dead_.empty() && stages_.empty() && !pending_zeroed_.p) return;
        (void)hipStreamSynchronize(stream_);
        if (pending_zeroed_.p) { DevicePool::get().give(pending_zeroed_.p); pending_zeroed_.p = nullptr; }
        for (const Stage& st : stages_) PinnedPool::get().give(st.pinned);
        stages_.clear();
        for (void* p : live_) DevicePool::get().give(p);
        live_.clear();
        recycle_dead();
    }

    template <class Step, class F>
    void for_each(Step, int64_t n, F f)
    {
        if (n <= 0) return;
        const int64_t blocks = (n + 255) / 256;
        if (blocks > 0x7fffffffLL) throw Error{ VPS_ERR_OOM, "step has too many items" };
        hipLaunchKernelGGL((k_for_each<Step, F>), dim3((unsigned)blocks), dim3(256), 0, stream_, f, n);
        VPS_HIP_CHECK(hipGetLastError());
    }

    // out[i] = in[0] + ... + in[i-1] for i in [0, n]; both arrays hold n+1 entries and in[n]
    // must be 0.  Up to 8 Ki entries one workgroup walks the array; beyond, every workgroup sums
    // its 2048 entries, one workgroup scans those sums, and a third launch finishes.
    void exclusive_scan(const int64_t* in, int64_t* out, int64_t n)
    {
        const int64_t count = n + 1;
        if (count <= 4 * SCAN_PER_GROUP) {
            hipLaunchKernelGGL(k_scan_one_group, dim3(1), dim3(256), 0, stream_, in, out, count);
            VPS_HIP_CHECK(hipGetLastError());
            return;
        }
        const int64_t groups = (count + SCAN_PER_GROUP - 1) / SCAN_PER_GROUP;
        int64_t* sums = alloc<int64_t>(groups);
        hipLaunchKernelGGL(k_scan_group_sums, dim3((unsigned)groups), dim3(256), 0, stream_, in, sums, count);
        hipLaunchKernelGGL(k_scan_one_group, dim3(1), dim3(256), 0, stream_, (const int64_t*)sums, sums, groups);
        hipLaunchKernelGGL(k_scan_with_offsets, dim3((unsigned)groups), dim3(256), 0, stream_, in, out, (const int64_t*)sums, count);
        VPS_HIP_CHECK(hipGetLastError());
        free(sums);
    }

    // exclusive_scan(in + r * stride, out + r * stride, n) for r in [0, rows), in one launch.
    void exclusive_scan_rows(const int64_t* in, int64_t* out, int64_t n, int64_t stride, int rows)
    {
        if (n + 1 > 4 * SCAN_PER_GROUP) {
            for (int r = 0; r < rows; ++r) exclusive_scan(in + r * stride, out + r * stride, n);
            return;
        }
        hipLaunchKernelGGL(k_scan_rows, dim3((unsigned)rows), dim3(256), 0, stream_, in, out, n + 1, stride);
        VPS_HIP_CHECK(hipGetLastError());
    }

    // The same over the first mult * (*count) + 1 entries, *count read on the device (at most
    // `bound` entries; nothing happens if there would be more), followed in the same launch by
    // f(i) for i in [0, m).
    template <class Step, class F>
    void exclusive_scan_counted_then_each(Step, const int64_t* in, int64_t* out, int64_t bound, const uint64_t* count,
                                          int mult, int64_t* rows, int64_t row_len, int nrows, int64_t m, F f,
                                          const uint64_t* blk, uint64_t* mirror, int64_t words)
    {
        // (the block of the next plan is cleared here, see alloc_zeroed)
        uint64_t* clear = words > 0 ? (uint64_t*)next_zeroed(sizeof(uint64_t) * (size_t)words) : nullptr;
        hipLaunchKernelGGL((k_scan_counted_then_each<Step, F>), dim3(1), dim3(256), 0, stream_, in, out, bound, count, mult, rows,
                           row_len, nrows, m, f, blk, mirror, words, clear);
        VPS_HIP_CHECK(hipGetLastError());
    }

    // f(k, place, part, pre(k, part)) for every box k < *nbox (at most `bound` boxes) and
    // part = 0 .. 15, place = order_by_counting; pre is evaluated before the counting.
    template <class Step, class P, class F>
    void order_by_counting_each(Step, const OrderRec* recs, const uint64_t* nbox, int64_t bound, P pre, F f)
    {
        const int64_t per = 256 / ORDER_GROUP;
        const int64_t blocks = (bound + per - 1) / per;
        hipLaunchKernelGGL((k_order_by_counting<Step, P, F>), dim3((unsigned)blocks), dim3(256), 0, stream_, recs, nbox, (uint32_t)bound,
                           pre, f);
        VPS_HIP_CHECK(hipGetLastError());
    }

    // tiles[t] for every tile t < min(tile_base[3n], cap), n = *nbox (skipped when n > bound) or,
    // with nbox = nullptr, n = n_host.  `lanes` tiles are launched.
    void tile_table(const int64_t* tile_base, const CopyDesc* descs, const uint64_t* nbox, int64_t n_host, int64_t bound,
                    TileRef* tiles, int64_t cap, int64_t lanes)
    {
        if (lanes <= 0) return;
        const int64_t per = 256 * TILE_TABLE_ROUNDS;
        hipLaunchKernelGGL(k_tile_table, dim3((unsigned)((lanes + per - 1) / per)), dim3(256), 0, stream_, tile_base, descs, nbox, n_host,
                           bound, tiles, cap);
        VPS_HIP_CHECK(hipGetLastError());
    }

    // f(j, before, bytes) for every record j of the pair buckets: see k_pair_rank.
    template <class Step, class F>
    void pair_rank_each(Step, const PairRec* bucket, const uint64_t* pstart, const uint64_t* pcount, int64_t n,
                        const uint64_t* work, uint64_t work_max, F f)
    {
        if (n <= 0) return;
        const int64_t per = 256 / ORDER_GROUP;
        hipLaunchKernelGGL((k_pair_rank<Step, F>), dim3((unsigned)((n + per - 1) / per)), dim3(256), 0, stream_, bucket, pstart,
                           pcount, n, work, work_max, f);
        VPS_HIP_CHECK(hipGetLastError());
    }

    void layout_classes(const ParConst& P, const ModelConst& M, TensorRec* T, TensorLayout* TL, ClassRec* C)
    {
        hipLaunchKernelGGL(k_layout_classes, dim3((unsigned)P.ncls), dim3(256), 0, stream_, P, M, T, TL, C);
        VPS_HIP_CHECK(hipGetLastError());
    }

    // `listed` (one 64-bit word, cleared by the caller) receives the length of the lane list when
    // the two-launch form is used; more than PLAN_LIST_CAP means that the list overflowed and
    // nothing was emitted: the caller then calls again with two_launches = false.
    static constexpr uint64_t PLAN_LIST_CAP = 1ull << 22;
    static constexpr int64_t PLAN_LIST_FROM = 1ll << 17;   // item grids from this many lanes on use the list
    static constexpr int64_t PLAN_LIST_FROM_ALL = 1ll << 13;   // the same for all-ranks plans

    bool plan_emit(const PlanCtx& pc, int mode, bool through, vps_box* raw, OrderRec* recs, uint64_t cap, uint64_t* counter,
                   uint64_t* listed, bool two_launches, const PairCounts& pairs)
    {
        const int64_t lanes = plan_num_lanes(pc, mode);
        if (lanes <= 0) return false;
        int64_t blocks = (lanes + 255) / 256;
        if (blocks > 8192) blocks = 8192;   // the kernels stride over the lanes
        if (two_launches && lanes >= (mode == PLAN_ALL ? PLAN_LIST_FROM_ALL : PLAN_LIST_FROM)) {
            uint64_t* list = alloc<uint64_t>((int64_t)PLAN_LIST_CAP);
            if (mode == PLAN_ALL) {
                const PlanGroupLanes gl = plan_group_lanes(pc);
                int64_t fb = (gl.lanes[0] + gl.lanes[1] + 255) / 256;
                if (fb > 2048) fb = 2048;   // the kernel strides over the lanes; few workgroups, few reservations
                if (fb < 1) fb = 1;
                hipLaunchKernelGGL(k_plan_filter_groups, dim3((unsigned)fb), dim3(256), 0, stream_, pc, gl, list,
                                   PLAN_LIST_CAP, (unsigned long long*)listed);
            } else {
                hipLaunchKernelGGL(k_plan_filter, dim3((unsigned)(blocks > 2048 ? 2048 : blocks)), dim3(256), 0, stream_, pc, mode, lanes,
                                   list, PLAN_LIST_CAP, (unsigned long long*)listed);
            }
            hipLaunchKernelGGL(k_plan_emit_listed, dim3(2048), dim3(256), 0, stream_, pc, mode, through ? 1 : 0,
                               (const uint64_t*)list, PLAN_LIST_CAP, (const unsigned long long*)listed, raw, recs, cap,
                               (unsigned long long*)counter, pairs);
            VPS_HIP_CHECK(hipGetLastError());
            free(list);
            return true;
        }
        const int64_t callers = lanes << plan_part_bits(mode);
        blocks = (callers + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(k_plan_emit, dim3((unsigned)blocks), dim3(256), 0, stream_, pc, mode, through ? 1 : 0, callers,
                           raw, recs, cap, (unsigned long long*)counter, pairs);
        VPS_HIP_CHECK(hipGetLastError());
        return false;
    }

    // Work queued on the null stream so far (the mapping kernels of vps_describe_config) comes
    // before what this backend's stream runs next.  A blocking stream is ordered against the null
    // stream by the runtime; any other stream waits for an event.
    void after_null_stream()
    {
        if (!stream_) return;
        unsigned flags = 0;
        if (hipStreamGetFlags(stream_, &flags) == hipSuccess && !(flags & hipStreamNonBlocking)) return;
        static thread_local hipEvent_t ev = nullptr;
        if (!ev) VPS_HIP_CHECK(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        VPS_HIP_CHECK(hipEventRecord(ev, nullptr));
        VPS_HIP_CHECK(hipStreamWaitEvent(stream_, ev, 0));
    }


    // Stable ascending sort of (key, value) pairs.  The arrays are passed by reference: after the
    // call they point at the sorted data (the sort ping-pongs between the inputs and two
    // scratch arrays instead of copying back).
    // Only the low `bits` bits of the keys are significant.
    void sort_pairs(uint64_t*& keys, uint32_t*& vals, int64_t n, int bits = 64)
    {
        if (n <= 1) return;
        uint64_t* k2 = alloc<uint64_t>(n);
        uint32_t* v2 = alloc<uint32_t>(n);
        const int64_t ntiles = (n + SORT_TILE - 1) / SORT_TILE;
        int64_t* count = alloc<int64_t>(256 * ntiles + 1);
        int64_t* start = alloc<int64_t>(256 * ntiles + 1);
        for (int shift = 0; shift < bits; shift += 8) {
            hipLaunchKernelGGL(k_sort_count, dim3((unsigned)ntiles), dim3(256), 0, stream_, (const uint64_t*)keys, n, shift, ntiles, count);
            VPS_HIP_CHECK(hipGetLastError());
            exclusive_scan(count, start, 256 * ntiles);
            hipLaunchKernelGGL(k_sort_scatter, dim3((unsigned)ntiles), dim3(256), 0, stream_, (const uint64_t*)keys,
                               (const uint32_t*)vals, n, shift, ntiles, (const int64_t*)start, k2, v2);
            VPS_HIP_CHECK(hipGetLastError());
            std::swap(keys, k2);
            std::swap(vals, v2);
        }
        free(count); free(start); free(k2); free(v2);
    }

    // The host array must stay valid until the next sync(); builders keep it alive.
    void upload(void* dev, const void* host, size_t bytes)
    {
        if (!bytes) return;
        size_t got = 0;
        void* stage = PinnedPool::get().take(bytes, got);
        stages_.push_back(Stage{ nullptr, stage, 0 });
        memcpy(stage, host, bytes);
        VPS_HIP_CHECK(hipMemcpyAsync(dev, stage, bytes, hipMemcpyHostToDevice, stream_));
    }

    // Pinned host memory that a kernel of this stream writes: its first `bytes` bytes arrive in
    // `host` at the next sync().
    void* host_mirror(void* host, size_t bytes)
    {
        size_t got = 0;
        void* stage = PinnedPool::get().take(bytes ? bytes : 1, got);
        stages_.push_back(Stage{ host, stage, bytes });
        return stage;
    }

    // A block of device memory that holds zeros.  Clearing it is a command of its own with a
    // launch of its own, at the very start of a plan, when the device has nothing else to do; so
    // a plan's last small kernel clears the block of the *next* plan on the side (next_zeroed
    // hands it the block), and the block is published at the plan's wait, after which the
    // clearing has certainly happened.
    void* alloc_zeroed(size_t bytes)
    {
        void* p = nullptr;
        {
            std::lock_guard<std::mutex> g(zeroed_mutex());
            ZeroedBlock& z = zeroed_slot();
            if (z.p && z.bytes == bytes) { p = z.p; z.p = nullptr; }
        }
        if (p) { live_.push_back(p); return p; }
        p = alloc<uint8_t>((int64_t)bytes);
        zero(p, bytes);
        return p;
    }

    // The block that a kernel launched next on this stream is going to clear, or nullptr when a
    // cleared block of this size is waiting already.
    void* next_zeroed(size_t bytes)
    {
        if (pending_zeroed_.p) return nullptr;
        {
            std::lock_guard<std::mutex> g(zeroed_mutex());
            const ZeroedBlock& z = zeroed_slot();
            if (z.p && z.bytes == bytes) return nullptr;
        }
        size_t got = 0;
        pending_zeroed_.p = DevicePool::get().take(bytes, got);
        pending_zeroed_.bytes = bytes;
        return pending_zeroed_.p;
    }

    // Needed at once (a count that sizes the next allocation).
    void download(void* host, const void* dev, size_t bytes)
    {
        download_later(host, dev, bytes);
        sync();
    }

    // Arrives in `host` at the next sync().
    void download_later(void* host, const void* dev, size_t bytes)
    {
        if (!bytes) return;
        size_t got = 0;
        void* stage = PinnedPool::get().take(bytes, got);
        stages_.push_back(Stage{ host, stage, bytes });
        VPS_HIP_CHECK(hipMemcpyAsync(stage, dev, bytes, hipMemcpyDeviceToHost, stream_));
    }

    // (a kernel of this library when the range is a whole number of aligned 64-bit words, which
    // the planner's tables are: the runtime's memset costs the host three times a kernel launch,
    // and a large plan clears several small tables between its passes)
    void zero(void* dev, size_t bytes)
    {
        if (!bytes) return;
        if (((uintptr_t)dev | bytes) & 7u) {
            VPS_HIP_CHECK(hipMemsetAsync(dev, 0, bytes, stream_));
            return;
        }
        const uint64_t words = bytes / 8;
        uint64_t blocks = (words + 1023) / 1024;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_zero_words, dim3((unsigned)blocks), dim3(256), 0, stream_, (uint64_t*)dev, words);
        VPS_HIP_CHECK(hipGetLastError());
    }

    void sync()
    {
        const hipError_t e = hipStreamSynchronize(stream_);
        for (const Stage& st : stages_) {
            if (e == hipSuccess && st.host) memcpy(st.host, st.pinned, st.bytes);
            PinnedPool::get().give(st.pinned);
        }
        stages_.clear();
        if (pending_zeroed_.p) {
            // cleared by now (or never, after an error): publish it, or put it back
            void* back = pending_zeroed_.p;
            if (e == hipSuccess) {
                std::lock_guard<std::mutex> g(zeroed_mutex());
                ZeroedBlock& z = zeroed_slot();
                back = z.p;   // a block of another size that nobody took
                z = pending_zeroed_;
            }
            pending_zeroed_.p = nullptr;
            if (back) DevicePool::get().give(back);
        }
        VPS_HIP_CHECK(e);
    }

    void set_ptr_table(void** table, void* const* host_ptrs, int n)
    {
        for (int off = 0; off < n; off += 384) {
            PtrChunk c;
            const int cnt = n - off < 384 ? n - off : 384;
            for (int i = 0; i < cnt; ++i) c.p[i] = (char*)host_ptrs[off + i];
            hipLaunchKernelGGL(k_set_ptrs, dim3(2), dim3(192), 0, stream_, (char**)table, off, cnt, c);
            VPS_HIP_CHECK(hipGetLastError());
        }
    }

    // A dispatch holds fewer than 2^32 work-items per dimension, i.e. fewer than 2^24 workgroups
    // of 256 lanes: larger tile ranges go out as several launches (a multiple of every XCD run
    // length per launch, so the block -> tile order is the same as in one launch).
    static constexpr int64_t MAX_GROUPS_PER_LAUNCH = (int64_t)1 << 23;

    void launch_copy(const CopyDesc* descs, const TileRef* tiles, int64_t tile0, int64_t ntiles,
                     const PtrArgs& pa, int alias)
    {
        for (int64_t off = 0; off < ntiles; off += MAX_GROUPS_PER_LAUNCH) {
            const int64_t n = ntiles - off < MAX_GROUPS_PER_LAUNCH ? ntiles - off : MAX_GROUPS_PER_LAUNCH;
            hipLaunchKernelGGL(k_copy_tiles, dim3((unsigned)n), dim3(COPY_THREADS), 0, stream_, descs,
                               tiles, (uint32_t)(tile0 + off), pa, alias, xcd_chunk());
            VPS_HIP_CHECK(hipGetLastError());
        }
    }

    void launch_plain_copy(void* dst, const void* src, uint64_t bytes)
    {
        const uint64_t nvec = bytes / 16;
        const uint64_t per_launch = (uint64_t)MAX_GROUPS_PER_LAUNCH * PLAIN_TILE_VECS;
        for (uint64_t v0 = 0; v0 < nvec; v0 += per_launch) {
            const uint64_t n = nvec - v0 < per_launch ? nvec - v0 : per_launch;
            const uint64_t blocks = (n + PLAIN_TILE_VECS - 1) / PLAIN_TILE_VECS;
            hipLaunchKernelGGL(k_plain_copy, dim3((unsigned)blocks), dim3(COPY_THREADS), 0, stream_,
                               (const char*)src + v0 * 16, (char*)dst + v0 * 16, n, xcd_chunk());
            VPS_HIP_CHECK(hipGetLastError());
        }
    }

    // mode 0: read `bytes` from src (sink: 4 bytes of device memory), mode 1: fill dst
    void launch_plain_half(int mode, void* dst, const void* src, uint64_t bytes, void* sink)
    {
        const uint64_t nvec = bytes / 16;
        const uint64_t per_launch = (uint64_t)MAX_GROUPS_PER_LAUNCH * PLAIN_TILE_VECS;
        for (uint64_t v0 = 0; v0 < nvec; v0 += per_launch) {
            const uint64_t n = nvec - v0 < per_launch ? nvec - v0 : per_launch;
            const uint64_t blocks = (n + PLAIN_TILE_VECS - 1) / PLAIN_TILE_VECS;
            if (mode == 0)
                hipLaunchKernelGGL(k_plain_read, dim3((unsigned)blocks), dim3(COPY_THREADS), 0, stream_,
                                   (const char*)src + v0 * 16, n, xcd_chunk(), (uint32_t*)sink);
            else
                hipLaunchKernelGGL(k_plain_fill, dim3((unsigned)blocks), dim3(COPY_THREADS), 0, stream_,
                                   (char*)dst + v0 * 16, n, xcd_chunk());
            VPS_HIP_CHECK(hipGetLastError());
        }
    }

    hipStream_t stream() const { return stream_; }

    // Tiles per XCD run (0 = plain round-robin).
    static std::atomic<uint32_t>& xcd_chunk_setting()
    {
        static std::atomic<uint32_t> v{ 64u };
        return v;
    }
    static uint32_t xcd_chunk() { return xcd_chunk_setting().load(); }
    static void set_xcd_chunk(uint32_t v) { xcd_chunk_setting() = v; }

    // Wait until the work queued on stream `s` has finished (errors, e.g. a stream that no longer
    // exists, are ignored: nothing can be running on it then).
    void wait_stream(void* s) { (void)hipStreamSynchronize((hipStream_t)s); }

private:
    void recycle_dead()
    {
        if (dead_.empty()) return;
        (void)hipStreamSynchronize(stream_);
        for (void* p : dead_) DevicePool::get().give(p);
        dead_.clear();
    }

    struct Stage {
        void* host;
        void* pinned;
        size_t bytes;
    };

    hipStream_t stream_;
    struct ZeroedBlock {
        void* p = nullptr;
        size_t bytes = 0;
    };
    static std::mutex& zeroed_mutex() { static std::mutex m; return m; }
    static ZeroedBlock& zeroed_slot() { static ZeroedBlock z; return z; }

    std::vector<void*> live_;
    std::vector<void*> dead_;
    std::vector<Stage> stages_;
    ZeroedBlock pending_zeroed_;
};

}  // namespace vps

// vps_copy_kernel.h - the descriptor-driven strided-box copy engine (PackData / UnpackData
// of DynaTrain Algorithm 1, plus the direct old-local -> new-local copy of retained slices).
//
// One workgroup per tile.  A tile is a slice of one box of roughly tile_bytes payload:
//   RUN   both sides are contiguous along the innermost collapsed axis.  Lanes own 16-byte
//         destination-aligned vectors: aligned 16-byte stores, 16-byte loads at whatever
//         element alignment the source has; the (at most two) partial vectors at the ends of
//         a run are moved in 2-byte units.  Long runs are cut into chunks, short runs are
//         batched several rows per tile.
//   ELEM  fallback when the two sides have no common contiguous axis: one element per lane.
// HBM-bound: every payload byte is read once and written once; descriptors and the tile
// table add well under 1 % of traffic.
#pragma once

#include <hip/hip_runtime.h>

#include "vps_core.h"

namespace vps {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_any __attribute__((aligned(2)));  // source vectors: element alignment only

__device__ __forceinline__ char* slot_ptr(const PtrArgs& pa, int32_t slot)
{
    return pa.tbl ? pa.tbl[slot] : pa.inl[slot];
}

constexpr int COPY_THREADS = 256;
constexpr int COPY_UNROLL = 4;

__device__ __forceinline__ void copy_partial(const char* s, char* t, uint32_t nb)
{
    for (uint32_t b = 0; b < nb; b += 2)
        *reinterpret_cast<uint16_t*>(t + b) = *reinterpret_cast<const uint16_t*>(s + b);
}

__global__ __launch_bounds__(COPY_THREADS) void k_copy_tiles(const CopyDesc* __restrict__ descs,
                                                             const TileRef* __restrict__ tiles,
                                                             uint32_t tile0, PtrArgs pa,
                                                             int alias_exchange)
{
    const TileRef tr = tiles[tile0 + blockIdx.x];
    const CopyDesc d = descs[tr.desc];
    const bool alias = alias_exchange && d.alt_src_slot >= 0;
    const char* sbase = (alias ? slot_ptr(pa, d.alt_src_slot) + d.alt_src_byte
                               : slot_ptr(pa, d.src_slot) + d.src_byte);
    char* dbase = slot_ptr(pa, d.dst_slot) + d.dst_byte;
    const uint32_t tid = threadIdx.x;

    if (d.mode == MODE_RUN) {
        uint32_t row0, nrows, w0, nw;
        run_tile_geometry(d, tr.q, row0, nrows, w0, nw);
        const uint64_t run_bytes = (uint64_t)d.ext[3] * d.es;
        const uint32_t total = nrows * nw;
        const char* srow0 = nullptr;
        char* drow0 = nullptr;
        if (nrows == 1) run_row_address(d, row0, sbase, dbase, srow0, drow0);
        for (uint32_t base = 0; base < total; base += COPY_THREADS * COPY_UNROLL) {
            u32x4 v[COPY_UNROLL];
            char* tp[COPY_UNROLL];
            bool full[COPY_UNROLL];
#pragma unroll
            for (int u = 0; u < COPY_UNROLL; ++u) {
                const uint32_t slot = base + u * COPY_THREADS + tid;
                full[u] = false;
                if (slot < total) {
                    const char* srow = srow0;
                    char* drow = drow0;
                    uint32_t w = w0 + slot;
                    if (nrows != 1) {
                        const uint32_t r = slot / nw;
                        w = slot - r * nw;
                        run_row_address(d, row0 + r, sbase, dbase, srow, drow);
                    }
                    const char* s;
                    char* t;
                    const uint32_t nb = run_vector_span(srow, drow, run_bytes, w, s, t);
                    if (nb == 16) {
                        full[u] = true;
                        tp[u] = t;
                        v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_any*>(s));
                    } else if (nb) {
                        copy_partial(s, t, nb);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < COPY_UNROLL; ++u)
                if (full[u]) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(tp[u]));
        }
    } else {
        const uint64_t vol = (uint64_t)d.ext[0] * d.ext[1] * d.ext[2] * d.ext[3];
        const uint64_t k0 = (uint64_t)tr.q * d.rows_per_tile;
        const uint64_t k1 = k0 + d.rows_per_tile < vol ? k0 + d.rows_per_tile : vol;
        for (uint64_t k = k0 + tid; k < k1; k += COPY_THREADS) {
            int64_t so, to;
            elem_offsets(d, k, so, to);
            if (d.es == 2)
                *reinterpret_cast<uint16_t*>(dbase + to) = *reinterpret_cast<const uint16_t*>(sbase + so);
            else
                *reinterpret_cast<uint32_t*>(dbase + to) = *reinterpret_cast<const uint32_t*>(sbase + so);
        }
    }
}

}  // namespace vps

// vps_backend_hip.h - device backend of the mapper/planner pipeline: one kernel lane per item,
// rocPRIM for the two generic primitives (exclusive scan, stable radix sort).
#pragma once

#include <cstdlib>
#include <cstring>

#include <hip/hip_runtime.h>
#include <rocprim/rocprim.hpp>

#include <algorithm>
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
        if (live_.empty() && dead_.empty() && stages_.empty()) return;
        (void)hipStreamSynchronize(stream_);
        for (const Stage& st : stages_) PinnedPool::get().give(st.pinned);
        stages_.clear();
        for (void* p : live_) DevicePool::get().give(p);
        live_.clear();
        recycle_dead();
    }

    // Wait until nothing on the device can still use blocks that are about to be recycled.
    void quiesce() { (void)hipDeviceSynchronize(); }

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
    // must be 0.
    void exclusive_scan(const int64_t* in, int64_t* out, int64_t n)
    {
        size_t tmp_bytes = 0;
        const size_t count = (size_t)n + 1;
        VPS_HIP_CHECK(rocprim::exclusive_scan(nullptr, tmp_bytes, in, out, (int64_t)0, count,
                                              rocprim::plus<int64_t>(), stream_));
        void* tmp = alloc<char>((int64_t)tmp_bytes);
        VPS_HIP_CHECK(rocprim::exclusive_scan(tmp, tmp_bytes, in, out, (int64_t)0, count,
                                              rocprim::plus<int64_t>(), stream_));
        free(tmp);
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
        size_t tmp_bytes = 0;
        VPS_HIP_CHECK(rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys, k2, vals, v2, (size_t)n, 0, (unsigned)bits, stream_));
        void* tmp = alloc<char>((int64_t)tmp_bytes);
        VPS_HIP_CHECK(rocprim::radix_sort_pairs(tmp, tmp_bytes, keys, k2, vals, v2, (size_t)n, 0, (unsigned)bits, stream_));
        free(tmp); free(keys); free(vals);
        keys = k2; vals = v2;
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

    void zero(void* dev, size_t bytes)
    {
        if (!bytes) return;
        VPS_HIP_CHECK(hipMemsetAsync(dev, 0, bytes, stream_));
    }

    void sync()
    {
        const hipError_t e = hipStreamSynchronize(stream_);
        for (const Stage& st : stages_) {
            if (e == hipSuccess && st.host) memcpy(st.host, st.pinned, st.bytes);
            PinnedPool::get().give(st.pinned);
        }
        stages_.clear();
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

    hipStream_t stream() const { return stream_; }

    // Tiles per XCD run (0 = plain round-robin); VPS_XCD_CHUNK overrides it for experiments.
    static uint32_t xcd_chunk()
    {
        static const uint32_t v = [] {
            const char* e = getenv("VPS_XCD_CHUNK");
            return e ? (uint32_t)atoi(e) : 64u;
        }();
        return v;
    }

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
    std::vector<void*> live_;
    std::vector<void*> dead_;
    std::vector<Stage> stages_;
};

}  // namespace vps

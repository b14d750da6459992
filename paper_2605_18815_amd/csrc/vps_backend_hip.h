// vps_backend_hip.h - device backend of the mapper/planner pipeline: one kernel lane per item,
// rocPRIM for the two generic primitives (exclusive scan, stable radix sort).
#pragma once

#include <cstring>

#include <hip/hip_runtime.h>
#include <rocprim/rocprim.hpp>

#include <algorithm>
#include <string>
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

template <class F>
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

class HipBackend {
public:
    explicit HipBackend(void* s) : stream_((hipStream_t)s) {}
    ~HipBackend() { release_all(); }

    template <class T>
    T* alloc(int64_t n)
    {
        void* p = nullptr;
        const size_t bytes = sizeof(T) * (size_t)(n > 0 ? n : 1);
        VPS_HIP_CHECK(hipMalloc(&p, bytes));
        live_.push_back(p);
        return (T*)p;
    }

    void free(void* p)
    {
        if (!p) return;
        auto it = std::find(live_.begin(), live_.end(), p);
        if (it != live_.end()) live_.erase(it);
        (void)hipFree(p);  // waits for outstanding device work
    }

    // Hand the remaining allocations over to the caller (the handle now owns them).
    void commit() { live_.clear(); }

    void release_all()
    {
        if (live_.empty()) return;
        (void)hipStreamSynchronize(stream_);
        for (void* p : live_) (void)hipFree(p);
        live_.clear();
    }

    template <class F>
    void for_each(int64_t n, F f)
    {
        if (n <= 0) return;
        const int64_t blocks = (n + 255) / 256;
        if (blocks > 0x7fffffffLL) throw Error{ VPS_ERR_OOM, "step has too many items" };
        hipLaunchKernelGGL(k_for_each<F>, dim3((unsigned)blocks), dim3(256), 0, stream_, f, n);
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

    // Stable ascending sort of (key, value) pairs, result back in the input arrays.
    void sort_pairs(uint64_t* keys, uint32_t* vals, int64_t n)
    {
        if (n <= 1) return;
        uint64_t* k2 = alloc<uint64_t>(n);
        uint32_t* v2 = alloc<uint32_t>(n);
        size_t tmp_bytes = 0;
        VPS_HIP_CHECK(rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys, k2, vals, v2, (size_t)n, 0, 64, stream_));
        void* tmp = alloc<char>((int64_t)tmp_bytes);
        VPS_HIP_CHECK(rocprim::radix_sort_pairs(tmp, tmp_bytes, keys, k2, vals, v2, (size_t)n, 0, 64, stream_));
        VPS_HIP_CHECK(hipMemcpyAsync(keys, k2, sizeof(uint64_t) * (size_t)n, hipMemcpyDeviceToDevice, stream_));
        VPS_HIP_CHECK(hipMemcpyAsync(vals, v2, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToDevice, stream_));
        free(tmp); free(k2); free(v2);
    }

    void upload(void* dev, const void* host, size_t bytes)
    {
        if (!bytes) return;
        VPS_HIP_CHECK(hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, stream_));
        VPS_HIP_CHECK(hipStreamSynchronize(stream_));
    }

    void download(void* host, const void* dev, size_t bytes)
    {
        if (!bytes) return;
        VPS_HIP_CHECK(hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, stream_));
        VPS_HIP_CHECK(hipStreamSynchronize(stream_));
    }

    void zero(void* dev, size_t bytes)
    {
        if (!bytes) return;
        VPS_HIP_CHECK(hipMemsetAsync(dev, 0, bytes, stream_));
    }

    void sync() { VPS_HIP_CHECK(hipStreamSynchronize(stream_)); }

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

    void launch_copy(const CopyDesc* descs, const TileRef* tiles, int64_t tile0, int64_t ntiles,
                     const PtrArgs& pa, int alias)
    {
        if (ntiles <= 0) return;
        hipLaunchKernelGGL(k_copy_tiles, dim3((unsigned)ntiles), dim3(COPY_THREADS), 0, stream_, descs,
                           tiles, (uint32_t)tile0, pa, alias);
        VPS_HIP_CHECK(hipGetLastError());
    }

    hipStream_t stream() const { return stream_; }

private:
    hipStream_t stream_;
    std::vector<void*> live_;
};

}  // namespace vps

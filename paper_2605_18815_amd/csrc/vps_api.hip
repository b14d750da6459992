// vps_api.hip - the product translation unit: the C ABI of include/vps.h over the HIP backend.
#include "vps_backend_hip.h"

#define VPS_BACKEND vps::HipBackend
#define VPS_FN(name) vps_##name
#include "vps_api_impl.h"

// ---------------------------------------------------------------------------------------------
// vps_apply_transition_static: the all-ranks transition for callers that cannot allocate device
// memory.  The staging area that vps_apply_transition takes as its `scratch` argument (every
// rank's send buffer; the exchange reads the peers' segments in place) lives in a file-scope
// device array instead.  Every GPU the library runs on holds its own copy of the array until the
// process ends; its address on a GPU is looked up once, with that GPU current.
// ---------------------------------------------------------------------------------------------

namespace {

static __device__ __align__(256) unsigned char scratch[VPS_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_static_scratch_mutex;
void* g_static_scratch_ptr[MAX_DEVICES];   // per device: address of that device's copy of `scratch`

// The device address of `scratch` on the current device (never the array's name: in host code
// that is a host-side stand-in, not a device address).
int static_scratch_address(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return vps::fail(VPS_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return vps::fail(VPS_ERR_HIP, "device index beyond the static scratch table");
    std::lock_guard<std::mutex> g(g_static_scratch_mutex);
    if (!g_static_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return vps::fail(VPS_ERR_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        g_static_scratch_ptr[dev] = p;
    }
    *out = g_static_scratch_ptr[dev];
    return VPS_OK;
}

}  // namespace

extern "C" {

uint64_t vps_static_scratch_bytes(void) { return VPS_STATIC_SCRATCH_BYTES; }

int vps_apply_transition_static(const vps_plan* plan, const void* const* src_bufs, void* const* dst_bufs,
                                void* stream)
{
    if (!plan || !src_bufs || !dst_bufs) return vps::fail(VPS_ERR_INVALID_ARG, "null argument");
    if (plan->d.rank >= 0)
        return vps::fail(VPS_ERR_INVALID_ARG,
                         "the static-scratch call takes an all-ranks plan (a single-rank plan's receive buffer is "
                         "filled by the caller, so it cannot be library memory)");
    uint64_t need = 0;
    if (int rc = vps_plan_buffer_bytes(plan, -1, nullptr, nullptr, nullptr, &need, nullptr)) return rc;
    if (need > VPS_STATIC_SCRATCH_BYTES)
        return vps::fail(VPS_ERR_SCRATCH_TOO_SMALL,
                         "the plan exchanges " + std::to_string(need) + " bytes, the static scratch holds " +
                             std::to_string((uint64_t)VPS_STATIC_SCRATCH_BYTES) + "; use vps_apply_transition with a caller-owned scratch");
    void* ptr = nullptr;
    if (int rc = static_scratch_address(&ptr)) return rc;
    // Nothing in the staging area has to start at zero: pack writes every payload byte that unpack
    // reads, and the pad bytes between boxes are never read.
    return vps_apply_transition(plan, -1, src_bufs, dst_bufs, ptr, VPS_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"

// vps_api.hip - the product translation unit: the C ABI of include/vps.h over the HIP backend.
#include "vps_backend_hip.h"

#define VPS_BACKEND vps::HipBackend
#define VPS_FN(name) vps_##name
#include "vps_api_impl.h"

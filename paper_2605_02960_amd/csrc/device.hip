// Per-device state of libmoeprefill: the compute-unit count and the one-time kernel attribute
// set-up, done once per device under a mutex (two host threads may make their first calls at the
// same time).  moe_init_device does it explicitly, for callers whose first compute call would
// otherwise fall inside a stream capture.
#include <mutex>

#include "common.h"

namespace moe {

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_mutex;
DeviceState g_state[MAX_DEVICES];
bool g_ready[MAX_DEVICES] = {};
}  // namespace

int32_t device_state(const DeviceState** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return MOE_ERR_LAUNCH_FAILED;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_ready[dev]) {
        int n_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
            return MOE_ERR_LAUNCH_FAILED;
        if (ffn_mfma_set_attributes() != MOE_OK || router_mfma_set_attributes() != MOE_OK)
            return MOE_ERR_LAUNCH_FAILED;
        g_state[dev].n_cu = n_cu;
        g_ready[dev] = true;
    }
    *out = &g_state[dev];
    return MOE_OK;
}

}  // namespace moe

extern "C" int32_t moe_init_device(void) {
    const moe::DeviceState* d = nullptr;
    return moe::device_state(&d);
}

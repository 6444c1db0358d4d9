// Per-device state of libmoeprefill: the compute-unit count and the one-time kernel attribute
// set-up, done once per device under a mutex (two host threads may make their first calls at the
// same time).  moe_init_device does it explicitly, for callers whose first compute call would
// otherwise fall inside a stream capture.
//
// Also here: the library's one allocation-free entry point, moe_permute_noalloc, for callers that
// can neither allocate a workspace nor pass one in (code under graph capture, tight serving
// loops).  Its scratch memory is a fixed array in device memory that every GPU the library runs
// on holds until the process ends; the array's device address is looked up once per device at
// set-up and only that address is ever handed to kernels (in host code the array's name is a
// host-side stand-in, not a device address).
#include <mutex>

#include "common.h"

// Segment histograms of moe_permute: ceil(T*K / 2048) * E counters.  1 MiB covers 524 288 routed
// rows at E = 1024 and 4 194 304 at E = 128.
static __device__ __align__(256) unsigned char scratch[MOE_NOALLOC_SCRATCH_BYTES];

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
        // each GPU holds its own copy of the scratch array at its own address
        void* scratch_ptr = nullptr;
        if (hipGetSymbolAddress(&scratch_ptr, HIP_SYMBOL(scratch)) != hipSuccess || !scratch_ptr)
            return MOE_ERR_LAUNCH_FAILED;
        g_state[dev].n_cu = n_cu;
        g_state[dev].scratch = scratch_ptr;
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

extern "C" int32_t moe_permute_noalloc(const moe_config_t* cfg, const int32_t* topk_idx, const void* x,
                                       int32_t* counts, int32_t* offsets, int32_t* perm,
                                       int32_t* inv_perm, void* x_perm, void* stream) {
    size_t need = 0;
    int32_t st = moe_workspace_bytes(cfg, MOE_CALL_PERMUTE, &need);     // validates cfg
    if (st != MOE_OK) return st;
    if (need > MOE_NOALLOC_SCRATCH_BYTES) return MOE_ERR_TOO_LARGE;
    const moe::DeviceState* d = nullptr;
    st = moe::device_state(&d);
    if (st != MOE_OK) return st;
    // Every counter the kernels read is written by the histogram kernel of the same call first, so
    // nothing has to be cleared; what the previous call left behind is never read.
    return moe_permute(cfg, topk_idx, x, counts, offsets, perm, inv_perm, x_perm, d->scratch,
                       MOE_NOALLOC_SCRATCH_BYTES, stream);
}

// sparsek_mask_static: the thresholds and lifetimes of sparsek_mask for callers that cannot bring a workspace
// (code under HIP graph capture, serving loops and harnesses that forbid allocation).  The kernels are those of
// sparsek_mask; their scratch -- the per-super-block lower bounds and the status word -- lives in a file-scope device
// array that every GPU holds once, until the process ends.  Nothing here allocates or frees.
#include <mutex>

#include "common.hpp"

namespace {

// rows * ceil(n / 2048) lower bounds (fp32) + 256 bytes for the status word must fit
constexpr size_t SCRATCH_BYTES = SPARSEK_MASK_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES];  // device address of `scratch` on each GPU, looked up once per device
std::mutex scratch_mutex;

// In host code `scratch` only names the symbol; its memory is reached through the address the runtime reports for
// the current device.
int scratch_address(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return SPARSEK_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SPARSEK_ERR_LAUNCH;
        }
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return SPARSEK_OK;
}

}  // namespace

extern "C" {

int sparsek_mask_static(const sparsek_cfg* cfg, const float* u, float* tau, int32_t* death, void* stream)
{
    // same argument rules as sparsek_mask
    if (sparsek_mask_workspace_bytes(cfg) == 0) {
        // the size query returns 0 exactly when the configuration is refused; ask sparsek_mask for the code
        return sparsek_mask(cfg, u, tau, death, nullptr, 0, stream);
    }
    if (!u || !tau || !death) return SPARSEK_ERR_INVALID_ARG;
    if (spk::mask_ws_bytes(*cfg) > SCRATCH_BYTES) return SPARSEK_ERR_TOO_LARGE;
    void* ws = nullptr;
    int rc = scratch_address(&ws);
    if (rc) return rc;
    // every word of the scratch that a call reads is written earlier in the same call (the lower bounds and the
    // cleared status word by the first kernel), so nothing needs clearing here
    return spk::launch_mask(*cfg, u, tau, death, ws, (hipStream_t)stream);
}

}  // extern "C"

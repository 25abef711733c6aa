// SPARSEK mask backward (gradient of sum(dO*O) w.r.t. the scores): placeholder until the
// fused kernel lands -- reports "unsupported" instead of computing anything.
#include "common.hpp"
namespace spk {
size_t mask_bwd_ws_bytes(const sparsek_cfg&) { return 256; }
int launch_mask_bwd(const sparsek_cfg&, const void*, const void*, const void*, const float*, const float*,
                    const int32_t*, const void*, const float*, const void*, float*, void*, hipStream_t)
{
    return SPARSEK_ERR_UNSUPPORTED;
}
}  // namespace spk

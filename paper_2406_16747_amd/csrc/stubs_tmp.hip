#include "common.hpp"
namespace spk {
size_t mask_bwd_ws_bytes(const sparsek_cfg&) { return 256; }
int launch_mask_bwd(const sparsek_cfg&, const void*, const void*, const void*, const float*, const float*, const int32_t*, const void*, const float*, const void*, float*, void*, hipStream_t) { return SPARSEK_ERR_UNSUPPORTED; }
size_t decode_state_bytes(const sparsek_decode_cfg&) { return 256; }
int launch_decode_init(const sparsek_decode_cfg&, void*, hipStream_t) { return SPARSEK_ERR_UNSUPPORTED; }
int launch_decode_load(const sparsek_decode_cfg&, void*, int, const void*, const void*, const float*, const float*, const int32_t*, hipStream_t) { return SPARSEK_ERR_UNSUPPORTED; }
int launch_decode_step(const sparsek_decode_cfg&, void*, const void*, const void*, const void*, const float*, void*, hipStream_t) { return SPARSEK_ERR_UNSUPPORTED; }
int decode_status(const sparsek_decode_cfg&, const void*, int32_t*, hipStream_t) { return SPARSEK_ERR_UNSUPPORTED; }
}

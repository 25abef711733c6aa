// Internal helpers shared by the HIP translation units of libsparsek (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparsek.h"

#define SPK_WAVE 64

namespace spk {

// Launch wrappers implemented in the .hip files; all return a SPARSEK_* code.
int launch_mask(const sparsek_cfg& c, const float* u, float* tau, int32_t* death, void* ws,
                hipStream_t st);
size_t mask_ws_bytes(const sparsek_cfg& c);
int launch_materialize(const sparsek_cfg& c, const float* u, const float* tau, const int32_t* death,
                       int t_begin, int t_end, int32_t* idx, float* gate, hipStream_t st);
int launch_attn_fwd(const sparsek_cfg& c, const void* q, const void* k, const void* v,
                    const float* u, const float* tau, const int32_t* death, void* o, float* lse,
                    void* ws, hipStream_t st);
size_t attn_fwd_ws_bytes(const sparsek_cfg& c);
int launch_mask_bwd(const sparsek_cfg& c, const void* q, const void* k, const void* v,
                    const float* u, const float* tau, const int32_t* death, const void* o,
                    const float* lse, const void* dO, float* du, void* ws, hipStream_t st);
size_t mask_bwd_ws_bytes(const sparsek_cfg& c);

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? SPARSEK_OK : SPARSEK_ERR_LAUNCH;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#ifdef __HIPCC__
// ---- wave-level reductions (all 64 lanes must be active) ----
__device__ __forceinline__ double wave_sum_f64(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_sum_f32(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ int wave_sum_i32(int x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_min_f32(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fminf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_max_f32(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned long long y = __shfl_xor(x, o, 64);
        x = y < x ? y : x;
    }
    return x;
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned long long y = __shfl_xor(x, o, 64);
        x = y > x ? y : x;
    }
    return x;
}

// Order-preserving map fp32 -> uint32 (-0.0 is folded onto +0.0 first).
__device__ __forceinline__ uint32_t score_key(float v)
{
    uint32_t b = __float_as_uint(v + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
// Selection order as one unsigned compare: larger score first, then the older position.
__device__ __forceinline__ unsigned long long sel_key(float v, int idx)
{
    return ((unsigned long long)score_key(v) << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)idx);
}
__device__ __forceinline__ float clip01(float x) { return __builtin_amdgcn_fmed3f(x, 0.0f, 1.0f); }

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40u);  // quiet NaN
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}
#endif

}  // namespace spk

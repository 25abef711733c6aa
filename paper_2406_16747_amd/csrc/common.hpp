// Internal helpers shared by the HIP translation units of libsparsek (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparsek.h"

#define SPK_WAVE 64

namespace spk {

// Launch wrappers implemented in the .hip files; all return a SPARSEK_* code.
// t_begin > 0: thresholds of prefixes before t_begin are not needed and deaths that fall before it are left at
// their preset (chunked prefill); the 128-prefix blocks that end at or before t_begin are skipped.
int launch_mask(const sparsek_cfg& c, const float* u, float* tau, int32_t* death, void* ws,
                hipStream_t st, int t_begin = 0);
size_t mask_ws_bytes(const sparsek_cfg& c);
// copies the status word that the last launch_mask on `ws` left (bit 0: a threshold solve hit its iteration cap) and waits
int mask_status(const sparsek_cfg& c, const void* ws, int32_t* host_flag, hipStream_t st);
int launch_materialize(const sparsek_cfg& c, const float* u, const float* tau, const int32_t* death,
                       int t_begin, int t_end, int32_t* idx, float* gate, hipStream_t st);
int launch_attn_fwd(const sparsek_cfg& c, const void* q, const void* k, const void* v,
                    const float* u, const float* tau, const int32_t* death, void* o, float* lse,
                    void* ws, hipStream_t st, int q_begin = 0, const int32_t* first_valid = nullptr,
                    int q_rows = 0);
// (query blocks that end at or before q_begin are skipped; keys before first_valid[row] are never attended;
//  q_rows != 0: q, o and lse hold q_rows rows per head, the first being query q_begin, a multiple of 128)
size_t attn_fwd_ws_bytes(const sparsek_cfg& c);
int launch_mask_bwd(const sparsek_cfg& c, const void* q, const void* k, const void* v,
                    const float* u, const float* tau, const int32_t* death, const void* o,
                    const float* lse, const void* dO, float* du, void* ws, hipStream_t st, int q_begin = 0,
                    int q_rows = 0, int t_min = 0);
// (q_begin, q_rows as in launch_attn_fwd, for q, o, dO and lse; thresholds of prefixes before t_min are not read;
//  bf16 with d = 64 or 128 only when any of them is set)
size_t mask_bwd_ws_bytes(const sparsek_cfg& c);
int launch_attn_bwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, const void* o, const float* lse, const void* dO,
                    void* dq, void* dk, void* dv, void* ws, hipStream_t st, int q_begin = 0,
                    const int32_t* first_valid = nullptr, int q_rows = 0);
// (q_rows != 0: q, o, dO, lse, dq and also dk, dv hold q_rows rows per head, the first being position q_begin: only
//  keys from q_begin on receive a gradient; keys before first_valid[row] are attended by nobody; bf16, d = 64 / 128)
size_t attn_bwd_ws_bytes(const sparsek_cfg& c);

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? SPARSEK_OK : SPARSEK_ERR_LAUNCH;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#ifdef __HIPCC__
// ---- wave-level reductions (all 64 lanes must be active; every lane gets the result) ----
// Four DPP steps reduce inside each row of 16 lanes (quad swaps, half-row mirror, row mirror),
// then the four row totals are read with v_readlane and combined.  No LDS round trips.
#define SPK_DPP(x, ctrl) __builtin_amdgcn_update_dpp(0, (x), (ctrl), 0xF, 0xF, true)
#define SPK_QP_SWAP1 0xB1   // quad_perm [1,0,3,2]
#define SPK_QP_SWAP2 0x4E   // quad_perm [2,3,0,1]
#define SPK_HALF_MIRROR 0x141
#define SPK_ROW_MIRROR 0x140

__device__ __forceinline__ float dpp_f32(float x, int which)
{
    const int i = __float_as_int(x);
    int r;
    switch (which) {
        case 0: r = SPK_DPP(i, SPK_QP_SWAP1); break;
        case 1: r = SPK_DPP(i, SPK_QP_SWAP2); break;
        case 2: r = SPK_DPP(i, SPK_HALF_MIRROR); break;
        default: r = SPK_DPP(i, SPK_ROW_MIRROR); break;
    }
    return __int_as_float(r);
}
__device__ __forceinline__ int dpp_i32(int i, int which)
{
    switch (which) {
        case 0: return SPK_DPP(i, SPK_QP_SWAP1);
        case 1: return SPK_DPP(i, SPK_QP_SWAP2);
        case 2: return SPK_DPP(i, SPK_HALF_MIRROR);
        default: return SPK_DPP(i, SPK_ROW_MIRROR);
    }
}
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long x, int which)
{
    const int lo = dpp_i32((int)(unsigned)(x & 0xFFFFFFFFull), which);
    const int hi = dpp_i32((int)(unsigned)(x >> 32), which);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned long long)(unsigned)lo;
}
__device__ __forceinline__ double dpp_f64(double x, int which)
{
    return __longlong_as_double((long long)dpp_u64((unsigned long long)__double_as_longlong(x), which));
}
__device__ __forceinline__ float readlane_f32(float x, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}
__device__ __forceinline__ unsigned long long readlane_u64(unsigned long long x, int l)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(x & 0xFFFFFFFFull), l);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(x >> 32), l);
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ double wave_sum_f64(double x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) x += dpp_f64(x, s);
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    return __longlong_as_double((long long)readlane_u64(b, 15)) + __longlong_as_double((long long)readlane_u64(b, 31)) +
           __longlong_as_double((long long)readlane_u64(b, 47)) + __longlong_as_double((long long)readlane_u64(b, 63));
}
__device__ __forceinline__ float wave_sum_f32(float x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) x += dpp_f32(x, s);
    return (readlane_f32(x, 15) + readlane_f32(x, 31)) + (readlane_f32(x, 47) + readlane_f32(x, 63));
}
__device__ __forceinline__ int wave_sum_i32(int x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) x += dpp_i32(x, s);
    return __builtin_amdgcn_readlane(x, 15) + __builtin_amdgcn_readlane(x, 31) + __builtin_amdgcn_readlane(x, 47) +
           __builtin_amdgcn_readlane(x, 63);
}
// two 32-bit counts packed into one 64-bit word (each < 2^31): summed as two ints
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long x)
{
    const int lo = wave_sum_i32((int)(unsigned)(x & 0xFFFFFFFFull));
    const int hi = wave_sum_i32((int)(unsigned)(x >> 32));
    return ((unsigned long long)(unsigned)hi << 32) + (unsigned long long)(unsigned)lo;
}
__device__ __forceinline__ float wave_min_f32(float x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) x = fminf(x, dpp_f32(x, s));
    return fminf(fminf(readlane_f32(x, 15), readlane_f32(x, 31)), fminf(readlane_f32(x, 47), readlane_f32(x, 63)));
}
__device__ __forceinline__ float wave_max_f32(float x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) x = fmaxf(x, dpp_f32(x, s));
    return fmaxf(fmaxf(readlane_f32(x, 15), readlane_f32(x, 31)), fmaxf(readlane_f32(x, 47), readlane_f32(x, 63)));
}
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const unsigned long long y = dpp_u64(x, s);
        x = y < x ? y : x;
    }
    unsigned long long a = readlane_u64(x, 15), b = readlane_u64(x, 31), c = readlane_u64(x, 47), d = readlane_u64(x, 63);
    a = b < a ? b : a;
    c = d < c ? d : c;
    return c < a ? c : a;
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x)
{
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const unsigned long long y = dpp_u64(x, s);
        x = y > x ? y : x;
    }
    unsigned long long a = readlane_u64(x, 15), b = readlane_u64(x, 31), c = readlane_u64(x, 47), d = readlane_u64(x, 63);
    a = b > a ? b : a;
    c = d > c ? d : c;
    return c > a ? c : a;
}

// Order-preserving map fp32 -> uint32 (-0.0 is folded onto +0.0 first).
__device__ __forceinline__ uint32_t score_key(float v)
{
    uint32_t b = __float_as_uint(v + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
// Inverse of score_key: the fp32 bit pattern of a key.
__device__ __forceinline__ uint32_t score_key_inv(uint32_t key)
{
    return (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
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

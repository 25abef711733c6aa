// Shared by the attention forward and the mask-backward MFMA kernels: vector types, tile
// geometry, the LDS staging area and the direct-to-LDS gather of one K/V tile.
#pragma once
#include "common.hpp"
#include <type_traits>

namespace spk {

constexpr int QB = 128;  // queries per workgroup block (also the granularity of the per-block top-k lists)

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

// The 4-byte form of async_load_lds16 below: lane l's word at gbase + voff lands at lds_dst + 4 * l.
__device__ __forceinline__ void async_load_lds4(const void* gbase, uint32_t voff, const void* lds_dst)
{
    const uint32_t m0v = (uint32_t)(uintptr_t)(lds_void_t*)lds_dst;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(m0v), "v"(voff), "s"(gbase)
                 : "memory", "m0");
}

// A 16-byte-per-lane direct-to-LDS load that the compiler does not track: lane l's 16 bytes at gbase + voff land
// at lds_dst + 16 * l (gbase and lds_dst uniform over the wave).  The compiler makes the first LDS read that
// follows a tracked direct-to-LDS load wait for all such loads (it cannot tell that the read goes to another
// buffer), which would put the whole memory latency of a prefetch in front of the next operand read.  The
// caller waits itself: s_waitcnt vmcnt(0) before the barrier that publishes the tile.
// The LDS base goes through M0, which the compiler reserves for itself and does not treat as clobbered by an asm
// statement: a kernel that uses these loads must give the compiler no reason to keep a value of its own in M0 across
// them (the builtin form of the same load, indirect register indexing).  The kernels here use one form or the other.
__device__ __forceinline__ void async_load_lds16(const void* gbase, uint32_t voff, const void* lds_dst)
{
    const uint32_t m0v = (uint32_t)(uintptr_t)(lds_void_t*)lds_dst;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(m0v), "v"(voff), "s"(gbase)
                 : "memory", "m0");
}

constexpr int KT = 64;     // keys per tile
constexpr int SEG = 1088;  // keys whose metadata is staged in LDS at a time (17 tiles)

// The double-buffered K and V tiles of a workgroup.
template <int D, int VPAD = 64>
struct MfmaTileBufs {
    static constexpr int RB = D * 2;        // bytes per K/V row
    static constexpr int RPL = 1024 / RB;   // rows per wave-load
    static constexpr int NL = KT / RPL;     // wave-loads (row groups) per tile and tensor
    static constexpr int GSK = 1024 + 16;   // group stride of the K buffer
    static constexpr int GSV = 1024 + VPAD; // group stride of the V buffer (64: transposing reads, 16: row reads)
    unsigned char kb[2][NL * GSK];
    unsigned char vb[2][NL * GSV];
};

// Tiles plus the metadata of one segment of keys, staged by the workgroup before the segment's tile loop.
template <int D, int VPAD = 64>
struct MfmaSmem : MfmaTileBufs<D, VPAD> {
    int32_t jpos[SEG];        // key position
    int32_t jlast[SEG];       // last query that attends the key: w - 1 + death[j]; -1 = padding
    float ju[SEG];            // key score
};

// The gather of one tile (64 rows of K and of V) into buffer `buf`, as NL/4 steps per wave:
// tile_rows() reads this lane's row numbers with one LDS load, tile_load_step(x) enqueues one
// K and one V wave-load.  Row offsets are 32-bit byte offsets from the head's base pointer
// (the host checks n * RB < 2^32), so every load is a uniform base plus one v_lshl_add_u32.
template <int D, int VPAD>
struct TileRows {
    int32_t j[MfmaTileBufs<D, VPAD>::NL / 4];
};

template <int D, int VPAD>
__device__ __forceinline__ TileRows<D, VPAD> tile_rows(const int32_t* jp, int wv, int lane)
{
    using S = MfmaTileBufs<D, VPAD>;
    constexpr int LPR = S::RB / 16;  // lanes per row
    constexpr int NX = S::NL / 4;
    const int jrow = lane / LPR;
    TileRows<D, VPAD> r;
    const int32_t* src = jp + wv * NX + S::NL * jrow;  // row L + NL * jrow for L = wv * NX + x
    if constexpr (NX == 4) {
        const int4 t = *(const int4*)src;
        r.j[0] = t.x; r.j[1] = t.y; r.j[2] = t.z; r.j[3] = t.w;
    } else {
        static_assert(NX == 2, "head dim 64 or 128");
        const int2 t = *(const int2*)src;
        r.j[0] = t.x; r.j[1] = t.y;
    }
    return r;
}

template <int D, int VPAD>
__device__ __forceinline__ void tile_load_step(MfmaTileBufs<D, VPAD>& sm, int buf, const TileRows<D, VPAD>& rows, int x,
                                               const uint16_t* __restrict__ kh, const uint16_t* __restrict__ vh,
                                               int wv, int lane)
{
    using S = MfmaTileBufs<D, VPAD>;
    constexpr int LPR = S::RB / 16;
    const int c = lane % LPR;
    const int L = wv * (S::NL / 4) + x;
    const uint32_t off = (uint32_t)rows.j[x] * (uint32_t)S::RB + 16u * (uint32_t)c;
    async_load_lds16(kh, off, &sm.kb[buf][L * S::GSK]);
    async_load_lds16(vh, off, &sm.vb[buf][L * S::GSV]);
}

template <int D, int VPAD>
__device__ __forceinline__ void issue_tile_loads(MfmaTileBufs<D, VPAD>& sm, int buf, const int32_t* jp,
                                                 const uint16_t* __restrict__ kh, const uint16_t* __restrict__ vh,
                                                 int wv, int lane)
{
    const TileRows<D, VPAD> rows = tile_rows<D, VPAD>(jp, wv, lane);
#pragma unroll
    for (int x = 0; x < MfmaTileBufs<D, VPAD>::NL / 4; x++) tile_load_step<D, VPAD>(sm, buf, rows, x, kh, vh, wv, lane);
}

// Compile-time loop: f(integral_constant<int, I>) for I = 0 .. N-1.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

}  // namespace spk

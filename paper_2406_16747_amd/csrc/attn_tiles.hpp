// Shared by the MFMA kernels of the attention forward, the attention backward and the mask backward: vector
// types, tile geometry, LDS staging areas, the direct-to-LDS gather of one K/V tile, the per-block key lists and
// the classification of a query block's tiles into kinds.
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

inline int nblocks(int n) { return (n + QB - 1) / QB; }

// The MFMA forward kernel reads a second form of the lists: per (row, block) three parallel arrays of KP entries --
// position, lifetime death[j] and score u[j] of every listed key -- so that it stages a segment of metadata with
// plain copies (no gather by position).  Entries from the list length up to the next multiple of the tile size are
// padding (position 0, lifetime INT_MIN: attended by nobody, score 0).
inline size_t ext_stride(const sparsek_cfg& c) { return align_up((size_t)(c.k > 0 ? c.k : 1), KT); }
inline size_t ext_array_bytes(const sparsek_cfg& c)
{
    return align_up((size_t)c.B * c.Gu * nblocks(c.n) * ext_stride(c) * sizeof(int32_t), 256);
}

struct ExtLists {
    int32_t* pos;
    int32_t* death;
    float* u;
    int KP;
};

// Builds the per-block lists (and, with x.pos != nullptr, their extended form) of every score row.
void launch_block_lists_ext(const sparsek_cfg& c, const int32_t* death, int32_t* lists, int32_t* counts,
                            const float* u, const ExtLists& x, hipStream_t st);

// Metadata (position, lifetime, score of every key of the block's key set) is staged in segments of TPS tiles, double
// buffered: while the tiles of one segment run, the next segment is copied into the other buffer.
constexpr int TPS = 9;
constexpr int SEGN = TPS * KT;

struct TileMeta {
    int32_t jpos[2][SEGN];    // key position
    int32_t jdeath[2][SEGN];  // death[j]: the key is attended by query i while i <= w - 1 + death[j]; INT_MIN = padding
    float ju[2][SEGN];        // key score
};

// Tile kinds.  Along a block's key set they come in runs (per wave), so the tile loop is a
// sequence of loops, one per kind, and each loop body is straight-line code:
//   LIST       selected keys that stay selected for every query of the block: gates, no mask
//   LIST_MASK  selected keys some of which expire inside the block (the tail of the list), and
//              contiguous keys that are behind every window of the wave: gates, lifetime test
//   EDGE       contiguous keys at the trailing edge of the wave's windows: gate 1 inside the
//              window, lifetime test (always true inside the window)
//   FAST       contiguous keys inside every query's window and not in its future: nothing
//   DIAG       contiguous keys inside every window, at the causal diagonal: causal test
//   CONT       everything at once (narrow windows, where EDGE and DIAG overlap)
//   SKIP       keys in the future of the whole wave: loads and barriers only
enum { TILE_FAST = 0, TILE_LIST = 1, TILE_LIST_MASK = 2, TILE_CONT = 3, TILE_EDGE = 4, TILE_DIAG = 5, TILE_SKIP = 6 };

template <int MODE, int KIND>
struct TileTraits {
    static constexpr bool SEL = KIND == TILE_LIST || KIND == TILE_LIST_MASK || KIND == TILE_CONT || KIND == TILE_EDGE;
    static constexpr bool GATED = SEL && MODE != 2;   // the value gate applies
    static constexpr bool KGATE = SEL && MODE == 0;   // the key gate applies
    static constexpr bool SELECT = KIND == TILE_CONT || KIND == TILE_EDGE;  // window keys mixed in: gate 1
    static constexpr bool MASKL = KIND == TILE_LIST_MASK || KIND == TILE_CONT || KIND == TILE_EDGE;
    static constexpr bool MASKC = KIND == TILE_CONT || KIND == TILE_DIAG;
};

// What a wave needs to stage a segment of metadata (see TileMeta).
struct StageSrc {
    const int32_t* xpos;    // extended list of this (row, block): positions, lifetimes, scores
    const int32_t* xdeath;
    const float* xu;
    const int32_t* dr;      // lifetimes and scores of the score row, for the contiguous keys
    const float* ur;
    int nkl, c0, c_end, nt; // list part in keys (whole tiles), first and last contiguous key, tiles in all
};

// Segment sg of the block's key set (tiles sg*TPS .. ) goes to metadata buffer sg & 1.  Each wave copies the tiles
// wv, wv + 4, ...: plain copies that land in LDS without passing through registers and that the compiler does not
// track (the per-tile s_waitcnt vmcnt(0) + barrier publishes them).  A tile lies entirely in the list part or
// entirely in the contiguous part.
__device__ __forceinline__ void stage_meta(TileMeta& sm, const StageSrc& src, int sg, int wv, int lane)
{
    const int mb = sg & 1;
    const int t_end = min(TPS, src.nt - sg * TPS);
    for (int lt = wv; lt < t_end; lt += 4) {
        const int E0 = (sg * TPS + lt) * KT;
        int32_t* dp = sm.jpos[mb] + lt * KT;
        int32_t* dd = sm.jdeath[mb] + lt * KT;
        float* du = sm.ju[mb] + lt * KT;
        if (E0 < src.nkl) {
            const uint32_t off = 4u * (uint32_t)(E0 + lane);
            async_load_lds4(src.xpos, off, dp);
            async_load_lds4(src.xdeath, off, dd);
            async_load_lds4(src.xu, off, du);
        } else {
            const int j = src.c0 + (E0 - src.nkl) + lane;
            const bool real = j <= src.c_end;
            dp[lane] = real ? j : 0;
            if (real) {
                async_load_lds4(src.dr, 4u * (uint32_t)j, dd);
                async_load_lds4(src.ur, 4u * (uint32_t)j, du);
            } else {   // beyond the block's last key: always behind the causal test; any finite value will do
                dd[lane] = INT32_MIN;
                du[lane] = 0.0f;
            }
        }
    }
}

// The runs of tile kinds for one wave (queries qa .. qb) along its block's key set, as tile numbers (wave-uniform):
//   [0,b0) LIST  [b0,b1) LIST_MASK  [b1,b2) EDGE or CONT  [b2,b3) FAST  [b3,b4) DIAG  [b4,..) SKIP
// nkl, nkc: list part and contiguous part in keys (whole tiles); nstay: listed keys that stay selected for the whole
// block; c0: first contiguous key.
struct WaveRuns {
    int b0, b1, b2, b3, b4;
    bool narrow;
};
__device__ __forceinline__ WaveRuns wave_runs(bool wave_live, int nkl, int nkc, int nstay, int qa, int qb, int w, int c0)
{
    WaveRuns r{0, 0, 0, 0, 0, false};
    if (wave_live) {
        const int TL = nkl / KT, NC = nkc / KT;
        r.b0 = min(nstay / KT, TL);
        // contiguous tile m covers positions c0 + 64m .. c0 + 64m + 63
        const int x_sel = qa - w - c0 - (KT - 1);     // m <= x_sel/64: behind every window of the wave
        const int x_fb = qb - w - c0;                 // m >  x_fb/64:  inside every window of the wave
        const int x_fe = qa - c0 - (KT - 1);          // m <= x_fe/64:  in nobody's future
        const int m_sel = x_sel >= 0 ? x_sel / KT + 1 : 0;
        const int m_fb = x_fb >= 0 ? x_fb / KT + 1 : 0;
        const int m_fe = x_fe >= 0 ? x_fe / KT + 1 : 0;
        const int m_skip = (qb - c0) / KT + 1;        // first tile entirely in the wave's future
        r.narrow = m_fb >= m_fe;                      // no tile is both inside every window and in the past
        r.b1 = TL + min(m_sel, NC);
        r.b4 = TL + min(m_skip, NC);
        r.b2 = r.narrow ? r.b4 : TL + min(m_fb, NC);
        r.b3 = r.narrow ? r.b4 : TL + min(m_fe, NC);
        r.b1 = min(r.b1, r.b2);
    }
    return r;
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

// SPARSEK mask backward: du = gradient of L = sum(dO * O) w.r.t. the scores (App. A.3).
//
// For prefix T (query i = T + w) the Jacobian-vector product is s * (g - mean_{S*} g) with
// S*_T = {j <= T : tau_T < u_j < tau_T + 1} and g_j = dL/dm_ij (0 outside the hard top-k).
// Summed over T:   du_j = C_j - sum_{T : j in S*_T} A_T / |S*_T|
//   C_j = sum_i g_ij [j in S*_{i-w}]   column sums   } accumulated by the main kernel while it
//   A_T = sum_j g_{T+w,j} [j in S*_T]  row sums      } recomputes p_ij from q, k, lse (one pass)
// Because tau_T does not decrease once the prefix holds k entries, "j in S*_T" holds on one
// contiguous range of T, found by binary search; |S*_T| and the second term then come from
// difference arrays and prefix sums in an O(n log n) epilogue -- nothing of size n*k is stored.
//
//   g_ij = p_ij (dO_i.v_j)                                          value gate (modes 0, 1, 3)
//        + scale (q_i.k_j) p_ij (m_ij dO_i.v_j - dO_i.o_i)          key gate   (mode 0; mode 3 with m_ij = 1)
// Mode 3 is the straight-through estimator (Sec. 3.4): p, o, lse come from the forward without
// gates and g_ij is the mode 0 derivative taken at m_ij = 1; membership in S* still follows the
// soft mask.
#include "common.hpp"
#include "attn_tiles.hpp"

namespace spk {

constexpr int QB_B = QB;

// implemented in attn_fwd.hip
void launch_block_lists(const sparsek_cfg& c, const int32_t* death, int32_t* lists, int32_t* counts,
                        hipStream_t st);
size_t block_lists_bytes(const sparsek_cfg& c, size_t* counts_offset);

struct BwdWs {
    size_t lists, counts, A, C, diff, G, ab, total;
};
static BwdWs bwd_ws(const sparsek_cfg& c)
{
    BwdWs W;
    size_t coff = 0;
    size_t lb = block_lists_bytes(c, &coff);
    const size_t rows = (size_t)c.B * c.Gu;
    W.lists = 0;
    W.counts = coff;
    size_t off = lb;
    W.A = off; off += align_up(rows * c.n * 4, 256);
    W.C = off; off += align_up(rows * c.n * 4, 256);
    W.diff = off; off += align_up(rows * (c.n + 1) * 4, 256);
    W.G = off; off += align_up(rows * (size_t)(c.n + 1) * 8, 256);
    W.ab = off; off += align_up(rows * (size_t)c.n * 8, 256);
    W.total = off;
    return W;
}
size_t mask_bwd_ws_bytes(const sparsek_cfg& c) { return bwd_ws(c).total; }

__global__ void zero_kernel(uint32_t* p, size_t nwords)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

// strict membership in the fractional set, decided in fp64 (both sides exact)
__device__ __forceinline__ bool strictly_fractional(float uj, float tauT)
{
    return (uj > tauT) && ((double)uj < (double)tauT + 1.0);
}

template <typename T>
__device__ __forceinline__ float ldv(const T* p);
template <>
__device__ __forceinline__ float ldv<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ldv<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

// ---------------------------------------------------------------------------------
// Generic main kernel: one wave per query, lanes over the selected keys.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void mask_bwd_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ kk, const T* __restrict__ v, const float* __restrict__ u,
    const float* __restrict__ tau, const int32_t* __restrict__ death, const int32_t* __restrict__ lists,
    const int32_t* __restrict__ counts, const T* __restrict__ o, const float* __restrict__ lse,
    const T* __restrict__ dO, float* __restrict__ A, float* __restrict__ C, int H, int Gu, int n, int d, int k,
    int w, int gate_mode, float scale, int nb)
{
    __shared__ float qs[4][128], ds[4][128];
    const int blk = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i0 = blk * QB_B;
    const T* qh = q + (size_t)bh * n * d;
    const T* kh = kk + (size_t)bh * n * d;
    const T* vh = v + (size_t)bh * n * d;
    const T* oh = o + (size_t)bh * n * d;
    const T* dh = dO + (size_t)bh * n * d;
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int32_t* list = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    const int cnt = counts[(size_t)row * nb + blk];
    const int c0 = max(0, i0 - w + 1);

    for (int qi = wv; qi < QB_B; qi += 4) {
        const int i = i0 + qi;
        if (i >= n) break;
        const int Tp = i - w;
        if (Tp < k) continue;  // prefixes with at most k entries have every gate at 1: no gradient
        float dpart = 0.0f;
        for (int c = lane; c < d; c += 64) {
            const float qv = ldv(qh + (size_t)i * d + c), dv = ldv(dh + (size_t)i * d + c);
            qs[wv][c] = qv;
            ds[wv][c] = dv;
            dpart += dv * ldv(oh + (size_t)i * d + c);
        }
        const float Di = wave_sum_f32(dpart);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        const float tauT = tr[Tp];
        const float lse_i = lse[(size_t)bh * n + i];
        const int n_cont = max(0, Tp - c0 + 1);  // contiguous keys already outside the window
        const int total = cnt + n_cont;
        float rowsum = 0.0f;
        for (int e0 = 0; e0 < total; e0 += 64) {
            const int e = e0 + lane;
            float gf = 0.0f;
            int j = -1;
            if (e < total) {
                j = (e < cnt) ? list[e] : c0 + (e - cnt);
                const float uj = ur[j];
                if (dr[j] > Tp && strictly_fractional(uj, tauT)) {
                    const float m = clip01(uj - tauT);
                    float qk = 0.0f, dov = 0.0f;
                    const T* kj = kh + (size_t)j * d;
                    const T* vj = vh + (size_t)j * d;
                    for (int c = 0; c < d; c++) {
                        qk += qs[wv][c] * ldv(kj + c);
                        dov += ds[wv][c] * ldv(vj + c);
                    }
                    const float s = scale * qk * (gate_mode == 0 ? m : 1.0f);
                    const float p = __expf(s - lse_i);
                    gf = p * dov;
                    if (gate_mode == 0) gf += scale * qk * p * (m * dov - Di);
                    if (gate_mode == 3) gf += scale * qk * p * (dov - Di);
                }
            }
            if (gf != 0.0f) unsafeAtomicAdd(C + (size_t)row * n + j, gf);
            rowsum += gf;
        }
        rowsum = wave_sum_f32(rowsum);
        if (lane == 0 && rowsum != 0.0f) unsafeAtomicAdd(A + (size_t)row * n + Tp, rowsum);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    }
}

// ---------------------------------------------------------------------------------
// MFMA main kernel (bf16, D = 64 or 128).  Same blocking as the forward: 128 queries x 4
// waves, 64-key tiles gathered straight into LDS.  The candidates of a block are its top-k
// list and the contiguous keys that have already left some query's window; before any
// arithmetic they are compacted to the keys that can carry a strictly fractional gate for
// some live query of the block:
//     tau_lo < u_j < tau_hi + 1     (tau_lo, tau_hi: extremes of tau over the block's prefixes)
//     j <= T_max  and  death_j > T_min   (in the prefix of, and still selected for, some query)
// Saturated keys (gate 1 for every query of the block) and unselected window leavers drop out
// here, which removes a large share of the tiles.  Per tile two contractions over d,
//   S^T  = K . Q^T    (recomputes the logits)      DV^T = V . dO^T   (dO_i . v_j),
// then g_ij elementwise; row sums stay in the lane that owns the query, column sums are
// reduced across the 32 query lanes with a halving butterfly (31 exchanges for 32 keys, all
// of them lane permutes in the vector ALU: permlane16_swap, DPP row rotate / mirror / quad),
// combined over the 4 waves in LDS and added to C[] with one atomic per key and tile.
// ---------------------------------------------------------------------------------
constexpr int RAW = 1024;  // candidates examined per segment (4 per thread); at most that many survive

// g_ij for one (key, query) pair from the two dot products (see the header comment).
// SURE: the key is selected and strictly fractional for every query of the block (decided once
// per key when the candidates are compacted), so the per-pair tests are skipped.
template <int MODE, bool SURE>
__device__ __forceinline__ float bwd_pair(float qk, float dov, int Jj, int Lj, float uj, int Tp, float tau_q,
                                          float tau1_up, float scale, float c2, float lse2, float Di)
{
    const float mg = clip01(uj - tau_q);
    const float p = __builtin_amdgcn_exp2f(fmaf(qk * (MODE == 0 ? mg : 1.0f), c2, -lse2));
    float g = dov;
    if (MODE == 0) g = fmaf(scale * qk, fmaf(mg, dov, -Di), dov);
    if (MODE == 3) g = fmaf(scale * qk, dov - Di, dov);
    if (SURE) return g * p;
    // key j counts for prefix T  <=>  j <= T < death_j  <=>  (unsigned)(T - j) < death_j - j
    // (T = -1 for a query without gradient, death_j - j = 0 for padding: never true)
    const bool valid = (uint32_t)(Tp - Jj) < (uint32_t)Lj;
    // strictly fractional gate: tau < u < tau + 1.  tau1_up is tau + 1 rounded up to fp32:
    // for an fp32 score, u < tau + 1 (exactly)  <=>  u < tau1_up
    const bool frac = (uj > tau_q) && (uj < tau1_up);
    return (valid && frac) ? g * p : 0.0f;
}

// Column sums over the 32 queries of a half-wave for the 16 keys of one key half: halving
// butterfly.  gv[r] is this lane's g for key 32 * mb + 8 * (r / 4) + 4 * half + r % 4.  After the
// step with partner lane ^ b a lane keeps the values whose index has the matching bit equal to its
// own lane bit; after four steps lanes c and c ^ 1 hold the two halves of the total of value
// index c >> 1, which the even one adds to the tile's sums in LDS.
__device__ __forceinline__ void bwd_column_sums(float (&gv)[16], float* colsum, int mb, int lane, int half)
{
    // The lane's target address is recomputed here on purpose (the empty asm hides that it is loop-invariant):
    // hoisted, it was one of the values the register allocator parked in scratch memory, and a reload inside
    // the tile loop waits for every outstanding memory operation, the prefetched tile included.
    asm volatile("" : "+v"(lane));
    half = lane >> 5;
    const int c31 = lane & 31;
#pragma unroll
    for (int r = 0; r < 8; r++) {
        // lane ^ 16: v_permlane16_swap hands the even row the odd row's first operand and the odd
        // row the even row's second operand, which is exactly "send one, keep the other"
        const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(gv[r]), __float_as_uint(gv[r + 8]), false, false);
        gv[r] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const bool up = c31 & 8;
        const float send = up ? gv[r] : gv[r + 4];
        const float keep = up ? gv[r + 4] : gv[r];
        gv[r] = keep + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), 0x128, 0xF, 0xF, true));  // row_ror:8 = lane ^ 8
    }
#pragma unroll
    for (int r = 0; r < 2; r++) {
        const bool up = c31 & 4;
        const float send = up ? gv[r] : gv[r + 2];
        const float keep = up ? gv[r + 2] : gv[r];
        int x = __builtin_amdgcn_update_dpp(0, __float_as_int(send), 0x141, 0xF, 0xF, true);  // half-row mirror: lane ^ 7
        x = __builtin_amdgcn_update_dpp(0, x, 0x1B, 0xF, 0xF, true);                          // quad reverse: lane ^ 3
        gv[r] = keep + __int_as_float(x);
    }
    {
        const bool up = c31 & 2;
        const float send = up ? gv[0] : gv[1];
        const float keep = up ? gv[1] : gv[0];
        gv[0] = keep + dpp_f32(send, 1);  // quad swap [2,3,0,1] = lane ^ 2
    }
    const float tot = gv[0] + dpp_f32(gv[0], 0);  // quad swap [1,0,3,2] = lane ^ 1
    const int vi = c31 >> 1;
    const int keyn = 32 * mb + 8 * (vi >> 2) + 4 * half + (vi & 3);
    if (!(c31 & 1) && tot != 0.0f) atomicAdd(&colsum[keyn], tot);
}

// What a wave carries from one tile to the next: the second key half's dot products, whose
// elementwise work runs under the next tile's first MFMAs.
struct BwdCarry {
    f32x16 s1, d1;
};

// One step of the software pipeline over the tiles of a segment (two key halves 0/1 per tile):
//   phase A:  MFMAs of (tile t, half 0)   with the elementwise work of (tile t-1, half 1)
//   phase B:  MFMAs of (tile t, half 1)   with the elementwise work of (tile t, half 0)
// each followed by the column sums of the 32 keys just finished.
// PREV = false on a segment's first tile, CUR = false for the drain step after its last one;
// SP / SC: tile t-1 / tile t holds only keys that need no per-pair tests.
// Every MFMA slot carries 32 / (D / 8) pairs of elementwise work; the LDS operand of a slot is
// requested DEPTH slots earlier.
template <int D, int MODE, bool PREV, bool CUR, bool SP, bool SC>
__device__ __forceinline__ void bwd_step(MfmaSmem<D, 16>& sm, float* colsum_prev, float* colsum_cur, int buf, int base, int base_prev,
                                         int col, int half, int lane, int Tp, float tau_q, float tau1_up,
                                         float scale, float lse2, float Di, const bf16x8 (&qreg)[D / 16],
                                         const bf16x8 (&dreg)[D / 16], BwdCarry& cy, float& rowsum)
{
    using S = MfmaSmem<D, 16>;
    constexpr int DS = D / 16;
    constexpr int NM = 2 * DS;     // MFMA slots per key half: K and V fragments alternate
    constexpr int EPM = 16 / NM;   // pairs of elementwise work per slot
    constexpr int DEPTH = 2;
    static_assert(NM % DEPTH == 0, "the ring runs on from phase A into phase B");
    static_assert(EPM * NM == 16 && (4 % EPM) == 0, "head dim 64 or 128");
    // Per-lane LDS addresses (metadata groups, operand rows) are formed again in every step: as loop-invariant
    // values they were spilled, and a reload inside the tile loop waits for the prefetched tile as well.
    asm volatile("" : "+v"(half), "+v"(col));
    const unsigned char* kbuf = sm.kb[buf];
    const unsigned char* vbuf = sm.vb[buf];
    const float c2 = scale * 1.4426950408889634f;
    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    int off[2];
#pragma unroll
    for (int mb = 0; mb < 2; mb++) {
        const int row = 32 * mb + col;
        off[mb] = (row % S::NL) * S::GSK + (row / S::NL) * S::RB + 16 * half;
    }
    auto operand = [&](int n) -> bf16x8 {  // n = slot number over both phases, a constant after unrolling
        const int mb = n / NM, s = (n % NM) / 2;
        return *(const bf16x8*)(((n & 1) ? vbuf : kbuf) + off[mb] + 32 * s);
    };
    bf16x8 ring[DEPTH];
    if (CUR) {
#pragma unroll
        for (int n = 0; n < DEPTH; n++) ring[n] = operand(n);
    }
    f32x16 s0, d0;
    float gv[16];
    int4 J4 = {0, 0, 0, 0}, L4 = {0, 0, 0, 0};
    float4 U4;
    auto pairs = [&](auto sure_c, int n, int mb, int mbase, const f32x16& as, const f32x16& ad, float* gout) {
        constexpr bool SURE = decltype(sure_c)::value;
#pragma unroll
        for (int e0 = 0; e0 < EPM; e0++) {
            const int r = n * EPM + e0, g4 = r / 4, e = r % 4;
            if (e == 0) {
                const int kb = mbase + 32 * mb + 8 * g4 + 4 * half;
                if (!SURE) {
                    J4 = *(const int4*)&sm.jpos[kb];
                    L4 = *(const int4*)&sm.jlast[kb];
                }
                U4 = *(const float4*)&sm.ju[kb];
            }
            const int Jj = e == 0 ? J4.x : e == 1 ? J4.y : e == 2 ? J4.z : J4.w;
            const int Lj = e == 0 ? L4.x : e == 1 ? L4.y : e == 2 ? L4.z : L4.w;
            const float uj = e == 0 ? U4.x : e == 1 ? U4.y : e == 2 ? U4.z : U4.w;
            const float g = bwd_pair<MODE, SURE>(as[r], ad[r], Jj, Lj, uj, Tp, tau_q, tau1_up, scale, c2, lse2, Di);
            gout[r] = g;
            rowsum += g;
        }
    };
    // ---- phase A ----
    static_for<0, NM>([&](auto nc) {
        constexpr int n = decltype(nc)::value;
        if (CUR) {
            const bf16x8 cur = ring[n % DEPTH];
            constexpr int s = n / 2;
            if (n & 1) d0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, dreg[s], n < 2 ? zero : d0, 0, 0, 0);
            else s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qreg[s], n < 2 ? zero : s0, 0, 0, 0);
            ring[n % DEPTH] = operand(n + DEPTH);
        }
        if (PREV) pairs(std::bool_constant<SP>{}, n, 1, base_prev, cy.s1, cy.d1, gv);
        __builtin_amdgcn_sched_barrier(0);
    });
    if (PREV) bwd_column_sums(gv, colsum_prev, 1, lane, half);
    // ---- phase B ----
    if (CUR) {
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NM>([&](auto nc) {
            constexpr int n = decltype(nc)::value;
            const bf16x8 cur = ring[n % DEPTH];
            constexpr int s = n / 2;
            if (n & 1) cy.d1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, dreg[s], n < 2 ? zero : cy.d1, 0, 0, 0);
            else cy.s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qreg[s], n < 2 ? zero : cy.s1, 0, 0, 0);
            if (n + DEPTH < NM) ring[n % DEPTH] = operand(NM + n + DEPTH);
            pairs(std::bool_constant<SC>{}, n, 0, base, s0, d0, gv);
            __builtin_amdgcn_sched_barrier(0);
        });
        bwd_column_sums(gv, colsum_cur, 0, lane, half);
    }
}

template <int D, int MODE>
__global__ __launch_bounds__(256, 2) void mask_bwd_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ kk, const uint16_t* __restrict__ v,
    const float* __restrict__ u, const float* __restrict__ tau, const int32_t* __restrict__ death,
    const int32_t* __restrict__ lists, const int32_t* __restrict__ counts, const uint16_t* __restrict__ o,
    const float* __restrict__ lse, const uint16_t* __restrict__ dO, float* __restrict__ A, float* __restrict__ C,
    int H, int Gu, int n, int k, int w, float scale, int nb, int BH, int q_begin, int q_rows)
{
    static_assert(RAW <= SEG, "survivors of one segment must fit the staged metadata");
    __shared__ __align__(16) MfmaSmem<D, 16> sm;
    __shared__ float colsum[3][KT];  // tile t adds into [t % 3] under tiles t and t+1; flushed under tile t+2
    __shared__ __align__(16) int wcnt[2][RAW / 256][4];  // survivors per (class, round, wave) of the compaction
    __shared__ float tred[2][4];
    constexpr int DS = D / 16;
    int bh, blk;
    {
        const int id = blockIdx.x;
        if (BH % 8 == 0) {
            const int xcd = id & 7, slot = id >> 3;
            bh = (slot / nb) * 8 + xcd;
            blk = nb - 1 - (slot % nb);
        } else {
            bh = id / nb;
            blk = nb - 1 - (id % nb);
        }
    }
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;
    const int i0 = blk * QB;
    // Queries before q_begin do not exist (a caller that attends a chunk against retained keys);
    // q, o, dO and lse then hold q_rows rows per head, the first of them query q_begin.
    if (i0 + QB <= q_begin) return;
    const ptrdiff_t qo = q_rows ? (ptrdiff_t)bh * q_rows - q_begin : (ptrdiff_t)bh * n;
    // prefixes of the block's queries that carry gradient: T = i - w with T >= k (prefixes with at
    // most k entries have every gate at 1)
    const int Tmax = min(n - 1, i0 + QB - 1) - w;
    const int Tmin = max(i0 - w, k);
    if (Tmax < Tmin) return;
    const uint16_t* kh = kk + (size_t)bh * n * D;
    const uint16_t* vh = v + (size_t)bh * n * D;
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int32_t* list = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    const int cnt = counts[(size_t)row * nb + blk];
    const int c0 = max(0, i0 - w + 1);           // contiguous candidates: c0 .. Tmax (outside some query's window)
    const int ncont = max(0, Tmax - c0 + 1);
    const int ncand = cnt + ncont;

    const int qa = i0 + 32 * wv;
    const int qb = min(qa + 31, n - 1);
    const int qi = qa + col;
    const int qrow = min(qi, n - 1);
    const bool qlive = (qi < n) && (qi - w >= k);
    const int Tp = qlive ? qi - w : -1;
    const bool wave_live = (qa < n) && (qb - w >= k);
    // Order of the prologue's loads: the small, cache-resident ones first (tau, lse, then the
    // candidates with their dependent score / death reads), the cold query rows of Q, dO, O last.
    // Loads complete in issue order, so this lets the candidates be classified and compacted, and
    // the first tile's gather be issued, while the rows are still on their way from HBM.
    const float tau_q = qlive ? tr[Tp] : 0.0f;
    const float lse2 = lse[qo + qrow] * 1.4426950408889634f;
    // candidates of a segment: position, death - position, score (4 per thread)
    int cj[RAW / 256], cl[RAW / 256];
    float cu[RAW / 256];
    auto load_candidates = [&](int r0) {
        // Branch-free, and independent of the list length until the values are used: the list
        // slots are read up to k (those beyond cnt hold stale numbers, clamped into the row and
        // discarded afterwards), so that cnt, the list and then all score / death reads are two
        // round trips in flight together rather than a chain of dependent ones.
        int lv[RAW / 256];
#pragma unroll
        for (int x = 0; x < RAW / 256; x++) lv[x] = list[min(r0 + 256 * x + tid, k - 1)];
#pragma unroll
        for (int x = 0; x < RAW / 256; x++) {
            const int E = r0 + 256 * x + tid;
            cj[x] = E < cnt ? min(max(lv[x], 0), n - 1) : min(c0 + max(E - cnt, 0), n - 1);
        }
#pragma unroll
        for (int x = 0; x < RAW / 256; x++) {
            cu[x] = ur[cj[x]];
            cl[x] = dr[cj[x]];  // death; turned into death - position when the candidate is classified
        }
    };
    load_candidates(0);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 qreg[DS], dreg[DS], oreg[DS];
#pragma unroll
    for (int s = 0; s < DS; s++) {
        const size_t off = (qo + qrow) * D + 16 * s + 8 * half;
        qreg[s] = *(const bf16x8*)(q + off);
        dreg[s] = *(const bf16x8*)(dO + off);
        oreg[s] = *(const bf16x8*)(o + off);
    }
    __builtin_amdgcn_sched_barrier(0);
    const float tau1_up = __double2float_ru((double)tau_q + 1.0);
    {
        const float lo = wave_min_f32(qlive ? tau_q : INFINITY);
        const float hi = wave_max_f32(qlive ? tau_q : -INFINITY);
        if (lane == 0) { tred[0][wv] = lo; tred[1][wv] = hi; }
    }
    float Di = 0.0f;       // dO_i . o_i, formed when the rows have arrived (first segment with tiles)
    bool have_di = false;
    float rowsum = 0.0f;
    BwdCarry cy;
    if (tid < 3 * KT) colsum[tid / KT][tid % KT] = 0.0f;
    const bool all_live = (i0 - w >= k) && (i0 + QB <= n);  // every lane of the block owns a query with gradient
    __syncthreads();
    const float tau_lo = fminf(fminf(tred[0][0], tred[0][1]), fminf(tred[0][2], tred[0][3]));
    const float tau_hi = fmaxf(fmaxf(tred[1][0], tred[1][1]), fmaxf(tred[1][2], tred[1][3]));
    const float tau_hi1 = __double2float_ru((double)tau_hi + 1.0);
    const float tau_lo1 = __double2float_ru((double)tau_lo + 1.0);

    for (int r0 = 0; r0 < ncand; r0 += RAW) {
        // ---- examine RAW candidates, keep those that can matter to this block ----
        // class 1 ("sure"): selected and strictly fractional for every query of the block -- placed
        // first, their tiles skip the per-pair tests; class 2: the other survivors
        int pre[RAW / 256], cls[RAW / 256];
        if (r0 > 0) load_candidates(r0);
#pragma unroll
        for (int x = 0; x < RAW / 256; x++) {
            const int j = cj[x], life = cl[x] - cj[x];  // death_j = j + life
            const float uj = cu[x];
            cl[x] = life;
            const bool keep = (r0 + 256 * x + tid < ncand) && (uj > tau_lo) && (uj < tau_hi1) && (j <= Tmax) && (j + life > Tmin) && (life > 0);
            const bool sure = keep && all_live && (uj > tau_hi) && (uj < tau_lo1) && (j <= Tmin) && (j + life > Tmax);
            cls[x] = sure ? 1 : keep ? 2 : 0;
            const unsigned long long b1 = __ballot(cls[x] == 1), b2 = __ballot(cls[x] == 2);
            const unsigned long long bal = cls[x] == 1 ? b1 : b2;
            pre[x] = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
            if (lane == 0) {
                wcnt[0][x][wv] = __popcll(b1);
                wcnt[1][x][wv] = __popcll(b2);
            }
        }
        __syncthreads();  // counts visible; the previous segment's tiles and column sums are done with
        int n1 = 0, n2 = 0, at1[RAW / 256], at2[RAW / 256];
#pragma unroll
        for (int x = 0; x < RAW / 256; x++) {
            const int4 c1 = *(const int4*)wcnt[0][x];
            const int4 c2 = *(const int4*)wcnt[1][x];
            at1[x] = n1 + (wv > 0 ? c1.x : 0) + (wv > 1 ? c1.y : 0) + (wv > 2 ? c1.z : 0);
            at2[x] = n2 + (wv > 0 ? c2.x : 0) + (wv > 1 ? c2.y : 0) + (wv > 2 ? c2.z : 0);
            n1 += c1.x + c1.y + c1.z + c1.w;
            n2 += c2.x + c2.y + c2.z + c2.w;
        }
        const int kept = n1 + n2;
#pragma unroll
        for (int x = 0; x < RAW / 256; x++) {
            if (cls[x] != 0) {
                const int idx = (cls[x] == 1 ? at1[x] : n1 + at2[x]) + pre[x];
                sm.jpos[idx] = cj[x];
                sm.jlast[idx] = cl[x];
                sm.ju[idx] = cu[x];
            }
        }
        const int nsure = n1 / KT;  // tiles made of class-1 keys only
        const int seg_n = (kept + KT - 1) / KT * KT;
        if (kept + tid < seg_n) {  // padding of the last tile: row 0, never valid
            sm.jpos[kept + tid] = 0;
            sm.jlast[kept + tid] = 0;
            sm.ju[kept + tid] = 0.0f;
        }
        __syncthreads();
        const int ntiles = seg_n / KT;
        if (ntiles == 0) continue;
        issue_tile_loads<D, 16>(sm, 0, sm.jpos, kh, vh, wv, lane);
        if (!have_di) {
            float dpart = 0.0f;
#pragma unroll
            for (int s = 0; s < DS; s++)
#pragma unroll
                for (int e = 0; e < 8; e++) dpart += (float)dreg[s][e] * (float)oreg[s][e];
            Di = dpart + __shfl_xor(dpart, 32, 64);
            have_di = true;
        }
        // column sums of tile t are formed under tiles t and t+1, in colsum[t % 3], and handed to
        // C[] under tile t+2; tile t+3 is the next one to use that buffer
        auto flush = [&](int tt, int c) {
            const float cs = colsum[tt % 3][c];
            if (cs != 0.0f) unsafeAtomicAdd(C + (size_t)row * n + sm.jpos[tt * KT + c], cs);
            colsum[tt % 3][c] = 0.0f;
        };
        for (int t = 0; t < ntiles; t++) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();  // tile t landed; everybody is done with the MFMAs of tile t-1 and the sums of tile t-2
            if (t + 1 < ntiles) issue_tile_loads<D, 16>(sm, (t + 1) & 1, sm.jpos + (t + 1) * KT, kh, vh, wv, lane);
            if (t >= 2 && tid < KT) flush(t - 2, tid);
            if (!wave_live) continue;
#define SPK_STEP(PREV, CUR, SP, SC)                                                                              \
    bwd_step<D, MODE, PREV, CUR, SP, SC>(sm, colsum[(t + 2) % 3], colsum[t % 3], t & 1, t * KT, (t - 1) * KT, col, half, lane, Tp, \
                                         tau_q, tau1_up, scale, lse2, Di, qreg, dreg, cy, rowsum)
            if (t == 0) {
                if (nsure > 0) SPK_STEP(false, true, false, true);
                else SPK_STEP(false, true, false, false);
            } else if (t < nsure) {
                SPK_STEP(true, true, true, true);
            } else if (t == nsure) {
                SPK_STEP(true, true, true, false);
            } else {
                SPK_STEP(true, true, false, false);
            }
        }
        if (wave_live) {
            const int t = ntiles;
            if (nsure == ntiles) SPK_STEP(true, false, true, false);
            else SPK_STEP(true, false, false, false);
        }
#undef SPK_STEP
        __syncthreads();
        if (tid < 2 * KT) {  // column sums of the segment's last two tiles
            const int tt = ntiles - 2 + tid / KT;
            if (tt >= 0) flush(tt, tid % KT);
        }
        __syncthreads();  // ... before the next segment overwrites the positions
    }
    const float rs = rowsum + __shfl_xor(rowsum, 32, 64);
    if (qlive && half == 0 && rs != 0.0f) unsafeAtomicAdd(A + (size_t)row * n + Tp, rs);
}

template <int D>
static void launch_bwd_mfma(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                            const float* tau, const int32_t* death, const int32_t* lists, const int32_t* counts,
                            const void* o, const float* lse, const void* dO, float* A, float* C, int nb,
                            hipStream_t st, int q_begin, int q_rows)
{
    const int BH = c.B * c.H;
    dim3 grid(nb * BH);
#define SPK_LAUNCH_B(MODE)                                                                                    \
    hipLaunchKernelGGL((mask_bwd_mfma_kernel<D, MODE>), grid, dim3(256), 0, st, (const uint16_t*)q,           \
                       (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, (const uint16_t*)o, \
                       lse, (const uint16_t*)dO, A, C, c.H, c.Gu, c.n, c.k, c.w, c.softmax_scale, nb, BH, q_begin, q_rows)
    if (c.gate_mode == 0) SPK_LAUNCH_B(0);
    else if (c.gate_mode == 3) SPK_LAUNCH_B(3);
    else SPK_LAUNCH_B(1);
#undef SPK_LAUNCH_B
}

// ---------------------------------------------------------------------------------
// Epilogue 1: per key j the range [a_j, b_j] of prefixes T with j in S*_T; difference array
// of |S*_T|.  tau is non-decreasing for T >= k-1, so both ends come from binary searches:
//   b_j = last  T in [max(j,k), n-1] with tau_T < u_j
//   a_j = first T in [max(j,k), n-1] with u_j < tau_T + 1      (compared in fp64, exact)
// A workgroup holds every stride-th threshold of its row in LDS (all of them up to n = 8192);
// a search runs on those samples first and finishes in global memory inside one stride.
// ---------------------------------------------------------------------------------
constexpr int RS_MAX = 8192;  // sampled thresholds per row held in LDS

// first T in [lo, n) with pred(tau_T), n if none; pred is monotone (false ... false true ... true)
template <typename Pred>
__device__ __forceinline__ int first_true(const float* __restrict__ tr, const float* ts, int lo, int n, int stride,
                                          int ns, Pred pred)
{
    const int ifirst = (lo + stride - 1) / stride;  // samples sit at T = i * stride
    int x = ifirst, y = ns;
    while (x < y) {
        const int m = (x + y) >> 1;
        if (pred(ts[m])) y = m;
        else x = m + 1;
    }
    int t0 = (x == ifirst) ? lo : (x - 1) * stride + 1;  // samples before x are false
    int t1 = (x < ns) ? x * stride : n;                  // sample x is true
    while (t0 < t1) {
        const int m = (t0 + t1) >> 1;
        if (pred(tr[m])) t1 = m;
        else t0 = m + 1;
    }
    return t0;
}

__global__ __launch_bounds__(1024) void mask_bwd_ranges_kernel(const float* __restrict__ u,
                                                                const float* __restrict__ tau, int n, int k,
                                                                int32_t* __restrict__ diff, int2* __restrict__ ab)
{
    __shared__ float ts[RS_MAX];
    const int row = blockIdx.y;
    const float* tr = tau + (size_t)row * n;
    const int stride = (n + RS_MAX - 1) / RS_MAX;
    const int ns = (n + stride - 1) / stride;
    for (int i = threadIdx.x; i < ns; i += blockDim.x) ts[i] = tr[(size_t)i * stride];
    __syncthreads();
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    int a = 1, b = 0;
    if (j < n) {
        const float uj = u[(size_t)row * n + j];
        const int lo = max(j, k);  // shorter prefixes have every gate at 1: S* empty
        if (lo <= n - 1) {
            b = first_true(tr, ts, lo, n, stride, ns, [&](float t) { return !(t < uj); }) - 1;
            a = first_true(tr, ts, lo, n, stride, ns, [&](float t) { return (double)uj < (double)t + 1.0; });
        }
        ab[(size_t)row * n + j] = make_int2(a, b);
    }
    // difference array: +1 at a_j, -1 at b_j + 1.  Two addresses collect most of the updates and
    // would serialise them: every key j <= k that is fractional from the start has a_j = k (one
    // add per wave instead), and every key still fractional at the end has b_j + 1 = n, an entry
    // the prefix sum never reads (dropped).
    const bool any = a <= b;
    int32_t* dr = diff + (size_t)row * (n + 1);
    const unsigned long long at_k = __ballot(any && a == k);
    if (any && a != k) atomicAdd(dr + a, 1);
    if (at_k != 0 && (threadIdx.x & 63) == 0) atomicAdd(dr + k, (int)__popcll(at_k));
    if (any && b + 1 < n) atomicAdd(dr + b + 1, -1);
}

// Exclusive prefix sum of one value per thread over the 1024 threads of a workgroup; `total`
// receives the sum over all of them.
template <typename T>
__device__ __forceinline__ T block_exclusive_scan_1024(T x, T* wtot /* [16] LDS */, T& total)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    T inc = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const T y = __shfl_up(inc, o, 64);
        if (lane >= o) inc += y;
    }
    __syncthreads();  // wtot may still be read from a previous call
    if (lane == 63) wtot[wv] = inc;
    __syncthreads();
    T before = inc - x;
    total = T(0);
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const T w = wtot[i];
        if (i < wv) before += w;
        total += w;
    }
    return before;
}

// Epilogue 2, one workgroup per row:
//   |S*_T| = prefix sum of diff;   G_T = sum_{T' <= T} A_T' / |S*_T'|  (fp64);
//   du_j = C_j - (G[b_j] - G[a_j - 1]).
// The prefix sums go over chunks of 8192 prefixes, 8 consecutive ones per thread, read in one
// batch; G is written to global memory and read back by the same workgroup after a barrier.
constexpr int SCAN_PER = 8;
__global__ __launch_bounds__(1024) void mask_bwd_scan_final_kernel(const float* __restrict__ A,
                                                                    const int32_t* __restrict__ diff,
                                                                    const float* __restrict__ C,
                                                                    const int2* __restrict__ ab, int n,
                                                                    double* __restrict__ G, float* __restrict__ du)
{
    __shared__ int cw[16];
    __shared__ double gw[16];
    const int row = blockIdx.x, tid = threadIdx.x;
    const float* Ar = A + (size_t)row * n;
    const int32_t* dr = diff + (size_t)row * (n + 1);
    double* Gr = G + (size_t)row * (n + 1);  // Gr[T+1] = sum_{T'<=T}; Gr[0] = 0
    if (tid == 0) Gr[0] = 0.0;
    int cnt_carry = 0;
    double g_carry = 0.0;
    for (int base = 0; base < n; base += 1024 * SCAN_PER) {
        const int i0 = base + SCAN_PER * tid;
        int dv[SCAN_PER];
        float av[SCAN_PER];
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++) {
            const int i = min(i0 + e, n - 1);
            dv[e] = dr[i];
            av[e] = Ar[i];
        }
        int csum = 0;
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++) {
            if (i0 + e >= n) dv[e] = 0;
            csum += dv[e];
        }
        int ctot;
        int cnt = cnt_carry + block_exclusive_scan_1024<int>(csum, cw, ctot);
        double gl[SCAN_PER], gsum = 0.0;
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++) {
            cnt += dv[e];
            if (cnt > 0 && i0 + e < n) gsum += (double)av[e] / (double)cnt;
            gl[e] = gsum;
        }
        double gtot;
        const double run = g_carry + block_exclusive_scan_1024<double>(gsum, gw, gtot);
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++)
            if (i0 + e < n) Gr[i0 + e + 1] = run + gl[e];
        cnt_carry += ctot;
        g_carry += gtot;
    }
    __syncthreads();  // the row's G is complete and visible to the whole workgroup
    const int2* abr = ab + (size_t)row * n;
    const float* Cr = C + (size_t)row * n;
    float* dur = du + (size_t)row * n;
    for (int base = 0; base < n; base += 1024 * SCAN_PER) {
        int2 r[SCAN_PER];
        float cv[SCAN_PER];
        double hi[SCAN_PER], lo[SCAN_PER];
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++) {
            const int j = min(base + 1024 * e + tid, n - 1);
            r[e] = abr[j];
            cv[e] = Cr[j];
        }
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++) {
            const bool any = r[e].x <= r[e].y;
            hi[e] = Gr[any ? r[e].y + 1 : 0];
            lo[e] = Gr[any ? r[e].x : 0];
        }
#pragma unroll
        for (int e = 0; e < SCAN_PER; e++) {
            const int j = base + 1024 * e + tid;
            if (j < n) dur[j] = (float)((double)cv[e] - (hi[e] - lo[e]));
        }
    }
}

int launch_mask_bwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, const void* o, const float* lse, const void* dO,
                    float* du, void* ws, hipStream_t st, int q_begin, int q_rows, int t_min)
{
    const BwdWs W = bwd_ws(c);
    char* base = (char*)ws;
    const int rows = c.B * c.Gu;
    const int nb = (c.n + QB_B - 1) / QB_B;
    int32_t* lists = (int32_t*)(base + W.lists);
    int32_t* counts = (int32_t*)(base + W.counts);
    float* A = (float*)(base + W.A);
    float* C = (float*)(base + W.C);
    int32_t* diff = (int32_t*)(base + W.diff);
    double* G = (double*)(base + W.G);
    int2* ab = (int2*)(base + W.ab);
    if (c.gate_mode == 2 || c.k <= 0 || c.n <= c.w) {
        // no soft gate anywhere: the gradient is identically zero
        hipLaunchKernelGGL(zero_kernel, dim3(512), dim3(256), 0, st, (uint32_t*)du, (size_t)rows * c.n);
        return launch_status();
    }
    // A, C, diff are contiguous: clear them with one fill kernel (safe under graph capture)
    hipLaunchKernelGGL(zero_kernel, dim3(512), dim3(256), 0, st, (uint32_t*)(base + W.A), (W.G - W.A) / 4);
    // t_min: thresholds of earlier prefixes are not available (and no query uses them)
    hipLaunchKernelGGL(mask_bwd_ranges_kernel, dim3((c.n + 1023) / 1024, rows), dim3(1024), 0, st, u, tau, c.n,
                       std::max(c.k, t_min), diff, ab);
    launch_block_lists(c, death, lists, counts, st);
    dim3 grid(nb, c.B * c.H);
    if (c.dtype == SPARSEK_BF16 && (c.d == 64 || c.d == 128) && (uint64_t)c.n * c.d * 2 <= 0xFFFFFFFFull) {
        if (c.d == 64)
            launch_bwd_mfma<64>(c, q, k, v, u, tau, death, lists, counts, o, lse, dO, A, C, nb, st, q_begin, q_rows);
        else
            launch_bwd_mfma<128>(c, q, k, v, u, tau, death, lists, counts, o, lse, dO, A, C, nb, st, q_begin, q_rows);
    } else if (q_begin != 0 || q_rows != 0 || t_min != 0)
        return SPARSEK_ERR_UNSUPPORTED;  // the offset-query form exists on the MFMA path only
    else if (c.dtype == SPARSEK_F32)
        hipLaunchKernelGGL(mask_bwd_generic_kernel<float>, grid, dim3(256), 0, st, (const float*)q, (const float*)k,
                           (const float*)v, u, tau, death, lists, counts, (const float*)o, lse, (const float*)dO, A, C,
                           c.H, c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale, nb);
    else
        hipLaunchKernelGGL(mask_bwd_generic_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)q,
                           (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, (const uint16_t*)o,
                           lse, (const uint16_t*)dO, A, C, c.H, c.Gu, c.n, c.d, c.k, c.w, c.gate_mode,
                           c.softmax_scale, nb);
    hipLaunchKernelGGL(mask_bwd_scan_final_kernel, dim3(rows), dim3(1024), 0, st, A, diff, C, ab, c.n, G, du);
    return launch_status();
}

}  // namespace spk

// Stage 3: gated attention forward over top-k + sliding window (Sec. 3.2, 3.4, 3.5).
//
// Key fact used everywhere (follows from the irreversible selection, Sec. 3.2): key j is
// attended by the contiguous query range j <= i <= L_j with L_j = w - 1 + death[j]; its gate
// is 1 while i - j < w and clip(u_j - tau_{i-w}, 0, 1) afterwards.  So a block of QB
// consecutive queries starting at i0 needs
//   (a) the top-k of prefix T0 = i0 - w   (a compact list, built once per score row), and
//   (b) the contiguous keys max(0, i0-w+1) .. i0+QB-1 (window + keys that become selected
//       while the block runs),
// with a per-pair validity/gate test.  That turns the per-query sparse gather into dense
// (queries x keys) tiles.
#include "common.hpp"
#include "attn_tiles.hpp"

namespace spk {


static inline int nblocks(int n) { return (n + QB - 1) / QB; }

// Workspace of the per-block top-k lists: lists [rows][nb][max(k,1)] int32, then counts [rows][nb].
size_t block_lists_bytes(const sparsek_cfg& c, size_t* counts_offset)
{
    size_t rows = (size_t)c.B * c.Gu;
    size_t nb = nblocks(c.n);
    size_t lists = align_up(rows * nb * (size_t)(c.k > 0 ? c.k : 1) * sizeof(int32_t), 256);
    size_t counts = align_up(rows * nb * sizeof(int32_t), 256);
    if (counts_offset) *counts_offset = lists;
    return lists + counts;
}

size_t attn_fwd_ws_bytes(const sparsek_cfg& c) { return block_lists_bytes(c, nullptr); }

// ---------------------------------------------------------------------------------
// Per (row, block): the positions of the top-k of prefix T0 = blk*QB - w, in two partitions:
// first the keys that stay selected for every query of the block (death >= T0 + QB, ascending),
// then, filled from the back, the keys that expire inside the block.  Only the tiles of the
// second partition need a per-pair validity test.  Each wave owns a quarter of [0, T0]: one
// counting pass, one barrier, one placement pass.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void block_lists_kernel(const int32_t* __restrict__ death, int n, int k,
                                                          int w, int nb, int32_t* __restrict__ lists,
                                                          int32_t* __restrict__ counts)
{
    __shared__ int wstay[4], wgo[4];
    const int blk = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int T0 = blk * QB - w;
    int32_t* lo = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    if (T0 < 0 || k == 0) {
        if (tid == 0) counts[(size_t)row * nb + blk] = 0;
        return;
    }
    const int32_t* dr = death + (size_t)row * n;
    const int len = T0 + 1;
    const int per = ((len + 3) / 4 + 255) / 256 * 256;
    const int j_lo = wv * per, j_hi = min(len, j_lo + per);
    const int stay_from = T0 + QB;
    const unsigned long long below = (1ull << lane) - 1ull;
    int ns = 0, ng = 0;
    for (int j0 = j_lo; j0 < j_hi; j0 += 256) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int j = j0 + 64 * e + lane;
            const int dj = j < j_hi ? dr[j] : 0;
            ns += __popcll(__ballot(dj >= stay_from));
            ng += __popcll(__ballot(dj > T0 && dj < stay_from));
        }
    }
    if (lane == 0) { wstay[wv] = ns; wgo[wv] = ng; }
    __syncthreads();
    int os = 0, og = 0;
    for (int i = 0; i < wv; i++) { os += wstay[i]; og += wgo[i]; }
    // min(k, T0 + 1) for a consistent death array; counted, so that every entry below cnt is written
    const int cnt = min(k, wstay[0] + wstay[1] + wstay[2] + wstay[3] + wgo[0] + wgo[1] + wgo[2] + wgo[3]);
    for (int j0 = j_lo; j0 < j_hi; j0 += 256) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int j = j0 + 64 * e + lane;
            const int dj = j < j_hi ? dr[j] : 0;
            const bool stay = dj >= stay_from, go = dj > T0 && dj < stay_from;
            const unsigned long long bs = __ballot(stay), bg = __ballot(go);
            if (stay) {
                const int o = os + __popcll(bs & below);
                if (o < cnt) lo[o] = j;
            }
            if (go) {
                const int o = cnt - 1 - (og + __popcll(bg & below));
                if (o >= 0) lo[o] = j;
            }
            os += __popcll(bs);
            og += __popcll(bg);
        }
    }
    if (tid == 0) counts[(size_t)row * nb + blk] = cnt;
}

// ---------------------------------------------------------------------------------
// Generic vector-ALU kernel (fp32 or bf16 storage, any d <= 128 that is a multiple of 4).
// One wave per query, lanes over keys for the logits and over columns for the output.
// Used for fp32 tensors and head dims the MFMA kernel does not cover.
// ---------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float ld(const T* p);
template <>
__device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ld<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <typename T>
__device__ __forceinline__ void st(T* p, float v);
template <>
__device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void st<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ kk, const T* __restrict__ v,
    const float* __restrict__ u, const float* __restrict__ tau, const int32_t* __restrict__ death,
    const int32_t* __restrict__ lists, const int32_t* __restrict__ counts, T* __restrict__ o,
    float* __restrict__ lse, int H, int Gu, int n, int d, int k, int w, int gate_mode, float scale, int nb)
{
    __shared__ float qs[4][128];
    const int blk = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i0 = blk * QB;
    const T* qh = q + (size_t)bh * n * d;
    const T* kh = kk + (size_t)bh * n * d;
    const T* vh = v + (size_t)bh * n * d;
    T* oh = o + (size_t)bh * n * d;
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int32_t* list = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    const int cnt = counts[(size_t)row * nb + blk];
    const int c0 = max(0, i0 - w + 1);

    for (int qi = wv; qi < QB; qi += 4) {
        const int i = i0 + qi;
        if (i >= n) break;
        for (int c = lane; c < d; c += 64) qs[wv][c] = ld(qh + (size_t)i * d + c);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        const int Tp = i - w;
        const float tauT = (Tp >= 0) ? tr[Tp] : 0.0f;
        float m_run = -INFINITY, l_run = 0.0f, acc0 = 0.0f, acc1 = 0.0f;
        const int n_list = (Tp >= 0) ? cnt : 0;
        const int n_cont = i - c0 + 1;
        const int total = n_list + n_cont;
        for (int e0 = 0; e0 < total; e0 += 64) {
            const int e = e0 + lane;
            int j = -1;
            if (e < total) j = (e < n_list) ? list[e] : c0 + (e - n_list);
            bool valid = false;
            float gate = 1.0f;
            if (j >= 0) {
                if (i - j < w) valid = true;  // window (j <= i by construction)
                else if (dr[j] > Tp) { valid = true; gate = clip01(ur[j] - tauT); }
            }
            float s = -INFINITY;
            if (valid) {
                float dot = 0.0f;
                const T* kj = kh + (size_t)j * d;
                for (int c = 0; c < d; c += 4) {
                    dot += qs[wv][c] * ld(kj + c) + qs[wv][c + 1] * ld(kj + c + 1) +
                           qs[wv][c + 2] * ld(kj + c + 2) + qs[wv][c + 3] * ld(kj + c + 3);
                }
                s = scale * dot * (gate_mode == 0 ? gate : 1.0f);
            }
            const float tmax = wave_max_f32(s);
            if (tmax == -INFINITY) continue;  // no valid key in this tile
            const float m_new = fmaxf(m_run, tmax);
            const float corr = __expf(m_run - m_new);
            const float p = valid ? __expf(s - m_new) : 0.0f;
            l_run = l_run * corr + wave_sum_f32(p);
            acc0 *= corr;
            acc1 *= corr;
            m_run = m_new;
            const float pv = p * (gate_mode == 2 ? 1.0f : gate);
            unsigned long long ball = __ballot(valid);
            while (ball) {
                const int src = __builtin_ctzll(ball);
                ball &= ball - 1;
                const float ps = __shfl(pv, src, 64);
                const int js = __shfl(j, src, 64);
                const T* vj = vh + (size_t)js * d;
                if (lane < d) acc0 += ps * ld(vj + lane);
                if (lane + 64 < d) acc1 += ps * ld(vj + lane + 64);
            }
        }
        const float inv = 1.0f / l_run;
        if (lane < d) st(oh + (size_t)i * d + lane, acc0 * inv);
        if (lane + 64 < d) st(oh + (size_t)i * d + lane + 64, acc1 * inv);
        if (lse && lane == 0) lse[(size_t)bh * n + i] = m_run + __logf(l_run);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    }
}

// ---------------------------------------------------------------------------------
// MFMA kernel (bf16 storage, D = 64 or 128).  One workgroup = 128 queries x 4 waves; each
// wave owns 32 queries and walks the block's key set in tiles of 64 keys:
//   S^T (keys x queries) = K_tile . Q^T     v_mfma_f32_32x32x16_bf16, K rows from LDS
//   online softmax down the key axis: every lane owns one query column, so row maxima and
//   sums stay inside a lane (one exchange with the lane holding the other half of the keys)
//   O^T (d x queries)   += V_tile^T . P^T   the A operand needs the key axis contiguous per
//   lane: V stays row-major in LDS and is read with the transposing LDS load
//   (ds_read_b64_tr_b16); P^T feeds the B operand straight from the accumulator layout.
// K/V rows are gathered from HBM by position straight into LDS (global_load_lds, 16 bytes per
// lane, no register staging), double-buffered, one tile ahead of the compute, one barrier per
// tile.  A wave-load moves 1 KB = RPL whole rows; tile row r goes to group r % NL, slot r / NL,
// and the groups are padded (16 bytes for K, 64 for V) so that the operand reads of 16
// consecutive lanes fall on distinct banks.
// ---------------------------------------------------------------------------------
// Tile kinds, chosen per wave and tile:
//   FAST       contiguous keys inside every query's window and not in its future: no mask, gate 1
//   LIST       selected keys that outlive every query of the wave: gates, no mask
//   LIST_MASK  selected keys, some of which expire inside the wave's query range
//   CONT       contiguous keys at the causal diagonal or at the window's trailing edge
enum { TILE_FAST = 0, TILE_LIST = 1, TILE_LIST_MASK = 2, TILE_CONT = 3 };

template <int D>
__device__ __forceinline__ void rescale_o(f32x16 (&acc_o)[D / 32], float alpha)
{
    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int x = 0; x < D / 32; x++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc_o[x][r] *= alpha;
    }
}

// Everything between the two MFMA phases of one tile, specialised by tile kind: gates and masks
// on the logits, the running maximum with its lazily moved reference point, the exponentials,
// the value gate, and P^T packed to bf16.  Returns the factor the output accumulator has to be
// rescaled by (1 for almost every tile).
template <int MODE, int KIND>
__device__ __forceinline__ float tile_softmax(f32x16 (&acc_s)[2], bf16x8 (&pb)[4], const int32_t* jlast,
                                              const float* ju, int half, int qi, int dqh, int dqw, float tau_q,
                                              float c2, float& m_run, float& l_run)
{
    constexpr bool GATED = (KIND != TILE_FAST) && (MODE != 2);  // the value gate applies
    constexpr bool KGATE = (KIND != TILE_FAST) && (MODE == 0);  // the key gate applies
    constexpr bool MASK = (KIND == TILE_LIST_MASK) || (KIND == TILE_CONT);
    constexpr float LAZY_LOG2 = 8.0f;
    float tmax = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 2; mb++) {
#pragma unroll
        for (int g4 = 0; g4 < 4; g4++) {
            const int kb = 32 * mb + 8 * g4 + 4 * half;  // first of 4 consecutive keys
            int4 L4 = make_int4(0, 0, 0, 0);
            float4 U4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (MASK) L4 = *(const int4*)&jlast[kb];
            if (KGATE) U4 = *(const float4*)&ju[kb];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int r = 4 * g4 + e;
                float s2 = acc_s[mb][r];
                const int Lj = e == 0 ? L4.x : e == 1 ? L4.y : e == 2 ? L4.z : L4.w;
                const float uj = e == 0 ? U4.x : e == 1 ? U4.y : e == 2 ? U4.z : U4.w;
                // key number within the tile minus the lane-dependent 4*half (folded into dqh, dqw so
                // that every compare below has a compile-time constant on one side)
                const int cst = 32 * mb + 8 * g4 + e;
                if (KGATE) {
                    const float g = clip01(uj - tau_q);
                    if (KIND == TILE_CONT) s2 = (cst > dqw) ? s2 : s2 * g;
                    else s2 *= g;
                }
                if (KIND == TILE_LIST_MASK) s2 = (qi <= Lj) ? s2 : -INFINITY;
                if (KIND == TILE_CONT) s2 = (cst <= dqh && qi <= Lj) ? s2 : -INFINITY;
                acc_s[mb][r] = s2;
                tmax = fmaxf(tmax, s2);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // Lazy reference point: m_run only moves when the maximum grows by more than 2^LAZY_LOG2 in
    // probability (softmax is shift-invariant; p stays below 2^LAZY_LOG2, harmless in fp32/bf16).
    // Otherwise some lane of the wave raises its maximum in nearly every tile and the whole
    // output accumulator would be rescaled every time.
    const float m_new = (tmax > m_run + LAZY_LOG2 / c2) ? tmax : m_run;
    const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_safe) * c2);
    const float mc = m_safe * c2;
    m_run = m_new;
    // ---- p = exp2(s*c2 - m*c2): one fma and one v_exp_f32 per logit; value gate; P^T in bf16 ----
    float psum = 0.0f;
#pragma unroll
    for (int mb = 0; mb < 2; mb++) {
#pragma unroll
        for (int g4 = 0; g4 < 4; g4++) {
            const int kb = 32 * mb + 8 * g4 + 4 * half;
            float4 U4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (GATED) U4 = *(const float4*)&ju[kb];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int r = 4 * g4 + e;
                const float p = __builtin_amdgcn_exp2f(fmaf(acc_s[mb][r], c2, -mc));
                psum += p;
                float pvv = p;
                if (GATED) {  // recomputed: one v_sub with clamp, cheaper than holding 32 registers
                    const float uj = e == 0 ? U4.x : e == 1 ? U4.y : e == 2 ? U4.z : U4.w;
                    const float g = clip01(uj - tau_q);
                    if (KIND == TILE_CONT) pvv = (32 * mb + 8 * g4 + e > dqw) ? p : p * g;
                    else pvv = p * g;
                }
                pb[2 * mb + (r >> 3)][r & 7] = (__bf16)pvv;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    l_run = l_run * alpha + psum;
    return alpha;
}

// One 64-key tile for one wave.  The two 32-key halves of S^T are accumulated as two
// interleaved (independent) MFMA chains, the softmax bookkeeping (max exchange, reference
// update, rescale) is done once per tile, and the 16 MFMAs of O^T += V^T.P^T run over four
// independent accumulators.  Only the element-wise gate/mask code depends on the tile kind;
// the two MFMA phases and everything that touches the output accumulator are common code.
template <int D, int MODE>
__device__ __forceinline__ void tile_compute(MfmaSmem<D>& sm, int kind, int buf, int base, int col, int half,
                                             int lane, int qi, int jbase, int w, float tau_q, float c2,
                                             const bf16x8 (&qreg)[D / 16], f32x16 (&acc_o)[D / 32], float& m_run,
                                             float& l_run)
{
    using S = MfmaSmem<D>;
    const unsigned char* kbuf = sm.kb[buf];
    const unsigned char* vbuf = sm.vb[buf];
    const int32_t* jlast = sm.jlast + base;
    const float* ju = sm.ju + base;
    const int dqh = qi - jbase - 4 * half;  // CONT: key number cst + 4*half sits dq - kk behind the query
    const int dqw = dqh - w;                // in the window  <=>  cst > dqw
    // ---- S^T = K . Q^T ----
    f32x16 acc_s[2];
    {
        const unsigned char* kr0 = kbuf + (col % S::NL) * S::GSK + (col / S::NL) * S::RB + 16 * half;
        const unsigned char* kr1 = kbuf + ((32 + col) % S::NL) * S::GSK + ((32 + col) / S::NL) * S::RB + 16 * half;
#pragma unroll
        for (int r = 0; r < 16; r++) { acc_s[0][r] = 0.0f; acc_s[1][r] = 0.0f; }
#pragma unroll
        for (int s = 0; s < D / 16; s++) {
            const bf16x8 a0 = *(const bf16x8*)(kr0 + 32 * s);
            const bf16x8 a1 = *(const bf16x8*)(kr1 + 32 * s);
            acc_s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qreg[s], acc_s[0], 0, 0, 0);
            acc_s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qreg[s], acc_s[1], 0, 0, 0);
            if ((s & 3) == 3) __builtin_amdgcn_sched_barrier(0);  // bound the operand loads in flight
        }
    }
    // ---- gates, masks, softmax: the only kind-specific code ----
    bf16x8 pb[4];
    float alpha;
    if (kind == TILE_FAST)
        alpha = tile_softmax<MODE, TILE_FAST>(acc_s, pb, jlast, ju, half, qi, dqh, dqw, tau_q, c2, m_run, l_run);
    else if (kind == TILE_LIST)
        alpha = tile_softmax<MODE, TILE_LIST>(acc_s, pb, jlast, ju, half, qi, dqh, dqw, tau_q, c2, m_run, l_run);
    else if (kind == TILE_LIST_MASK)
        alpha = tile_softmax<MODE, TILE_LIST_MASK>(acc_s, pb, jlast, ju, half, qi, dqh, dqw, tau_q, c2, m_run, l_run);
    else
        alpha = tile_softmax<MODE, TILE_CONT>(acc_s, pb, jlast, ju, half, qi, dqh, dqw, tau_q, c2, m_run, l_run);
    __builtin_amdgcn_sched_barrier(0);
    rescale_o<D>(acc_o, alpha);
    // ---- O^T += V^T . P^T ----
    // The A operand comes through transposing LDS loads: within each group of 16 lanes, lane r
    // points at (row r/4, 4-column block r%4) of a 4-row x 16-column patch of V and receives the
    // 4 rows of column r.  MFMA g (16 keys) uses rows 16g + 4*half + {0..3} (k-slots 0..3) and
    // 16g + 8 + 4*half + {0..3} (k-slots 4..7): the key order P^T already has.
    const int r16 = lane & 15, grp2 = (lane >> 4) & 1;
#pragma unroll
    for (int g = 0; g < 4; g++) {
        const int row0 = 16 * g + 4 * half + (r16 >> 2);
        const int row1 = row0 + 8;
        const unsigned char* v0 = vbuf + (row0 % S::NL) * S::GSV + (row0 / S::NL) * S::RB + (16 * grp2 + 4 * (r16 & 3)) * 2;
        const unsigned char* v1 = vbuf + (row1 % S::NL) * S::GSV + (row1 / S::NL) * S::RB + (16 * grp2 + 4 * (r16 & 3)) * 2;
#pragma unroll
        for (int x = 0; x < D / 32; x++) {
            const i16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)(v0 + 64 * x));
            const i16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)(v1 + 64 * x));
            const bf16x4 lo = __builtin_bit_cast(bf16x4, lo4), hi = __builtin_bit_cast(bf16x4, hi4);
            const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            acc_o[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[g], acc_o[x], 0, 0, 0);
        }
        if (g & 1) __builtin_amdgcn_sched_barrier(0);
    }
}

template <int D, int MODE>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ kk, const uint16_t* __restrict__ v,
    const float* __restrict__ u, const float* __restrict__ tau, const int32_t* __restrict__ death,
    const int32_t* __restrict__ lists, const int32_t* __restrict__ counts, uint16_t* __restrict__ o,
    float* __restrict__ lse, int H, int Gu, int n, int k, int w, float scale, int nb, int BH)
{
    __shared__ __align__(16) MfmaSmem<D> sm;
    constexpr int DS = D / 16;   // MFMA k-steps over the head dim
    constexpr int DB = D / 32;   // 32-row blocks of O^T

    // ---- block -> (head, query block): heads are dealt to the 8 XCDs so that one head's
    // blocks share an L2; late (long) blocks go first
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
    const uint16_t* qh = q + (size_t)bh * n * D;
    const uint16_t* kh = kk + (size_t)bh * n * D;
    const uint16_t* vh = v + (size_t)bh * n * D;
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int32_t* list = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    const int cnt = counts[(size_t)row * nb + blk];
    const int c0 = max(0, i0 - w + 1);
    const int c_end = min(n - 1, i0 + QB - 1);
    const int nkl = (cnt + KT - 1) / KT * KT;                // list part, padded to whole tiles
    const int nkc = (c_end - c0 + 1 + KT - 1) / KT * KT;     // contiguous part, padded
    const int nk_total = nkl + nkc;

    // ---- this wave's queries ----
    const int qa = i0 + 32 * wv;          // first query of the wave
    const int qb = min(qa + 31, n - 1);   // last real query of the wave
    const int qi = qa + col;              // this lane's query
    const bool wave_live = qa < n;
    const int qrow = min(qi, n - 1);
    const float tau_q = (qi < n && qi - w >= 0) ? tr[qi - w] : 0.0f;
    bf16x8 qreg[DS];
#pragma unroll
    for (int s = 0; s < DS; s++)
        qreg[s] = *(const bf16x8*)(qh + (size_t)qrow * D + 16 * s + 8 * half);

    f32x16 acc_o[DB];
#pragma unroll
    for (int x = 0; x < DB; x++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc_o[x][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float c2 = scale * 1.4426950408889634f;

    for (int seg0 = 0; seg0 < nk_total; seg0 += SEG) {
        const int seg_n = min(SEG, nk_total - seg0);
        __syncthreads();  // previous segment fully consumed (metadata and both tile buffers)
        for (int e = tid; e < seg_n; e += 256) {
            const int E = seg0 + e;
            int j = 0;
            bool real;
            if (E < nkl) {
                real = E < cnt;
                if (real) j = list[E];
            } else {
                j = c0 + (E - nkl);
                real = j <= c_end;
                if (!real) j = 0;
            }
            sm.jpos[e] = j;
            sm.jlast[e] = real ? (w - 1 + dr[j]) : -1;
            sm.ju[e] = real ? ur[j] : 0.0f;
        }
        __syncthreads();
        for (int t = wv; t < seg_n / KT; t += 4) {
            int lm = sm.jlast[t * KT + lane];
#pragma unroll
            for (int o2 = 32; o2 > 0; o2 >>= 1) lm = min(lm, __shfl_xor(lm, o2, 64));
            if (lane == 0) sm.tile_lmin[t] = lm;
        }
        const int ntiles = seg_n / KT;
        issue_tile_loads<D, 64>(sm, 0, sm.jpos, kh, vh, wv, lane);
        for (int t = 0; t < ntiles; t++) {
            // tile t has landed (this wave's part: vmcnt; the other waves' parts: barrier); the
            // barrier also says that everybody is done with tile t-1, whose buffer is refilled next
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (t + 1 < ntiles) issue_tile_loads<D, 64>(sm, (t + 1) & 1, sm.jpos + (t + 1) * KT, kh, vh, wv, lane);

            // ---- classify the tile for this wave (all conditions are wave-uniform) ----
            const int base = t * KT;
            const int E0 = seg0 + base;
            const bool is_list = E0 < nkl;
            const int jbase = is_list ? 0 : c0 + (E0 - nkl);  // first position of a contiguous tile
            int kind = -1;  // -1: nothing of this tile is visible to the wave
            if (wave_live) {
                if (is_list) {
                    kind = (sm.tile_lmin[t] >= qb) ? TILE_LIST : TILE_LIST_MASK;
                } else if (jbase <= qb) {  // else every key is in the future of every query of the wave
                    const int jend = jbase + KT - 1;
                    kind = (jend <= qa && qb - jbase < w && jend <= c_end) ? TILE_FAST : TILE_CONT;
                }
            }
            if (kind >= 0)
                tile_compute<D, MODE>(sm, kind, t & 1, base, col, half, lane, qi, jbase, w, tau_q, c2, qreg, acc_o,
                                      m_run, l_run);
        }
    }

    // ---- epilogue: O = O^T / l, lse ----
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (qi < n) {
        const float inv = 1.0f / l_tot;
        uint16_t* orow = o + ((size_t)bh * n + qi) * D;
#pragma unroll
        for (int x = 0; x < DB; x++) {
#pragma unroll
            for (int g4 = 0; g4 < 4; g4++) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; e++) pk[e] = (__bf16)(acc_o[x][4 * g4 + e] * inv);
                *(bf16x4*)(orow + 32 * x + 8 * g4 + 4 * half) = pk;
            }
        }
        if (lse && half == 0) lse[(size_t)bh * n + qi] = (m_run * c2 + log2f(l_tot)) * 0.6931471805599453f;
    }
}

template <int D>
static void launch_mfma(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                        const float* tau, const int32_t* death, const int32_t* lists, const int32_t* counts,
                        void* o, float* lse, int nb, hipStream_t st)
{
    const int BH = c.B * c.H;
    dim3 grid(nb * BH);
#define SPK_LAUNCH(MODE)                                                                                   \
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, MODE>), grid, dim3(256), 0, st, (const uint16_t*)q,        \
                       (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, (uint16_t*)o, \
                       lse, c.H, c.Gu, c.n, c.k, c.w, c.softmax_scale, nb, BH)
    if (c.gate_mode == 0) SPK_LAUNCH(0);
    else if (c.gate_mode == 1) SPK_LAUNCH(1);
    else SPK_LAUNCH(2);
#undef SPK_LAUNCH
}

void launch_block_lists(const sparsek_cfg& c, const int32_t* death, int32_t* lists, int32_t* counts,
                        hipStream_t st)
{
    const int nb = nblocks(c.n);
    hipLaunchKernelGGL(block_lists_kernel, dim3(nb, c.B * c.Gu), dim3(256), 0, st, death, c.n, c.k, c.w, nb,
                       lists, counts);
}

int launch_attn_fwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, void* o, float* lse, void* ws,
                    hipStream_t st)
{
    const int nb = nblocks(c.n);
    size_t coff = 0;
    block_lists_bytes(c, &coff);
    int32_t* lists = (int32_t*)ws;
    int32_t* counts = (int32_t*)((char*)ws + coff);
    launch_block_lists(c, death, lists, counts, st);
    if (c.dtype == SPARSEK_BF16 && (c.d == 64 || c.d == 128) && (uint64_t)c.n * c.d * 2 <= 0xFFFFFFFFull) {
        if (c.d == 64) launch_mfma<64>(c, q, k, v, u, tau, death, lists, counts, o, lse, nb, st);
        else launch_mfma<128>(c, q, k, v, u, tau, death, lists, counts, o, lse, nb, st);
        return launch_status();
    }
    dim3 grid(nb, c.B * c.H);
    if (c.dtype == SPARSEK_F32) {
        hipLaunchKernelGGL(attn_fwd_generic_kernel<float>, grid, dim3(256), 0, st, (const float*)q,
                           (const float*)k, (const float*)v, u, tau, death, lists, counts, (float*)o, lse, c.H,
                           c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale, nb);
    } else {
        hipLaunchKernelGGL(attn_fwd_generic_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)q,
                           (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, (uint16_t*)o,
                           lse, c.H, c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale, nb);
    }
    return launch_status();
}

}  // namespace spk

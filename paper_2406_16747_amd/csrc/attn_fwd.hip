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
#include <type_traits>

namespace spk {


// Workspace of the per-block top-k lists: lists [rows][nb][max(k,1)] int32, then counts [rows][nb]
// (list lengths) and stays [rows][nb] (lengths of the first partitions).
size_t block_lists_bytes(const sparsek_cfg& c, size_t* counts_offset)
{
    size_t rows = (size_t)c.B * c.Gu;
    size_t nb = nblocks(c.n);
    size_t lists = align_up(rows * nb * (size_t)(c.k > 0 ? c.k : 1) * sizeof(int32_t), 256);
    size_t counts = align_up(2 * rows * nb * sizeof(int32_t), 256);
    if (counts_offset) *counts_offset = lists;
    return lists + counts;
}

size_t attn_fwd_ws_bytes(const sparsek_cfg& c) { return block_lists_bytes(c, nullptr) + 3 * ext_array_bytes(c); }

// ---------------------------------------------------------------------------------
// Per (row, block): the positions of the top-k of prefix T0 = blk*QB - w, in two partitions:
// first the keys that stay selected for every query of the block (death >= T0 + QB, ascending),
// then, filled from the back, the keys that expire inside the block.  Only the tiles of the
// second partition need a per-pair validity test.  Each of the 16 waves owns a slice of
// [0, T0]: one counting pass, one barrier, one placement pass.
// With xpos != nullptr the same lists are also written in the extended form described above.
// ---------------------------------------------------------------------------------
constexpr int BL_WAVES = 16;   // waves per workgroup of block_lists_kernel
constexpr int BL_UNROLL = 8;   // loads in flight per lane

__global__ __launch_bounds__(64 * BL_WAVES) void block_lists_kernel(const int32_t* __restrict__ death, int n, int k,
                                                                     int w, int nb, int32_t* __restrict__ lists,
                                                                     int32_t* __restrict__ counts,
                                                                     const float* __restrict__ u,
                                                                     int32_t* __restrict__ xpos,
                                                                     int32_t* __restrict__ xdeath,
                                                                     float* __restrict__ xu, int KP)
{
    __shared__ int wstay[BL_WAVES], wgo[BL_WAVES];
    const int blk = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int T0 = blk * QB - w;
    int32_t* lo = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    if (T0 < 0 || k == 0) {
        if (tid == 0) {
            counts[(size_t)row * nb + blk] = 0;
            counts[((size_t)gridDim.y + row) * nb + blk] = 0;
        }
        return;
    }
    const int32_t* dr = death + (size_t)row * n;
    const float* ur = u ? u + (size_t)row * n : nullptr;
    const size_t xo = ((size_t)row * nb + blk) * (size_t)KP;
    const int len = T0 + 1;
    constexpr int STEP = 64 * BL_UNROLL;
    const int per = ((len + BL_WAVES - 1) / BL_WAVES + STEP - 1) / STEP * STEP;
    const int j_lo = wv * per, j_hi = min(len, j_lo + per);
    const int stay_from = T0 + QB;
    const unsigned long long below = (1ull << lane) - 1ull;
    int ns = 0, ng = 0;
    for (int j0 = j_lo; j0 < j_hi; j0 += STEP) {
        int dj[BL_UNROLL];
#pragma unroll
        for (int e = 0; e < BL_UNROLL; e++) {
            const int j = j0 + 64 * e + lane;
            dj[e] = j < j_hi ? dr[j] : 0;
        }
#pragma unroll
        for (int e = 0; e < BL_UNROLL; e++) {
            ns += __popcll(__ballot(dj[e] >= stay_from));
            ng += __popcll(__ballot(dj[e] > T0 && dj[e] < stay_from));
        }
    }
    if (lane == 0) { wstay[wv] = ns; wgo[wv] = ng; }
    __syncthreads();
    int os = 0, og = 0, tot_s = 0, tot_g = 0;
    for (int i = 0; i < BL_WAVES; i++) {
        if (i < wv) { os += wstay[i]; og += wgo[i]; }
        tot_s += wstay[i];
        tot_g += wgo[i];
    }
    // min(k, T0 + 1) for a consistent death array; counted, so that every entry below cnt is written
    const int cnt = min(k, tot_s + tot_g);
    for (int j0 = j_lo; j0 < j_hi; j0 += STEP) {
        int dj[BL_UNROLL];
#pragma unroll
        for (int e = 0; e < BL_UNROLL; e++) {
            const int j = j0 + 64 * e + lane;
            dj[e] = j < j_hi ? dr[j] : 0;
        }
#pragma unroll
        for (int e = 0; e < BL_UNROLL; e++) {
            const int j = j0 + 64 * e + lane;
            const bool stay = dj[e] >= stay_from, go = dj[e] > T0 && dj[e] < stay_from;
            const unsigned long long bs = __ballot(stay), bg = __ballot(go);
            int o = -1;
            if (stay) {
                o = os + __popcll(bs & below);
                if (o >= cnt) o = -1;
            }
            if (go) o = cnt - 1 - (og + __popcll(bg & below));
            if (o >= 0) {
                lo[o] = j;
                if (xpos) {
                    xpos[xo + o] = j;
                    xdeath[xo + o] = dj[e];
                    xu[xo + o] = ur[j];
                }
            }
            os += __popcll(bs);
            og += __popcll(bg);
        }
    }
    if (tid == 0) {
        counts[(size_t)row * nb + blk] = cnt;
        counts[((size_t)gridDim.y + row) * nb + blk] = min(cnt, tot_s);
    }
    if (xpos) {
        // padding up to the tile boundary above min(k, T0 + 1), the length the forward kernel lays its tiles out for
        const int padded = (min(k, len) + KT - 1) / KT * KT;
        for (int o = cnt + tid; o < padded; o += 64 * BL_WAVES) {
            xpos[xo + o] = 0;
            xdeath[xo + o] = INT32_MIN;
            xu[xo + o] = 0.0f;
        }
    }
}

// ---------------------------------------------------------------------------------
// Generic vector-ALU kernel (fp32 or bf16 storage, any d <= 128 that is a multiple of 4).
// One wave per query, lanes over keys for the logits and over columns for the output.
// Used for fp32 tensors and head dims the MFMA kernel does not cover.  A query block of QB
// queries (the granularity of the lists) is spread over GEN_SPLIT workgroups of four waves, one
// query per wave, so that small problems still fill the chip.
// ---------------------------------------------------------------------------------
constexpr int GEN_SPLIT = QB / 4;
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
    float* __restrict__ lse, int H, int Gu, int n, int d, int k, int w, int gate_mode, float scale, int nb,
    int q_begin, const int32_t* __restrict__ first_valid, int q_rows)
{
    __shared__ float qs[4][128];
    const int blk = blockIdx.x / GEN_SPLIT, sub = blockIdx.x % GEN_SPLIT, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i0 = blk * QB;
    if (i0 + QB <= q_begin) return;  // queries before q_begin are not wanted (chunked prefill)
    // q and o hold q_rows rows per head starting at query q_begin (0: all n rows)
    const ptrdiff_t qo = q_rows ? (ptrdiff_t)bh * q_rows - q_begin : (ptrdiff_t)bh * n;
    const T* qh = q + qo * d;
    const T* kh = kk + (size_t)bh * n * d;
    const T* vh = v + (size_t)bh * n * d;
    T* oh = o + qo * d;
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int32_t* list = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    const int cnt = counts[(size_t)row * nb + blk];
    // keys before first_valid[row] (padding of a chunked prefill) are attended by nobody
    const int c0 = max(max(0, i0 - w + 1), first_valid ? first_valid[row] : 0);

    {
        const int i = i0 + 4 * sub + wv;
        if (i >= n || i < q_begin) return;
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
        if (lse && lane == 0) lse[qo + i] = m_run + __logf(l_run);
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
//
// The kernel is bound by vector-ALU issue (gates, masks, exponentials), not by the matrix
// cores, so inside a tile the two are interleaved by hand: the tile is split into two halves
// of 32 keys, and the instruction stream is
//   S_A | S_B + softmax(A) | O += V_A^T.P_A + softmax(B) | O += V_B^T.P_B
// with one MFMA followed by a slice of the softmax work, the slices fenced with sched_barrier
// so that the compiler keeps the order.
// ---------------------------------------------------------------------------------
// The forward's LDS: the double-buffered K and V tiles and the staged metadata.
template <int D>
struct FwdSmem : MfmaTileBufs<D, 64>, TileMeta {};
static_assert(sizeof(FwdSmem<128>) <= 80 * 1024, "two workgroups per CU");

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

// The reference point of the online softmax of one query: m (logit units, -inf before the
// first visible key) and mc = m * scale * log2(e) (0 while m is -inf), what the exponent subtracts.
struct SoftRef {
    float m, mc;
};

// Softmax state of one 32-key half of a tile: this lane holds 16 of its logits (4 groups of 4
// consecutive keys), their gates and lifetimes.
struct HalfState {
    float4 G[4];   // scores, overwritten by the gates
    float tmax, mc, alpha, psum;
    bf16x8 pb[2];  // P^T in operand layout
};

template <int MODE, int KIND>
__device__ __forceinline__ void load_meta(HalfState& h, const float* ju, int hf, int half)
{
    using TT = TileTraits<MODE, KIND>;
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
        const int kb = 32 * hf + 8 * g4 + 4 * half;
        if (TT::GATED) h.G[g4] = *(const float4*)&ju[kb];
    }
    h.tmax = -INFINITY;
    h.psum = 0.0f;
}

// Slice U of the softmax work of one half.  U = 0..3: gates and masks of key group U and the
// running maximum; after group 3 the maximum is exchanged with the partner lane and the
// reference point moves if it has to (lazily: only when the maximum grew by more than 2^8 in
// probability; softmax is shift-invariant and p stays below 2^8, harmless in fp32/bf16; this
// keeps the rescale of the output accumulator a rare event).  U = 4..7: exponentials, row sum,
// value gate and bf16 packing of key group U - 4.
template <int MODE, int KIND, int U>
__device__ __forceinline__ void softmax_slice(HalfState& h, f32x16& sv, const int32_t* jdeath, int half, int hf,
                                              int qw, int dqh, int dqw, float tau_q, float c2, SoftRef& ref)
{
    using TT = TileTraits<MODE, KIND>;
    constexpr float LAZY_LOG2 = 8.0f;
    if (U < 4) {
        constexpr int g4 = U & 3;
        float gg[4] = {h.G[g4].x, h.G[g4].y, h.G[g4].z, h.G[g4].w};
        // lifetimes are read where they are used (only the few masked tile kinds need them):
        // holding them across the tile costs more registers than the kernel has
        int4 L4 = make_int4(0, 0, 0, 0);
        if (TT::MASKL) L4 = *(const int4*)&jdeath[32 * hf + 8 * g4 + 4 * half];
        const int ll[4] = {L4.x, L4.y, L4.z, L4.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int r = 4 * g4 + e;
            // key number within the tile minus the lane-dependent 4*half (folded into dqh, dqw so
            // that every compare below has a compile-time constant on one side)
            const int cst = 32 * hf + 8 * g4 + e;
            float s2 = sv[r];
            if (TT::GATED) {
                float g = clip01(gg[e] - tau_q);
                if (TT::SELECT) g = (cst > dqw) ? 1.0f : g;
                gg[e] = g;
                if (TT::KGATE) s2 *= g;
            }
            // key j is attended by query i while i <= w - 1 + death[j], i.e. qw = i - (w - 1) <= death[j]
            if (TT::MASKL && TT::MASKC) s2 = (cst <= dqh && qw <= ll[e]) ? s2 : -INFINITY;
            else if (TT::MASKL) s2 = (qw <= ll[e]) ? s2 : -INFINITY;
            else if (TT::MASKC) s2 = (cst <= dqh) ? s2 : -INFINITY;
            sv[r] = s2;
            h.tmax = fmaxf(h.tmax, s2);
        }
        if (TT::GATED) h.G[g4] = make_float4(gg[0], gg[1], gg[2], gg[3]);
        if (U == 3) {
            // Almost always no lane of the wave has to move its reference point: one compare and
            // a wave-uniform branch; the exchange with the partner lane, the new reference and
            // the rescale factor are computed only in the rare other case.
            const float limit = ref.m + LAZY_LOG2 / c2;
            h.alpha = 1.0f;
            if (__any(h.tmax > limit)) {
                const unsigned tb = __float_as_uint(h.tmax);
                const auto sw = __builtin_amdgcn_permlane32_swap(tb, tb, false, false);  // both halves, no LDS
                const float tq = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                const float m_new = (tq > limit) ? tq : ref.m;
                const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
                h.alpha = __builtin_amdgcn_exp2f((ref.m - m_safe) * c2);
                ref.mc = m_safe * c2;
                ref.m = m_new;
            }
            h.mc = ref.mc;
        }
    } else {
        constexpr int g4 = U & 3;
        const float gg[4] = {h.G[g4].x, h.G[g4].y, h.G[g4].z, h.G[g4].w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int r = 4 * g4 + e;
            const float p = __builtin_amdgcn_exp2f(fmaf(sv[r], c2, -h.mc));
            h.psum += p;
            const float pv = TT::GATED ? p * gg[e] : p;
            h.pb[r >> 3][r & 7] = (__bf16)pv;
        }
    }
}

template <int MODE, int KIND, int U0, int U1>
__device__ __forceinline__ void softmax_slices(HalfState& h, f32x16& sv, const int32_t* jdeath, int half, int hf,
                                               int qw, int dqh, int dqw, float tau_q, float c2, SoftRef& ref)
{
    if constexpr (U0 < U1) {
        softmax_slice<MODE, KIND, U0>(h, sv, jdeath, half, hf, qw, dqh, dqw, tau_q, c2, ref);
        softmax_slices<MODE, KIND, U0 + 1, U1>(h, sv, jdeath, half, hf, qw, dqh, dqw, tau_q, c2, ref);
    }
}

// One 64-key tile for one wave (see the schedule in the header comment).  The tile is a
// sequence of MFMA slots (S_A, S_B, PV_A, PV_B); the LDS operand of slot n is requested DEPTH
// slots earlier into a small register ring, so that no MFMA waits for a read it has just issued.
template <int D, int MODE, int KIND>
__device__ __forceinline__ void tile_body(FwdSmem<D>& sm, int buf, const int32_t* jdeath, const float* ju,
                                          const int32_t* jp_next, int jbase, bool more,
                                          const uint16_t* kh, const uint16_t* vh, int wv, int col, int half,
                                          int lane, int qi, int w, float tau_q, float c2,
                                          const bf16x8 (&qreg)[D / 16], f32x16 (&acc_o)[D / 32], SoftRef& ref,
                                          float& l_run)
{
    using S = FwdSmem<D>;
    constexpr int NS = D / 16;      // MFMAs per half of S^T
    constexpr int DB = D / 32;      // 32-row blocks of O^T
    constexpr int NP = 2 * DB;      // MFMAs per half of O^T += V^T.P^T
    constexpr int US = 8 / NS;      // softmax slices per MFMA of S_B
    constexpr int UP = 8 / NP;      // softmax slices per MFMA of the first PV half
    constexpr int NSLOT = 2 * NS + 2 * NP;
    constexpr int DEPTH = 2;
    constexpr int NX = S::NL / 4;   // gather steps of the next tile, one per S_A slot
    static_assert(NX <= NS, "one gather step per S_A slot");
    const unsigned char* kbuf = sm.kb[buf];
    const unsigned char* vbuf = sm.vb[buf];
    const int qw = qi - (w - 1);
    const int dqh = qi - jbase - 4 * half;  // contiguous tiles: key number cst + 4*half sits dqh - cst behind the query
    const int dqw = dqh - w;                // in the window  <=>  cst > dqw
    const unsigned char* krA = kbuf + (col % S::NL) * S::GSK + (col / S::NL) * S::RB + 16 * half;
    const unsigned char* krB = kbuf + ((32 + col) % S::NL) * S::GSK + ((32 + col) / S::NL) * S::RB + 16 * half;
    // The A operand of O^T += V^T.P^T comes through transposing LDS loads: within each group of
    // 16 lanes, lane r points at (row r/4, 4-column block r%4) of a 4-row x 16-column patch of V
    // and receives the 4 rows of column r.  MFMA g (16 keys) uses rows 16g + 4*half + {0..3}
    // (k-slots 0..3) and 16g + 8 + 4*half + {0..3} (k-slots 4..7): the key order P^T already has.
    const int r16 = lane & 15, grp2 = (lane >> 4) & 1;
    const int vcol = (16 * grp2 + 4 * (r16 & 3)) * 2;
    const int vrow = 4 * half + (r16 >> 2);
    auto v_operand = [&](int g, int x) -> bf16x8 {
        const int row0 = 16 * g + vrow;
        const int row1 = row0 + 8;
        const unsigned char* v0 = vbuf + (row0 % S::NL) * S::GSV + (row0 / S::NL) * S::RB + vcol + 64 * x;
        const unsigned char* v1 = vbuf + (row1 % S::NL) * S::GSV + (row1 / S::NL) * S::RB + vcol + 64 * x;
        const i16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)v0);
        const i16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)v1);
        const bf16x4 lo = __builtin_bit_cast(bf16x4, lo4), hi = __builtin_bit_cast(bf16x4, hi4);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto operand = [&](int n) -> bf16x8 {  // n is a compile-time constant after unrolling
        if (n < NS) return *(const bf16x8*)(krA + 32 * n);
        if (n < 2 * NS) return *(const bf16x8*)(krB + 32 * (n - NS));
        const int i = n - 2 * NS;
        return v_operand(i / DB, i % DB);
    };

    HalfState A, B;
    f32x16 sA, sB;
#pragma unroll
    for (int r = 0; r < 16; r++) { sA[r] = 0.0f; sB[r] = 0.0f; }
    bf16x8 ring[DEPTH];
#pragma unroll
    for (int n = 0; n < DEPTH; n++) ring[n] = operand(n);
    TileRows<D, 64> rows;
    if (more) rows = tile_rows<D, 64>(jp_next, wv, lane);
    load_meta<MODE, KIND>(A, ju, 0, half);
    __builtin_amdgcn_sched_barrier(0);
    // ---- S_A, then S_B with softmax(A) ----
    static_for<0, 2 * NS>([&](auto nc) {
        constexpr int n = decltype(nc)::value;
        const bf16x8 cur = ring[n % DEPTH];
        if constexpr (n < NS) sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qreg[n], sA, 0, 0, 0);
        else sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qreg[n - NS], sB, 0, 0, 0);
        if (n + DEPTH < NSLOT) ring[n % DEPTH] = operand(n + DEPTH);
        // the gather of the next tile rides on the S_A slots, whose issue is otherwise idle
        // (every wave is past this tile's barrier, so the other buffer is free)
        if (n < NX && more) tile_load_step<D, 64>(sm, buf ^ 1, rows, n, kh, vh, wv, lane);
        if (n >= NS) {
            constexpr int s = n >= NS ? n - NS : 0;
            softmax_slices<MODE, KIND, US * s, US * (s + 1)>(A, sA, jdeath, half, 0, qw, dqh, dqw, tau_q, c2, ref);
            if (US * (s + 1) == 4) load_meta<MODE, KIND>(B, ju, 1, half);
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    // (the empty asm uses keep the compiler from sinking the exponentials below the rescale branch)
    asm volatile("" ::"v"(A.pb[0]), "v"(A.pb[1]), "v"(A.psum));
    l_run = l_run * A.alpha + A.psum;
    rescale_o<D>(acc_o, A.alpha);
    // ---- O^T += V_A^T . P_A^T with softmax(B) ----
    static_for<0, NP>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int n = 2 * NS + i;
        const bf16x8 cur = ring[n % DEPTH];
        acc_o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, A.pb[i / DB], acc_o[i % DB], 0, 0, 0);
        if (n + DEPTH < NSLOT) ring[n % DEPTH] = operand(n + DEPTH);
        softmax_slices<MODE, KIND, UP * i, UP * (i + 1)>(B, sB, jdeath, half, 1, qw, dqh, dqw, tau_q, c2, ref);
        __builtin_amdgcn_sched_barrier(0);
    });
    asm volatile("" ::"v"(B.pb[0]), "v"(B.pb[1]), "v"(B.psum));
    l_run = l_run * B.alpha + B.psum;
    rescale_o<D>(acc_o, B.alpha);
    // ---- O^T += V_B^T . P_B^T ----
    static_for<0, NP>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int n = 2 * NS + NP + i;
        const bf16x8 cur = ring[n % DEPTH];
        acc_o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, B.pb[i / DB], acc_o[i % DB], 0, 0, 0);
        if (n + DEPTH < NSLOT) ring[n % DEPTH] = operand(n + DEPTH);
    });
}

// The tiles [T, T_end) of the block's key set, all of one kind.  T counts the block's tiles; tile T uses K/V buffer
// T & 1 and the metadata of segment T / TPS.
template <int D, int MODE, int KIND>
__device__ __forceinline__ void run_tiles(FwdSmem<D>& sm, const StageSrc& src, int& T, int T_end, int jbase0,
                                          const uint16_t* kh, const uint16_t* vh, int wv, int col, int half,
                                          int lane, int qi, int w, float tau_q, float c2,
                                          const bf16x8 (&qreg)[D / 16], f32x16 (&acc_o)[D / 32], SoftRef& ref,
                                          float& l_run)
{
    for (; T < T_end; T++) {
        // tile T has landed (this wave's part: vmcnt; the other waves' parts: barrier); the
        // barrier also says that everybody is done with tile T-1, whose buffer is refilled next
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const int sg = T / TPS, lt = T - sg * TPS;
        // first tile of a segment: everybody has left the segment before, so its metadata buffer takes the next one
        if (lt == 0 && (sg + 1) * TPS < src.nt) stage_meta(sm, src, sg + 1, wv, lane);
        const int sgn = (T + 1) / TPS;
        const int32_t* jp_next = sm.jpos[sgn & 1] + (T + 1 - sgn * TPS) * KT;
        const bool more = T + 1 < src.nt;
        if (KIND != TILE_SKIP)
            tile_body<D, MODE, KIND>(sm, T & 1, sm.jdeath[sg & 1] + lt * KT, sm.ju[sg & 1] + lt * KT, jp_next,
                                     jbase0 + T * KT, more, kh, vh, wv, col, half, lane, qi, w, tau_q, c2, qreg,
                                     acc_o, ref, l_run);
        else if (more)
            issue_tile_loads<D, 64>(sm, (T + 1) & 1, jp_next, kh, vh, wv, lane);
    }
}

template <int D, int MODE>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ kk, const uint16_t* __restrict__ v,
    const float* __restrict__ u, const float* __restrict__ tau, const int32_t* __restrict__ death,
    const int32_t* __restrict__ xpos, const int32_t* __restrict__ xdeath, const float* __restrict__ xu, int KP,
    const int32_t* __restrict__ counts, uint16_t* __restrict__ o,
    float* __restrict__ lse, int H, int Gu, int n, int k, int w, float scale, int nb, int BH, int nrows,
    int q_begin, const int32_t* __restrict__ first_valid, int q_rows)
{
    __shared__ __align__(16) FwdSmem<D> sm;
    constexpr int DS = D / 16;   // MFMA k-steps over the head dim
    constexpr int DB = D / 32;   // 32-row blocks of O^T
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;

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
    const int i0 = blk * QB;
    if (i0 + QB <= q_begin) return;  // queries before q_begin are not wanted (chunked prefill)
    // q and o hold q_rows rows per head starting at query q_begin (0: all n rows)
    const ptrdiff_t qo = q_rows ? (ptrdiff_t)bh * q_rows - q_begin : (ptrdiff_t)bh * n;
    const uint16_t* qh = q + qo * D;
    const uint16_t* kh = kk + (size_t)bh * n * D;
    const uint16_t* vh = v + (size_t)bh * n * D;
    const float* tr = tau + (size_t)row * n;
    const int nstay = counts[(size_t)nrows * nb + (size_t)row * nb + blk];
    // keys before first_valid[row] (padding of a chunked prefill) are attended by nobody
    const int c0 = max(max(0, i0 - w + 1), first_valid ? first_valid[row] : 0);
    const int c_end = min(n - 1, i0 + QB - 1);
    // The list part is laid out for min(k, T0 + 1) keys, the length of a complete top-k list (known without a load);
    // a shorter list (lifetimes cleared by a chunked prefill) ends in padding that nobody attends.
    const int T0 = i0 - w;
    const int nkl = (T0 >= 0 && k > 0) ? (min(k, T0 + 1) + KT - 1) / KT * KT : 0;   // list part, whole tiles
    const int nkc = max(0, (c_end - c0 + 1 + KT - 1) / KT * KT);                    // contiguous part, padded
    const int NT = (nkl + nkc) / KT;

    StageSrc src;
    {
        const size_t xo = ((size_t)row * nb + blk) * (size_t)KP;
        src.xpos = xpos + xo;
        src.xdeath = xdeath + xo;
        src.xu = xu + xo;
        src.dr = death + (size_t)row * n;
        src.ur = u + (size_t)row * n;
        src.nkl = nkl;
        src.c0 = c0;
        src.c_end = c_end;
        src.nt = NT;
    }

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
    // the first segment of metadata: its copies need nothing that is loaded above, so they fly together
    stage_meta(sm, src, 0, wv, lane);

    // ---- the runs of tile kinds for this wave, as tile numbers (all wave-uniform) ----
    const WaveRuns wr = wave_runs(wave_live, nkl, nkc, nstay, qa, qb, w, c0);
    const int b0 = wr.b0, b1 = wr.b1, b2 = wr.b2, b3 = wr.b3, b4 = wr.b4;
    const bool narrow = wr.narrow;

    f32x16 acc_o[DB];
#pragma unroll
    for (int x = 0; x < DB; x++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc_o[x][r] = 0.0f;
    SoftRef ref{-INFINITY, 0.0f};
    float l_run = 0.0f;
    const float c2 = scale * 1.4426950408889634f;

    // The metadata copies and the tile gathers are direct-to-LDS loads that the compiler does not track.  Everything
    // it does track (the Q fragments, tau, the counts) is waited for here, ahead of the first gather: left to their
    // first use inside the tile loop, those waits would count the prefetched tile too and drain it early.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int s = 0; s < DS; s++) asm volatile("" ::"v"(qreg[s]));
    __syncthreads();  // segment 0 of the metadata is in place
    if (NT > 0) issue_tile_loads<D, 64>(sm, 0, sm.jpos[0], kh, vh, wv, lane);
    {
        const int jbase0 = c0 - nkl;     // position of tile 0's first key if the whole key set were contiguous
        int T = 0;
#define SPK_RUN(KIND, bound)                                                                                     \
    run_tiles<D, MODE, KIND>(sm, src, T, min(NT, (bound)), jbase0, kh, vh, wv, col, half, lane, qi, w, tau_q, c2, \
                             qreg, acc_o, ref, l_run)
        SPK_RUN(TILE_LIST, b0);
        SPK_RUN(TILE_LIST_MASK, b1);
        if (narrow) SPK_RUN(TILE_CONT, b2);
        else SPK_RUN(TILE_EDGE, b2);
        SPK_RUN(TILE_FAST, b3);
        SPK_RUN(TILE_DIAG, b4);
        SPK_RUN(TILE_SKIP, NT);
#undef SPK_RUN
    }

    // ---- epilogue: O = O^T / l, lse ----
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (qi < n) {
        const float inv = 1.0f / l_tot;
        uint16_t* orow = o + (qo + qi) * D;
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
        if (lse && half == 0) lse[qo + qi] = (ref.m * c2 + log2f(l_tot)) * 0.6931471805599453f;
    }
}

template <int D>
static void launch_mfma(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                        const float* tau, const int32_t* death, const ExtLists& x, const int32_t* counts,
                        void* o, float* lse, int nb, int q_begin, const int32_t* first_valid,
                        int q_rows, hipStream_t st)
{
    const int BH = c.B * c.H;
    dim3 grid(nb * BH);
#define SPK_LAUNCH(MODE)                                                                                          \
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, MODE>), grid, dim3(256), 0, st, (const uint16_t*)q,               \
                       (const uint16_t*)k, (const uint16_t*)v, u, tau, death, (const int32_t*)x.pos,              \
                       (const int32_t*)x.death, (const float*)x.u, x.KP, counts, (uint16_t*)o, lse, c.H, c.Gu,    \
                       c.n, c.k, c.w, c.softmax_scale, nb, BH, c.B * c.Gu, q_begin, first_valid, q_rows)
    if (c.gate_mode == 0) SPK_LAUNCH(0);
    else if (c.gate_mode == 1) SPK_LAUNCH(1);
    else SPK_LAUNCH(2);
#undef SPK_LAUNCH
}

void launch_block_lists_ext(const sparsek_cfg& c, const int32_t* death, int32_t* lists, int32_t* counts,
                                   const float* u, const ExtLists& x, hipStream_t st)
{
    const int nb = nblocks(c.n);
    hipLaunchKernelGGL(block_lists_kernel, dim3(nb, c.B * c.Gu), dim3(64 * BL_WAVES), 0, st, death, c.n, c.k, c.w, nb,
                       lists, counts, u, x.pos, x.death, x.u, x.KP);
}

void launch_block_lists(const sparsek_cfg& c, const int32_t* death, int32_t* lists, int32_t* counts,
                        hipStream_t st)
{
    launch_block_lists_ext(c, death, lists, counts, nullptr, ExtLists{nullptr, nullptr, nullptr, 0}, st);
}

int launch_attn_fwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, void* o, float* lse, void* ws,
                    hipStream_t st, int q_begin, const int32_t* first_valid, int q_rows)
{
    const int nb = nblocks(c.n);
    size_t coff = 0;
    const size_t lb = block_lists_bytes(c, &coff);
    int32_t* lists = (int32_t*)ws;
    int32_t* counts = (int32_t*)((char*)ws + coff);
    if (c.dtype == SPARSEK_BF16 && (c.d == 64 || c.d == 128) && (uint64_t)c.n * c.d * 2 <= 0xFFFFFFFFull) {
        const size_t xb = ext_array_bytes(c);
        ExtLists x;
        x.pos = (int32_t*)((char*)ws + lb);
        x.death = (int32_t*)((char*)ws + lb + xb);
        x.u = (float*)((char*)ws + lb + 2 * xb);
        x.KP = (int)ext_stride(c);
        launch_block_lists_ext(c, death, lists, counts, u, x, st);
        if (c.d == 64) launch_mfma<64>(c, q, k, v, u, tau, death, x, counts, o, lse, nb, q_begin, first_valid, q_rows, st);
        else launch_mfma<128>(c, q, k, v, u, tau, death, x, counts, o, lse, nb, q_begin, first_valid, q_rows, st);
        return launch_status();
    }
    launch_block_lists(c, death, lists, counts, st);
    dim3 grid(nb * GEN_SPLIT, c.B * c.H);
    if (c.dtype == SPARSEK_F32) {
        hipLaunchKernelGGL(attn_fwd_generic_kernel<float>, grid, dim3(256), 0, st, (const float*)q,
                           (const float*)k, (const float*)v, u, tau, death, lists, counts, (float*)o, lse, c.H,
                           c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale, nb, q_begin, first_valid, q_rows);
    } else {
        hipLaunchKernelGGL(attn_fwd_generic_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)q,
                           (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, (uint16_t*)o,
                           lse, c.H, c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale, nb, q_begin, first_valid, q_rows);
    }
    return launch_status();
}

}  // namespace spk

// Attention backward: gradients of L = sum(dO * O) with respect to q, k, v, the gates held fixed
// (the gradient with respect to the scores is mask_bwd.hip's).  From the selected-attention
// equations of Sec. 3.2 with the gating variants: with s_ij = scale gk_ij (q_i.k_j), p = softmax,
// o_i = sum_j p_ij gv_ij v_j and D_i = dO_i.o_i,
//     dV_j = sum_i p_ij gv_ij dO_i        dp_ij = gv_ij (dO_i.v_j)      ds_ij = p_ij (dp_ij - D_i)
//     dQ_i = sum_j ds_ij scale gk_ij k_j  dK_j  = sum_i ds_ij scale gk_ij q_i
// gk = gate in mode 0, else 1; gv = gate in modes 0 and 1, else 1; window keys carry gate 1.
// p_ij is recomputed from q, k and the forward's lse; nothing of size n x (k + w) is stored.
#include "common.hpp"
#include "attn_tiles.hpp"

namespace spk {

void launch_block_lists(const sparsek_cfg& c, const int32_t* death, int32_t* lists, int32_t* counts,
                        hipStream_t st);
size_t block_lists_bytes(const sparsek_cfg& c, size_t* counts_offset);

struct AbwdWs {
    size_t lists, counts, xpos, xdeath, xu, delta, lse2, elist, ecount, eslot, dk32, dv32, sk32, sv32, total;
};
static AbwdWs abwd_ws(const sparsek_cfg& c)
{
    AbwdWs W;
    size_t coff = 0;
    const size_t lb = block_lists_bytes(c, &coff);
    const size_t BH = (size_t)c.B * c.H;
    W.lists = 0;
    W.counts = coff;
    size_t off = align_up(lb, 256);
    W.xpos = off; off += ext_array_bytes(c);
    W.xdeath = off; off += ext_array_bytes(c);
    W.xu = off; off += ext_array_bytes(c);
    W.delta = off; off += align_up(BH * c.n * 4, 256);
    W.lse2 = off; off += align_up(BH * c.n * 4, 256);
    W.elist = off; off += align_up((size_t)c.B * c.Gu * c.n * 4, 256);
    W.ecount = off; off += align_up((size_t)c.B * c.Gu * 4, 256);
    W.eslot = off; off += align_up((size_t)c.B * c.Gu * c.n * 4, 256);
    W.dk32 = off; off += align_up(BH * c.n * c.d * 4, 256);
    W.dv32 = off; off += align_up(BH * c.n * c.d * 4, 256);
    W.sk32 = off; off += align_up(BH * c.n * c.d * 4, 256);
    W.sv32 = off; off += align_up(BH * c.n * c.d * 4, 256);
    W.total = off;
    return W;
}
size_t attn_bwd_ws_bytes(const sparsek_cfg& c) { return abwd_ws(c).total; }

template <typename T>
__device__ __forceinline__ float ldg(const T* p);
template <>
__device__ __forceinline__ float ldg<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ldg<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <typename T>
__device__ __forceinline__ void stg(T* p, float v);
template <>
__device__ __forceinline__ void stg<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void stg<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

__global__ void abwd_zero_kernel(uint4* p, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = make_uint4(0, 0, 0, 0);
}

// delta[bh][i] = dO_i . o_i: one wave per row.
template <typename T>
__global__ __launch_bounds__(256) void abwd_delta_kernel(const T* __restrict__ o, const T* __restrict__ dO, size_t rows,
                                                         int d, float* __restrict__ delta)
{
    const size_t r = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= rows) return;
    float s = 0.0f;
    for (int c = lane; c < d; c += 64) s += ldg(o + r * d + c) * ldg(dO + r * d + c);
    s = wave_sum_f32(s);
    if (lane == 0) delta[r] = s;
}

// The same for bf16 rows of d = 8 * LPR elements: LPR lanes per row, 16 bytes per lane.  Also writes
// lse2 = lse * log2(e), the form the exponent of the dK/dV kernel subtracts.
template <int LPR>
__global__ __launch_bounds__(256) void abwd_delta_bf16_kernel(const uint16_t* __restrict__ o, const uint16_t* __restrict__ dO,
                                                              size_t rows, float* __restrict__ delta,
                                                              const float* __restrict__ lse, float* __restrict__ lse2)
{
    constexpr int RPB = 256 / LPR;  // rows per workgroup
    const size_t r = (size_t)blockIdx.x * RPB + threadIdx.x / LPR;
    if (r >= rows) return;  // whole groups of LPR lanes leave together
    const size_t off = (r * LPR + threadIdx.x % LPR) * 8;
    const uint4 a = *(const uint4*)(o + off), b = *(const uint4*)(dO + off);
    const unsigned aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        s = fmaf(__uint_as_float(aw[i] << 16), __uint_as_float(bw[i] << 16), s);
        s = fmaf(__uint_as_float(aw[i] & 0xffff0000u), __uint_as_float(bw[i] & 0xffff0000u), s);
    }
#pragma unroll
    for (int m = LPR / 2; m > 0; m >>= 1) s += __shfl_xor(s, m, 64);
    if (threadIdx.x % LPR == 0) {
        delta[r] = s;
        lse2[r] = lse[r] * 1.4426950408889634f;
    }
}

// fp32 accumulators -> storage type
template <typename T>
__global__ void abwd_convert_kernel(const float* __restrict__ a, const float* __restrict__ b, T* __restrict__ oa,
                                    T* __restrict__ ob, size_t nelem)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nelem; i += (size_t)gridDim.x * blockDim.x) {
        stg(oa + i, a[i]);
        stg(ob + i, b[i]);
    }
}

// ---------------------------------------------------------------------------------
// Generic vector-ALU kernel (fp32 or bf16 storage, any d <= 128 that is a multiple of 4): one wave
// per query, lanes over keys for the dot products, over columns for the row updates.  dQ stays
// with the wave; dK and dV rows are accumulated in fp32 with one atomic per column.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ kk, const T* __restrict__ v, const float* __restrict__ u,
    const float* __restrict__ tau, const int32_t* __restrict__ death, const int32_t* __restrict__ lists,
    const int32_t* __restrict__ counts, const float* __restrict__ lse, const T* __restrict__ dO,
    const float* __restrict__ delta, T* __restrict__ dq, float* __restrict__ dk32, float* __restrict__ dv32, int H,
    int Gu, int n, int d, int k, int w, int gate_mode, float scale, int nb)
{
    __shared__ float qs[4][128], ds[4][128];
    const int blk = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i0 = blk * QB;
    const size_t hb = (size_t)bh * n * d;
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int32_t* list = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    const int cnt = counts[(size_t)row * nb + blk];
    const int c0 = max(0, i0 - w + 1);
    const bool gate_k = gate_mode == 0, gate_v = gate_mode == 0 || gate_mode == 1;

    for (int qi = wv; qi < QB; qi += 4) {
        const int i = i0 + qi;
        if (i >= n) break;
        for (int c = lane; c < d; c += 64) {
            qs[wv][c] = ldg(q + hb + (size_t)i * d + c);
            ds[wv][c] = ldg(dO + hb + (size_t)i * d + c);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        const int Tp = i - w;
        const float tauT = (Tp >= 0) ? tr[Tp] : 0.0f;
        const float lse_i = lse[(size_t)bh * n + i];
        const float Di = delta[(size_t)bh * n + i];
        float dq0 = 0.0f, dq1 = 0.0f;  // columns lane and lane + 64 of dQ_i
        const int n_list = (Tp >= 0) ? cnt : 0;
        const int total = n_list + (i - c0 + 1);
        for (int e0 = 0; e0 < total; e0 += 64) {
            const int e = e0 + lane;
            int j = -1;
            if (e < total) j = (e < n_list) ? list[e] : c0 + (e - n_list);
            bool valid = false;
            float gate = 1.0f;
            if (j >= 0) {
                if (i - j < w) valid = true;
                else if (dr[j] > Tp) { valid = true; gate = clip01(ur[j] - tauT); }
            }
            float pv = 0.0f, coef = 0.0f;
            if (valid) {
                float qk = 0.0f, dov = 0.0f;
                const T* kj = kk + hb + (size_t)j * d;
                const T* vj = v + hb + (size_t)j * d;
                for (int c = 0; c < d; c++) {
                    qk += qs[wv][c] * ldg(kj + c);
                    dov += ds[wv][c] * ldg(vj + c);
                }
                const float gk = gate_k ? gate : 1.0f, gv = gate_v ? gate : 1.0f;
                const float p = __expf(scale * gk * qk - lse_i);
                pv = p * gv;
                coef = p * (gv * dov - Di) * scale * gk;
            }
            unsigned long long ball = __ballot(valid);
            while (ball) {
                const int src = __builtin_ctzll(ball);
                ball &= ball - 1;
                const float ps = __shfl(pv, src, 64), cs = __shfl(coef, src, 64);
                const int js = __shfl(j, src, 64);
                const size_t ro = hb + (size_t)js * d;
                if (lane < d) {
                    dq0 += cs * ldg(kk + ro + lane);
                    unsafeAtomicAdd(dv32 + ro + lane, ps * ds[wv][lane]);
                    unsafeAtomicAdd(dk32 + ro + lane, cs * qs[wv][lane]);
                }
                if (lane + 64 < d) {
                    dq1 += cs * ldg(kk + ro + lane + 64);
                    unsafeAtomicAdd(dv32 + ro + lane + 64, ps * ds[wv][lane + 64]);
                    unsafeAtomicAdd(dk32 + ro + lane + 64, cs * qs[wv][lane + 64]);
                }
            }
        }
        if (dq) {  // null: dQ comes from the MFMA kernel
            if (lane < d) stg(dq + hb + (size_t)i * d + lane, dq0);
            if (lane + 64 < d) stg(dq + hb + (size_t)i * d + lane + 64, dq1);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    }
}

// ---------------------------------------------------------------------------------
// MFMA kernel for dQ (bf16, D = 64 or 128).  Same blocking and the same walk over a query block's key set as the
// forward (attn_fwd.hip): 128 queries x 4 waves, 64-key tiles (the block's top-k list, then the contiguous keys up
// to the block's last query) in runs of one kind per wave, so that only the tiles that need a test or a gate pay
// for it; metadata staged in segments, tiles gathered straight into LDS one tile ahead.  Per 32-key half:
// S^T = K.Q^T and DV^T = V.dO^T (row reads of the K and V tiles), the elementwise step to ds_ij gk_ij in bf16, then
// dQ^T += K^T.dS^T with K^T through transposing reads of the same K tile (see tile_swz).  The softmax scale is
// applied once, to the finished dQ.
// ---------------------------------------------------------------------------------
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
// two floats rounded to bf16 (nearest even), the first in the low half
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b)
{
    f32x2v f = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2v));
}

// A 64-row tile in LDS (K rows in the dQ kernel, Q and dO rows in the dK/dV kernel) serves two kinds of reads: 16-byte
// row reads (A operand of the contractions over the head dimension) and transposing 8-byte reads (A operand of the
// contractions over the tile's rows).  Each row lands once, unpadded, with its 16-byte chunks
// permuted: chunk c of tile row R sits at chunk position c ^ swz(R).  swz is chosen so that both read patterns
// touch every bank once per pass:
//   row reads take one chunk column of 16 consecutive rows per 16 lanes  -> swz must differ on those rows
//   transposing reads take 4 neighbouring chunks of 4 consecutive rows per 32 lanes -> swz / 4 must differ on those rows
// (head dim 64: a row is half of the 64 banks, two rows share a pass, and the row's parity takes the place of one bit).
template <int D>
__device__ __forceinline__ int tile_swz(int R)
{
    if constexpr (D == 128) return 4 * (R & 3) + ((R >> 2) & 3);
    else return 4 * ((R >> 1) & 1) + ((R >> 2) & 3);
}

// K lands twice, once per padding (row reads and transposing reads of one padded copy would conflict; the
// chunk-permuted single copy the dK/dV kernel uses needs 16 more address registers than this kernel has at two
// workgroups per compute unit); the tile is single-buffered and the two workgroups of a compute unit cover each
// other's gathers.
template <int D>
struct DqSmem : TileMeta {
    using S = MfmaTileBufs<D, 64>;
    unsigned char kr[S::NL * S::GSK];  // K rows, padded for row reads
    unsigned char kt[S::NL * S::GSV];  // K rows, padded for transposing reads
    unsigned char vr[S::NL * S::GSK];  // V rows, padded for row reads
};
static_assert(sizeof(DqSmem<128>) <= 80 * 1024, "two workgroups per CU");

// What a lane of the dQ kernel keeps for the whole block.
struct DqLane {
    float tau_q, lse2, Di; // threshold of the query's prefix, lse * log2(e), dO.o
    int qi;
};

// The gather of one tile: K (twice) and V rows at the positions jp[0..63].
template <int D>
__device__ __forceinline__ void dq_issue(DqSmem<D>& sm, const int32_t* jp, const unsigned char* kh,
                                         const unsigned char* vh, int wv, int lane)
{
    using S = MfmaTileBufs<D, 64>;
    constexpr int NX = S::NL / 4, LPR = S::RB / 16;
    const TileRows<D, 64> rows = tile_rows<D, 64>(jp, wv, lane);
    const int c = lane % LPR;
#pragma unroll
    for (int x = 0; x < NX; x++) {
        const int L = wv * NX + x;
        const uint32_t off = (uint32_t)rows.j[x] * (uint32_t)S::RB + 16u * (uint32_t)c;
        async_load_lds16(kh, off, &sm.kr[L * S::GSK]);
        async_load_lds16(vh, off, &sm.vr[L * S::GSK]);
        async_load_lds16(kh, off, &sm.kt[L * S::GSV]);
    }
}

// One 64-key tile for one wave.  jbase: position of the tile's first key if the key set were contiguous.
template <int D, int MODE, int KIND>
__device__ __forceinline__ void dq_tile_body(DqSmem<D>& sm, const int32_t* jdeath, const float* ju, int jbase,
                                             const DqLane& ln, int lane, int w, float c2,
                                             const bf16x8 (&qreg)[D / 16], const bf16x8 (&dreg)[D / 16],
                                             f32x16 (&acc_q)[D / 32])
{
    using TT = TileTraits<MODE, KIND>;
    using S = MfmaTileBufs<D, 64>;
    constexpr int DS = D / 16, DB = D / 32;
    const int half = lane >> 5, col = lane & 31;
    const int qw = ln.qi - (w - 1);
    const int dqh = ln.qi - jbase - 4 * half;  // contiguous tiles: key number cst + 4*half sits dqh - cst behind the query
    const int dqw = dqh - w;                   // in the window  <=>  cst > dqw
    // transposing reads of K^T (see the forward's V^T operand): lane -> (row, column block)
    const int r16 = lane & 15, grp2 = (lane >> 4) & 1;
    const int tcol = (16 * grp2 + 4 * (r16 & 3)) * 2;
    const int trow = 4 * half + (r16 >> 2);
    auto kt_operand = [&](int g, int x) -> bf16x8 {
        const int row0 = 16 * g + trow, row1 = row0 + 8;
        const unsigned char* p0 = sm.kt + (row0 % S::NL) * S::GSV + (row0 / S::NL) * S::RB + tcol + 64 * x;
        const unsigned char* p1 = sm.kt + (row1 % S::NL) * S::GSV + (row1 / S::NL) * S::RB + tcol + 64 * x;
        const i16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)p0);
        const i16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)p1);
        const bf16x4 lo = __builtin_bit_cast(bf16x4, lo4), hi = __builtin_bit_cast(bf16x4, hi4);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
#pragma unroll
    for (int mb = 0; mb < 2; mb++) {
        const int trw = 32 * mb + col;
        const int off = (trw % S::NL) * S::GSK + (trw / S::NL) * S::RB + 16 * half;
        const f32x16 zero = {0};
        f32x16 acc_s = zero, acc_d = zero;
        __builtin_amdgcn_sched_barrier(0);  // one half at a time: there are no registers for two in flight
#pragma unroll
        for (int s = 0; s < DS; s++) {
            const bf16x8 ka = *(const bf16x8*)(sm.kr + off + 32 * s);
            const bf16x8 va = *(const bf16x8*)(sm.vr + off + 32 * s);
            acc_s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], s == 0 ? zero : acc_s, 0, 0, 0);
            acc_d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, dreg[s], s == 0 ? zero : acc_d, 0, 0, 0);
        }
        // ds_ij gk_ij without the softmax scale; a pair that is not attended gets p = 0 through the exponent
        u32x4 dsb[2];
        float hold = 0.0f;
#pragma unroll
        for (int g4 = 0; g4 < 4; g4++) {
            const int kb = 32 * mb + 8 * g4 + 4 * half;
            float4 U4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            int4 L4 = make_int4(0, 0, 0, 0);
            if (TT::GATED) U4 = *(const float4*)&ju[kb];
            if (TT::MASKL) L4 = *(const int4*)&jdeath[kb];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int r = 4 * g4 + e;
                const int cst = 32 * mb + 8 * g4 + e;  // key number in the tile minus the lane's 4 * half (folded into dqh, dqw)
                const int Lj = e == 0 ? L4.x : e == 1 ? L4.y : e == 2 ? L4.z : L4.w;
                const float uj = e == 0 ? U4.x : e == 1 ? U4.y : e == 2 ? U4.z : U4.w;
                const float qk = acc_s[r], dov = acc_d[r];
                float gate = 1.0f;
                if (TT::GATED) {
                    gate = clip01(uj - ln.tau_q);
                    if (TT::SELECT) gate = (cst > dqw) ? 1.0f : gate;
                }
                float arg = TT::KGATE ? fmaf(qk, gate * c2, -ln.lse2) : fmaf(qk, c2, -ln.lse2);
                // key j is attended by query i while j <= i and i - (w - 1) <= death[j]
                if (TT::MASKL && TT::MASKC) arg = (cst <= dqh && qw <= Lj) ? arg : -INFINITY;
                else if (TT::MASKL) arg = (qw <= Lj) ? arg : -INFINITY;
                else if (TT::MASKC) arg = (cst <= dqh) ? arg : -INFINITY;
                const float p = __builtin_amdgcn_exp2f(arg);
                float ds = p * (TT::GATED ? fmaf(gate, dov, -ln.Di) : dov - ln.Di);
                if (TT::KGATE) ds *= gate;
                if ((r & 1) == 0) hold = ds;
                else dsb[r >> 3][(r & 7) >> 1] = pack_bf16x2(hold, ds);
            }
        }
#pragma unroll
        for (int i = 0; i < 2 * DB; i++)
            acc_q[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_operand(2 * mb + i / DB, i % DB),
                                                                    __builtin_bit_cast(bf16x8, dsb[i / DB]),
                                                                    acc_q[i % DB], 0, 0, 0);
    }
}

// The tiles [T, T_end) of the block's key set, all of one kind; the metadata of tile T sits in segment T / TPS.
template <int D, int MODE, int KIND>
__device__ __forceinline__ void dq_run_tiles(DqSmem<D>& sm, const StageSrc& src, int& T, int T_end, int jbase0,
                                             const unsigned char* kh, const unsigned char* vh, int wv, int lane,
                                             const DqLane& ln, int w, float c2, const bf16x8 (&qreg)[D / 16],
                                             const bf16x8 (&dreg)[D / 16], f32x16 (&acc_q)[D / 32])
{
    for (; T < T_end; T++) {
        const int sg = T / TPS, lt = T - sg * TPS;
        __syncthreads();  // everybody is done with tile T-1 (and, at the first tile of a segment, with the segment before)
        if (lt == 0 && (sg + 1) * TPS < src.nt) stage_meta(sm, src, sg + 1, wv, lane);
        dq_issue<D>(sm, sm.jpos[sg & 1] + lt * KT, kh, vh, wv, lane);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // the tile (and any metadata staged above) has landed
        if (KIND != TILE_SKIP)
            dq_tile_body<D, MODE, KIND>(sm, sm.jdeath[sg & 1] + lt * KT, sm.ju[sg & 1] + lt * KT, jbase0 + T * KT, ln,
                                        lane, w, c2, qreg, dreg, acc_q);
    }
}

template <int D, int MODE>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ kk, const uint16_t* __restrict__ v,
    const float* __restrict__ u, const float* __restrict__ tau, const int32_t* __restrict__ death,
    const int32_t* __restrict__ xpos, const int32_t* __restrict__ xdeath, const float* __restrict__ xu, int KP,
    const int32_t* __restrict__ counts, const float* __restrict__ lse, const uint16_t* __restrict__ dO,
    const float* __restrict__ delta, uint16_t* __restrict__ dq, int H, int Gu, int n, int k, int w, float scale,
    int nb, int BH, int nrows, int q_begin, const int32_t* __restrict__ first_valid, int q_rows)
{
    __shared__ __align__(16) DqSmem<D> sm;
    constexpr int DS = D / 16, DB = D / 32;
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
    // queries before q_begin do not exist; q, dO, lse, delta and dq then hold q_rows rows per head from query q_begin
    if (i0 + QB <= q_begin) return;
    const ptrdiff_t qo = q_rows ? (ptrdiff_t)bh * q_rows - q_begin : (ptrdiff_t)bh * n;
    const unsigned char* kh = (const unsigned char*)(kk + (size_t)bh * n * D);
    const unsigned char* vh = (const unsigned char*)(v + (size_t)bh * n * D);
    const float* tr = tau + (size_t)row * n;
    const int nstay = counts[(size_t)nrows * nb + (size_t)row * nb + blk];
    const int c0 = max(max(0, i0 - w + 1), first_valid ? first_valid[row] : 0);
    const int c_end = min(n - 1, i0 + QB - 1);
    // the list part is laid out for min(k, T0 + 1) keys, the length of a complete top-k list (see the forward)
    const int T0 = i0 - w;
    const int nkl = (T0 >= 0 && k > 0) ? (min(k, T0 + 1) + KT - 1) / KT * KT : 0;
    const int nkc = max(0, (c_end - c0 + 1 + KT - 1) / KT * KT);
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

    const int qa = i0 + 32 * wv;
    const int qb = min(qa + 31, n - 1);
    const bool wave_live = qa < n;
    DqLane ln;
    ln.qi = qa + col;
    const int qrow = min(ln.qi, n - 1);
    ln.tau_q = (ln.qi < n && ln.qi - w >= 0) ? tr[ln.qi - w] : 0.0f;
    ln.lse2 = lse[qo + qrow] * 1.4426950408889634f;
    ln.Di = delta[qo + qrow];
    bf16x8 qreg[DS], dreg[DS];
#pragma unroll
    for (int s = 0; s < DS; s++) {
        const size_t off = (size_t)(qo + qrow) * D + 16 * s + 8 * half;
        qreg[s] = *(const bf16x8*)(q + off);
        dreg[s] = *(const bf16x8*)(dO + off);
    }
    stage_meta(sm, src, 0, wv, lane);
    const WaveRuns wr = wave_runs(wave_live, nkl, nkc, nstay, qa, qb, w, c0);
    f32x16 acc_q[DB];
#pragma unroll
    for (int x = 0; x < DB; x++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc_q[x][r] = 0.0f;
    const float c2 = scale * 1.4426950408889634f;
    // Everything the compiler tracks must have arrived before the first untracked load (see the forward).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int s = 0; s < DS; s++) asm volatile("" ::"v"(qreg[s]), "v"(dreg[s]));
    asm volatile("" ::"v"(ln.tau_q), "v"(ln.lse2), "v"(ln.Di));
    // (segment 0 of the metadata is published by the first tile's barriers: each wave waits for its own copies
    //  before the second one)
    {
        const int jbase0 = c0 - nkl;
        int T = 0;
#define SPK_RUN(KIND, bound) \
    dq_run_tiles<D, MODE, KIND>(sm, src, T, min(NT, (bound)), jbase0, kh, vh, wv, lane, ln, w, c2, qreg, dreg, acc_q)
        SPK_RUN(TILE_LIST, wr.b0);
        SPK_RUN(TILE_LIST_MASK, wr.b1);
        if (wr.narrow) SPK_RUN(TILE_CONT, wr.b2);
        else SPK_RUN(TILE_EDGE, wr.b2);
        SPK_RUN(TILE_FAST, wr.b3);
        SPK_RUN(TILE_DIAG, wr.b4);
        SPK_RUN(TILE_SKIP, NT);
#undef SPK_RUN
    }
    if (ln.qi < n) {
        uint16_t* orow = dq + (size_t)(qo + ln.qi) * D;
#pragma unroll
        for (int x = 0; x < DB; x++) {
#pragma unroll
            for (int g4 = 0; g4 < 4; g4++) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; e++) pk[e] = (__bf16)(scale * acc_q[x][4 * g4 + e]);
                *(bf16x4*)(orow + 32 * x + 8 * g4 + 4 * half) = pk;
            }
        }
    }
}

template <int D>
static void launch_dq_mfma(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                           const float* tau, const int32_t* death, const ExtLists& x, const int32_t* counts,
                           const float* lse, const void* dO, const float* delta, void* dq, int nb, hipStream_t st,
                           int q_begin, const int32_t* first_valid, int q_rows)
{
    const int BH = c.B * c.H;
    dim3 grid(nb * BH);
#define SPK_LAUNCH_DQ(MODE)                                                                                        \
    hipLaunchKernelGGL((attn_bwd_dq_kernel<D, MODE>), grid, dim3(256), 0, st, (const uint16_t*)q, (const uint16_t*)k, \
                       (const uint16_t*)v, u, tau, death, (const int32_t*)x.pos, (const int32_t*)x.death,          \
                       (const float*)x.u, x.KP, counts, lse, (const uint16_t*)dO, delta, (uint16_t*)dq, c.H, c.Gu, \
                       c.n, c.k, c.w, c.softmax_scale, nb, BH, c.B * c.Gu, q_begin, first_valid, q_rows)
    if (c.gate_mode == 0) SPK_LAUNCH_DQ(0);
    else if (c.gate_mode == 1) SPK_LAUNCH_DQ(1);
    else SPK_LAUNCH_DQ(2);
#undef SPK_LAUNCH_DQ
}

// ---------------------------------------------------------------------------------
// MFMA kernel for dK and dV (bf16, D = 64 or 128): the mirror image of the forward.  A workgroup
// owns 128 keys (4 waves x 32 keys) whose K and V fragments stay in registers, and streams 64-query
// tiles of Q and dO through LDS, so S = Q.K^T and dO.V^T land with lane = key; P and dS are then
// directly the B operands of dV^T += dO^T.P and dK^T += Q^T.dS (Q^T, dO^T through transposing LDS
// reads).  Nothing is reduced across waves and no row data goes through atomics inside the loop.
// Because a key is attended on one contiguous range of queries, two kinds of key blocks cover all
// pairs with one interval test per pair:
//   window blocks    128 consecutive positions, queries j <= i <= j + w - 1, gate 1;
//   selected blocks  128 ever-selected keys (death_j > j, listed by death, see abwd_elist_kernel), queries
//                    j + w <= i <= death_j + w - 1, gate clip(u_j - tau_{i-w}).
// Every key belongs to exactly one window block and at most one selected block, so nothing needs an
// atomic: a window block stores the final dk, dv rows of the keys that are never selected, and its
// fp32 part of the others into dk32 / dv32 by position; a selected block stores into sk32 / sv32 at
// the key's slot of the list; abwd_merge_kernel adds the two parts and rounds.
// With q_rows != 0 the queries are offset (a chunk attending retained keys): q, dO, lse, delta, dk, dv
// hold q_rows rows per head from position q_begin, and only keys from q_begin on are processed.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ int wave_max_i32(int x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = max(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ int wave_min_i32(int x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = min(x, __shfl_xor(x, o, 64));
    return x;
}

__device__ __forceinline__ int b_row(int bh, int H, int Gu) { return (bh / H) * Gu + (Gu == 1 ? 0 : bh % H); }

// elist: the ever-selected keys of a score row (death_j > j), ordered by death_j / bw and then by position,
// so that the 32 keys of a wave and the 128 of a block stop being attended at about the same query and the
// span of query tiles they walk is short.  eslot[j]: where key j sits in that list, -1 if it is not in it.
// A counting sort whose result does not depend on timing: every wave owns a contiguous range of positions
// and its own cursor per bucket.
constexpr int EBK = 512;
__global__ __launch_bounds__(1024) void abwd_elist_kernel(const int32_t* __restrict__ death, int n, int j_min,
                                                          int32_t* __restrict__ elist, int32_t* __restrict__ ecount,
                                                          int32_t* __restrict__ eslot)
{
    __shared__ int cur[16][EBK];
    __shared__ int start[EBK];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int32_t* dr = death + (size_t)row * n;
    int32_t* el = elist + (size_t)row * n;
    int32_t* es = eslot + (size_t)row * n;
    const int bw = max(256, (n + EBK) / EBK);  // death <= n, so death / bw < EBK
    for (int i = tid; i < 16 * EBK; i += 1024) (&cur[0][0])[i] = 0;
    __syncthreads();
    const int per = ((n + 15) / 16 + 63) / 64 * 64;
    const int j_begin = min(n, wv * per), j_end = min(n, j_begin + per);
    for (int j0 = j_begin; j0 < j_end; j0 += 64) {
        const int j = j0 + lane;
        const int dj = j < j_end ? dr[j] : 0;
        if (j < j_end && dj > j && j >= j_min) atomicAdd(&cur[wv][dj / bw], 1);
    }
    __syncthreads();
    if (tid < EBK) {  // per bucket: each wave's offset inside the bucket, and the bucket's size
        int acc = 0;
#pragma unroll
        for (int x = 0; x < 16; x++) {
            const int c = cur[x][tid];
            cur[x][tid] = acc;
            acc += c;
        }
        start[tid] = acc;
    }
    __syncthreads();
    if (wv == 0) {  // exclusive scan of the bucket sizes, 8 buckets per lane
        int v[EBK / 64], sum = 0;
#pragma unroll
        for (int i = 0; i < EBK / 64; i++) { v[i] = start[lane * (EBK / 64) + i]; sum += v[i]; }
        int incl = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o, 64);
            if (lane >= o) incl += y;
        }
        int ex = incl - sum;
#pragma unroll
        for (int i = 0; i < EBK / 64; i++) { start[lane * (EBK / 64) + i] = ex; ex += v[i]; }
        if (lane == 63) ecount[row] = incl;
    }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int j0 = j_begin; j0 < j_end; j0 += 64) {
        const int j = j0 + lane;
        const int dj = j < j_end ? dr[j] : 0;
        const bool sel = j < j_end && dj > j && j >= j_min;  // keys before j_min receive no gradient
        const int bkt = sel ? dj / bw : -1;
        int slot = -1;
        unsigned long long rem = __ballot(sel);
        while (rem) {  // one turn per distinct bucket among this step's lanes
            const int l = __ffsll((long long)rem) - 1;
            const int bb = __shfl(bkt, l, 64);
            const unsigned long long m = __ballot(bkt == bb);
            const int base = start[bb] + cur[wv][bb];
            if (bkt == bb) slot = base + __popcll(m & below);
            if (lane == l) cur[wv][bb] += __popcll(m);
            rem &= ~m;
        }
        if (sel) el[slot] = j;
        if (j < j_end) es[j] = slot;
    }
}

constexpr int DKV_NBUF = 2;  // tiles in LDS: one in use, one being filled
template <int D>
struct DkvSmem {
    struct Tile {
        unsigned char q[KT * D * 2];   // Q rows of a tile
        unsigned char g[KT * D * 2];   // dO rows
    } t[DKV_NBUF];
    int red[2][4];
};

template <int D, int MODE>
__global__ __launch_bounds__(256, 1) void attn_bwd_dkv_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ kk, const uint16_t* __restrict__ v,
    const float* __restrict__ u, const float* __restrict__ tau, const int32_t* __restrict__ death,
    const int32_t* __restrict__ elist, const int32_t* __restrict__ ecount, const float* __restrict__ lse2s,
    const uint16_t* __restrict__ dO, const float* __restrict__ delta, float* __restrict__ dk32,
    float* __restrict__ dv32, float* __restrict__ sk32, float* __restrict__ sv32, const int32_t* __restrict__ eslot,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int H, int Gu, int n, int w, float scale, int nb,
    int q_begin, int q_rows)
{
    using S = MfmaTileBufs<D, 64>;  // (tile geometry only)
    __shared__ __align__(16) DkvSmem<D> sm;
    // per query of a tile: lse * log2(e), D_i, tau_{i-w} (and a fourth row that only keeps the loads branch-free)
    __shared__ __align__(16) float meta[DKV_NBUF][4][KT];
    constexpr int DS = D / 16, DB = D / 32, NX = S::NL / 4, LPR = S::RB / 16, RB = S::RB, RPL = S::RPL;
    const int bh = blockIdx.x;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;
    // The head is the fast grid index: workgroups go to the chip's 8 partitions in turn, so each partition
    // keeps whole heads (the same mix of block lengths everywhere, and a head's rows in one L2).  Blocks of
    // selected keys come first, latest deaths (longest spans) first; the short window blocks fill the tail.
    const bool selected_kind = (int)blockIdx.y < nb;
    int kblk = blockIdx.y - nb;
    if (selected_kind) {  // y = 0 is the list's last block; the workgroups beyond the list come after it and leave at once
        const int ne_blocks = (ecount[b_row(blockIdx.x, H, Gu)] + 127) / 128;
        kblk = (int)blockIdx.y < ne_blocks ? ne_blocks - 1 - (int)blockIdx.y : nb;
    }
    const float* ur = u + (size_t)row * n;
    const float* tr = tau + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const int ne = selected_kind ? ecount[row] : n;
    if (kblk * 128 >= ne) return;  // no such block of selected keys
    // Keys before q_begin receive no gradient and queries before it do not exist (q_begin is a multiple of
    // 128); q, dO, lse, delta, dk and dv then hold q_rows rows per head from position q_begin.
    if (!selected_kind && kblk * 128 + 128 <= q_begin) return;
    const ptrdiff_t qo = q_rows ? (ptrdiff_t)bh * q_rows - q_begin : (ptrdiff_t)bh * n;

    // ---- this lane's key and the queries that attend it ----
    const int kidx = kblk * 128 + 32 * wv + col;
    const bool kreal = kidx < ne;
    const int j = !kreal ? 0 : selected_kind ? elist[(size_t)row * n + kidx] : kidx;
    int lo = 1, hi = 0;  // empty for a filler lane
    float uj = 0.0f;
    if (kreal) {
        if (selected_kind) { lo = j + w; hi = min(n - 1, dr[j] + w - 1); uj = ur[j]; }
        else { lo = j; hi = min(n - 1, j + w - 1); }
    }
    const bool kvalid = lo <= hi;
    const int wlo = wave_min_i32(kvalid ? lo : 0x7fffffff);
    const int whi = wave_max_i32(kvalid ? hi : -1);
    // a tile inside [wfull_lo, wfull_hi] is attended in full by every key of the wave: no interval tests there
    const int wfull_lo = wave_max_i32(kvalid ? lo : 0x7fffffff);
    const int wfull_hi = wave_min_i32(kvalid ? hi : -1);
    // query i attends this lane's key iff (unsigned)(i - lo_eff) <= span (never for an empty lane)
    const int lo_eff = kvalid ? lo : 0x7fffffff;
    const unsigned span = kvalid ? (unsigned)(hi - lo) : 0u;
    if (lane == 0) { sm.red[0][wv] = wlo; sm.red[1][wv] = whi; }
    bf16x8 kreg[DS], vreg[DS];
#pragma unroll
    for (int s = 0; s < DS; s++) {
        const size_t off = ((size_t)bh * n + j) * D + 16 * s + 8 * half;
        kreg[s] = *(const bf16x8*)(kk + off);
        vreg[s] = *(const bf16x8*)(v + off);
    }
    f32x16 acc_k[DB], acc_v[DB];
#pragma unroll
    for (int x = 0; x < DB; x++)
#pragma unroll
        for (int r = 0; r < 16; r++) { acc_k[x][r] = 0.0f; acc_v[x][r] = 0.0f; }
    __syncthreads();
    const int blo = min(min(sm.red[0][0], sm.red[0][1]), min(sm.red[0][2], sm.red[0][3]));
    const int bhi = max(max(sm.red[1][0], sm.red[1][1]), max(sm.red[1][2], sm.red[1][3]));
    const int ntiles = blo > bhi ? 0 : (bhi - blo) / KT + 1;  // (uniform) 0: nothing attends these keys
    const float c2 = scale * 1.4426950408889634f;
    const unsigned char* qh = (const unsigned char*)(q + qo * D);
    const unsigned char* gh = (const unsigned char*)(dO + qo * D);

    // LDS byte offsets of this lane's operand reads (see tile_swz):
    //   row reads: tile row 32 * run + col, chunk 2 * step + half          -> roff[run][step]
    //   transposing reads: rows 16 g + 4 half + r16 / 4 (+ 8), chunk 4 x + 2 grp2 + (r16 % 4) / 2, 8-byte half r16 % 2
    //                                                                      -> toff[0 / 1][x] + 16 g rows
    const int r16 = lane & 15, grp2 = (lane >> 4) & 1;
    int roff[2][DS], toff[2][DB];
#pragma unroll
    for (int run = 0; run < 2; run++) {
        const int R = 32 * run + col, sw = tile_swz<D>(R);
#pragma unroll
        for (int st = 0; st < DS; st++) roff[run][st] = R * RB + (((2 * st + half) ^ sw) << 4);
    }
#pragma unroll
    for (int hl = 0; hl < 2; hl++) {
        const int R = 4 * half + (r16 >> 2) + 8 * hl, sw = tile_swz<D>(R);  // (swz has period 16 in R)
#pragma unroll
        for (int x = 0; x < DB; x++)
            toff[hl][x] = R * RB + (((4 * x + 2 * grp2 + ((r16 & 3) >> 1)) ^ sw) << 4) + 8 * (r16 & 1);
    }
    auto t_operand = [&](const unsigned char* tbuf, int g, int x) -> bf16x8 {
        const unsigned char* p0 = tbuf + 16 * g * RB + toff[0][x];
        const unsigned char* p1 = tbuf + 16 * g * RB + toff[1][x];
        const i16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)p0);
        const i16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3)))*)p1);
        const bf16x4 l4 = __builtin_bit_cast(bf16x4, lo4), h4 = __builtin_bit_cast(bf16x4, hi4);
        return __builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // The gather of one tile (64 consecutive queries from i_first, clamped to the last row): a wave-load fills RPL
    // consecutive tile rows; lane l delivers position l % LPR of row l / LPR, i.e. chunk (l % LPR) ^ swz(row).
    int goff[NX];  // byte offset of this lane's chunk inside a tile whose first row is at 0
#pragma unroll
    for (int x = 0; x < NX; x++) {
        const int R = RPL * (wv * NX + x) + lane / LPR;
        goff[x] = R * RB + (((lane % LPR) ^ tile_swz<D>(R)) << 4);
    }
    auto issue = [&](int buf, int i_first) {
#pragma unroll
        for (int x = 0; x < NX; x++) {
            const int R = RPL * (wv * NX + x) + lane / LPR;
            // rows past the end of the sequence repeat the last row (their pairs are masked)
            const int over = max(i_first + R - (n - 1), 0);
            const uint32_t off = (uint32_t)i_first * (uint32_t)RB + (uint32_t)(goff[x] - over * RB);
            async_load_lds16(qh, off, &sm.t[buf].q[(wv * NX + x) * 1024]);
            async_load_lds16(gh, off, &sm.t[buf].g[(wv * NX + x) * 1024]);
        }
    };
    // the tile's per-query values: waves 0, 1, 2 load one row each (wave 3 a copy of tau into the spare row)
    const float* msrc = wv == 0 ? lse2s + qo : wv == 1 ? delta + qo : tr;
    auto issue_meta = [&](int buf, int i_first) {
        const int i = min(i_first + lane, n - 1);
        async_load_lds4(msrc, 4u * (uint32_t)(wv >= 2 ? max(i - w, 0) : i), &meta[buf][wv][0]);
    };
    if (ntiles > 0) {
        issue_meta(0, blo);
        issue(0, blo);
    }
    // The K / V fragments must have arrived before the tile loop: the compiler's own wait for them would otherwise
    // sit at their first use, inside the loop, and count the prefetches of every iteration too.  (The first tile's
    // gather is already in flight beside them; the loop waits for it anyway.)
#pragma unroll
    for (int s = 0; s < DS; s++) asm volatile("" ::"v"(kreg[s]), "v"(vreg[s]));
    // One tile for this wave, as four runs of NS MFMAs:
    //   1: S and dO.V of queries 0..31            2: the same for queries 32..63, under it the elementwise
    //   3: dV, dK += from queries 0..31, under        work (P, dS) of queries 0..31
    //      it the elementwise work of 32..63       4: dV, dK += from queries 32..63
    // Every step issues one MFMA and a slice of elementwise work, fenced so that the interleave survives the
    // scheduler; MFMA operands come from LDS through a small ring filled DEPTH steps ahead.  GATED: the keys
    // carry soft gates (selected keys, gate modes 0 and 1); CHECK: some (query, key) pair of the tile may lie
    // outside the key's interval.  The softmax scale of dS is applied once, to the finished dK.
    constexpr int NS = 2 * DS, EPM = 16 / NS, DEPTH = 4;
    static_assert(NS == 4 * DB && EPM * NS == 16, "stage lengths");
    const unsigned char* mbase = (const unsigned char*)&meta[0][0][0];
    // (the buffer number is a compile-time constant, so that every LDS address is a per-lane register plus an immediate)
    auto tile = [&](auto gated_c, auto check_c, auto buf_c, int i_first) {
        constexpr bool GATED = decltype(gated_c)::value, CHECK = decltype(check_c)::value;
        constexpr int buf = decltype(buf_c)::value;
        constexpr bool GK = GATED && MODE == 0, GV = GATED && MODE != 2;
        const f32x16 zero = {0};
        f32x16 s0 = zero, d0 = zero, s1 = zero, d1 = zero;
        u32x4 pb0[2], dsb0[2], pb1[2], dsb1[2];
        const int rel0 = i_first + 4 * half - lo_eff;
        // operand idx of the tile's 4 * NS MFMAs, in issue order
        auto operand = [&](auto ic) -> bf16x8 {
            constexpr int idx = decltype(ic)::value, run = idx / NS, m = idx % NS;
            if constexpr (run < 2) {
                const unsigned char* base = (m & 1) ? sm.t[buf].g : sm.t[buf].q;
                return *(const bf16x8*)(base + roff[run][m / 2]);
            } else {
                constexpr int qb = run - 2, i2 = m / 2, g = 2 * qb + i2 / DB, x = i2 % DB;
                return t_operand((m & 1) ? sm.t[buf].q : sm.t[buf].g, g, x);
            }
        };
        bf16x8 ring[DEPTH];
        static_for<0, DEPTH>([&](auto ic) { ring[decltype(ic)::value] = operand(ic); });
        auto refill = [&](auto ic) {
            constexpr int idx = decltype(ic)::value;
            if constexpr (idx + DEPTH < 4 * NS) ring[idx % DEPTH] = operand(std::integral_constant<int, idx + DEPTH>{});
        };
        float4 L4, D4, T4;
        float hold_p = 0.0f, hold_s = 0.0f;
        auto element = [&](auto qbc, auto rc, const f32x16& sacc, const f32x16& dacc, u32x4(&pb)[2], u32x4(&dsb)[2]) {
            constexpr int qb = decltype(qbc)::value, r = decltype(rc)::value, g4 = r / 4, e = r % 4;
            if constexpr (e == 0) {
                const int qo = 32 * qb + 8 * g4 + 4 * half;  // first of 4 consecutive queries of the tile
                const unsigned char* mp = mbase + (buf * 4 * KT + qo) * 4;
                L4 = *(const float4*)(mp);
                D4 = *(const float4*)(mp + KT * 4);
                if constexpr (GATED) T4 = *(const float4*)(mp + 2 * KT * 4);
            }
            const float l2 = e == 0 ? L4.x : e == 1 ? L4.y : e == 2 ? L4.z : L4.w;
            const float Di = e == 0 ? D4.x : e == 1 ? D4.y : e == 2 ? D4.z : D4.w;
            float gate = 1.0f;
            if constexpr (GATED) gate = clip01(uj - (e == 0 ? T4.x : e == 1 ? T4.y : e == 2 ? T4.z : T4.w));
            const float qk = sacc[r], dov = dacc[r];
            float arg = GK ? fmaf(qk, gate * c2, -l2) : fmaf(qk, c2, -l2);
            if constexpr (CHECK) {
                const bool valid = (unsigned)(rel0 + (32 * qb + 8 * g4 + e)) <= span;
                arg = valid ? arg : -INFINITY;  // p = 0, and with it dS
            }
            const float p = __builtin_amdgcn_exp2f(arg);
            const float pvv = GV ? p * gate : p;
            const float tt = GV ? fmaf(gate, dov, -Di) : dov - Di;
            const float ds = GK ? pvv * tt : p * tt;
            if constexpr ((r & 1) == 0) {
                hold_p = pvv;
                hold_s = ds;
            } else {
                pb[r >> 3][(r & 7) >> 1] = pack_bf16x2(hold_p, pvv);
                dsb[r >> 3][(r & 7) >> 1] = pack_bf16x2(hold_s, ds);
            }
        };
        static_for<0, NS>([&](auto mc) {  // run 1
            constexpr int m = decltype(mc)::value;
            const bf16x8 cur = ring[m % DEPTH];
            if constexpr (m & 1) d0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, vreg[m / 2], m < 2 ? zero : d0, 0, 0, 0);
            else s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, kreg[m / 2], m < 2 ? zero : s0, 0, 0, 0);
            refill(mc);
            __builtin_amdgcn_sched_barrier(0);
        });
        static_for<0, NS>([&](auto mc) {  // run 2
            constexpr int m = decltype(mc)::value;
            const bf16x8 cur = ring[(NS + m) % DEPTH];
            if constexpr (m & 1) d1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, vreg[m / 2], m < 2 ? zero : d1, 0, 0, 0);
            else s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, kreg[m / 2], m < 2 ? zero : s1, 0, 0, 0);
            refill(std::integral_constant<int, NS + m>{});
            static_for<0, EPM>([&](auto ec) {
                element(std::integral_constant<int, 0>{}, std::integral_constant<int, m * EPM + decltype(ec)::value>{}, s0, d0, pb0, dsb0);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        static_for<0, NS>([&](auto mc) {  // run 3
            constexpr int m = decltype(mc)::value, i2 = m / 2, x = i2 % DB;
            const bf16x8 cur = ring[(2 * NS + m) % DEPTH];
            if constexpr (m & 1) acc_k[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, __builtin_bit_cast(bf16x8, dsb0[i2 / DB]), acc_k[x], 0, 0, 0);
            else acc_v[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, __builtin_bit_cast(bf16x8, pb0[i2 / DB]), acc_v[x], 0, 0, 0);
            refill(std::integral_constant<int, 2 * NS + m>{});
            static_for<0, EPM>([&](auto ec) {
                element(std::integral_constant<int, 1>{}, std::integral_constant<int, m * EPM + decltype(ec)::value>{}, s1, d1, pb1, dsb1);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        static_for<0, NS>([&](auto mc) {  // run 4
            constexpr int m = decltype(mc)::value, i2 = m / 2, x = i2 % DB;
            const bf16x8 cur = ring[(3 * NS + m) % DEPTH];
            if constexpr (m & 1) acc_k[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, __builtin_bit_cast(bf16x8, dsb1[i2 / DB]), acc_k[x], 0, 0, 0);
            else acc_v[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, __builtin_bit_cast(bf16x8, pb1[i2 / DB]), acc_v[x], 0, 0, 0);
            refill(std::integral_constant<int, 3 * NS + m>{});
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto step = [&](auto gated_c, auto buf_c, int t) {
        constexpr int buf = decltype(buf_c)::value;
        const int i_first = blo + t * KT;
        // the dK / dV accumulators stay in the accumulation registers: only MFMAs touch them until the end
#pragma unroll
        for (int x = 0; x < DB; x++) asm volatile("" : "+a"(acc_k[x]), "+a"(acc_v[x]));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // tile t landed (rows and per-query values); everybody is done with tile t-1
        if (t + 1 < ntiles) {
            issue_meta(buf ^ 1, i_first + KT);
            issue(buf ^ 1, i_first + KT);
        }
        if (i_first <= whi && i_first + KT - 1 >= wlo) {  // some key of this wave is attended from this tile
            const bool full = i_first >= wfull_lo && i_first + KT - 1 <= wfull_hi;
            if (full) tile(gated_c, std::false_type{}, buf_c, i_first);
            else tile(gated_c, std::true_type{}, buf_c, i_first);
        }
    };
    auto tiles = [&](auto gated_c) {
        for (int t = 0; t < ntiles; t += 2) {
            step(gated_c, std::integral_constant<int, 0>{}, t);
            if (t + 1 < ntiles) step(gated_c, std::integral_constant<int, 1>{}, t + 1);
        }
    };
    if (selected_kind && MODE != 2) tiles(std::true_type{});
    else tiles(std::false_type{});
    // A key that is never selected gets all of its gradient here: round and store it.  The other keys' two parts
    // (window block, selected block) go to fp32 buffers and are added by the merge kernel.
    if (kreal) {
        const bool final_here = !selected_kind && eslot[(size_t)row * n + j] < 0;
        const size_t ro = selected_kind ? ((size_t)bh * n + kidx) * D : ((size_t)bh * n + j) * D;
        const size_t fo = (size_t)(qo + j) * D;
        if (final_here) {
#pragma unroll
            for (int x = 0; x < DB; x++)
#pragma unroll
                for (int g4 = 0; g4 < 4; g4++) {
                    const int dcol = 32 * x + 8 * g4 + 4 * half;
                    uint2 ok, ov;
                    ok.x = pack_bf16x2(scale * acc_k[x][4 * g4], scale * acc_k[x][4 * g4 + 1]);
                    ok.y = pack_bf16x2(scale * acc_k[x][4 * g4 + 2], scale * acc_k[x][4 * g4 + 3]);
                    ov.x = pack_bf16x2(acc_v[x][4 * g4], acc_v[x][4 * g4 + 1]);
                    ov.y = pack_bf16x2(acc_v[x][4 * g4 + 2], acc_v[x][4 * g4 + 3]);
                    *(uint2*)(dk + fo + dcol) = ok;
                    *(uint2*)(dv + fo + dcol) = ov;
                }
        } else {
            float* pk = (selected_kind ? sk32 : dk32) + ro;
            float* pv = (selected_kind ? sv32 : dv32) + ro;
#pragma unroll
            for (int x = 0; x < DB; x++)
#pragma unroll
                for (int g4 = 0; g4 < 4; g4++) {
                    const int dcol = 32 * x + 8 * g4 + 4 * half;
                    *(float4*)(pk + dcol) = make_float4(scale * acc_k[x][4 * g4], scale * acc_k[x][4 * g4 + 1],
                                                        scale * acc_k[x][4 * g4 + 2], scale * acc_k[x][4 * g4 + 3]);
                    *(float4*)(pv + dcol) = make_float4(acc_v[x][4 * g4], acc_v[x][4 * g4 + 1], acc_v[x][4 * g4 + 2], acc_v[x][4 * g4 + 3]);
                }
        }
    }
}

// For every ever-selected key (list slot e, position j): dk_j = dk32_j + sk32_e rounded to bf16; same for dv.
__global__ __launch_bounds__(256) void abwd_merge_kernel(const float* __restrict__ dk32, const float* __restrict__ dv32,
                                                         const float* __restrict__ sk32, const float* __restrict__ sv32,
                                                         const int32_t* __restrict__ elist, const int32_t* __restrict__ ecount,
                                                         int H, int Gu, int n, int d4, uint16_t* __restrict__ dk,
                                                         uint16_t* __restrict__ dv, int q_begin, int q_rows)
{
    const int bh = blockIdx.y;
    const ptrdiff_t qo = q_rows ? (ptrdiff_t)bh * q_rows - q_begin : (ptrdiff_t)bh * n;  // rows of dk, dv
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const size_t total = (size_t)ecount[row] * d4;  // float4 units of this head's list
    for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < total; x += (size_t)gridDim.x * 256) {
        const int e = (int)(x / d4), c4 = (int)(x % d4);
        const int j = elist[(size_t)row * n + e];
        const size_t src = ((size_t)bh * n + j) * d4 + c4, s2 = ((size_t)bh * n + e) * d4 + c4;
        float4 a = ((const float4*)dk32)[src], c = ((const float4*)dv32)[src];
        const float4 a2 = ((const float4*)sk32)[s2], c2 = ((const float4*)sv32)[s2];
        a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
        c.x += c2.x; c.y += c2.y; c.z += c2.z; c.w += c2.w;
        ushort4 oa, oc;
        oa.x = f32_to_bf16(a.x); oa.y = f32_to_bf16(a.y); oa.z = f32_to_bf16(a.z); oa.w = f32_to_bf16(a.w);
        oc.x = f32_to_bf16(c.x); oc.y = f32_to_bf16(c.y); oc.z = f32_to_bf16(c.z); oc.w = f32_to_bf16(c.w);
        const size_t dst = (size_t)(qo + j) * d4 + c4;
        ((ushort4*)dk)[dst] = oa;
        ((ushort4*)dv)[dst] = oc;
    }
}

template <int D>
static void launch_dkv_mfma(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                            const float* tau, const int32_t* death, const int32_t* elist, const int32_t* ecount,
                            const float* lse, const void* dO, const float* delta, float* dk32, float* dv32,
                            float* sk32, float* sv32, const int32_t* eslot, void* dk, void* dv, int nb, hipStream_t st,
                            int q_begin, int q_rows)
{
    dim3 grid(c.B * c.H, 2 * nb);  // per head: (up to) nb blocks of selected keys, then the nb window blocks
#define SPK_LAUNCH_KV(MODE)                                                                                         \
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, MODE>), grid, dim3(256), 0, st, (const uint16_t*)q, (const uint16_t*)k, \
                       (const uint16_t*)v, u, tau, death, elist, ecount, lse, (const uint16_t*)dO, delta, dk32, dv32,  \
                       sk32, sv32, eslot, (uint16_t*)dk, (uint16_t*)dv, c.H, c.Gu, c.n, c.w, c.softmax_scale, nb, q_begin, \
                       q_rows)
    if (c.gate_mode == 0) SPK_LAUNCH_KV(0);
    else if (c.gate_mode == 1) SPK_LAUNCH_KV(1);
    else SPK_LAUNCH_KV(2);
#undef SPK_LAUNCH_KV
}

int launch_attn_bwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, const void* o, const float* lse, const void* dO, void* dq,
                    void* dk, void* dv, void* ws, hipStream_t st, int q_begin, const int32_t* first_valid, int q_rows)
{
    const AbwdWs W = abwd_ws(c);
    char* base = (char*)ws;
    const int nb = (c.n + QB - 1) / QB;
    const size_t BH = (size_t)c.B * c.H, rows = BH * (q_rows ? q_rows : c.n), nelem = rows * c.d;
    int32_t* lists = (int32_t*)(base + W.lists);
    int32_t* counts = (int32_t*)(base + W.counts);
    float* delta = (float*)(base + W.delta);
    float* lse2 = (float*)(base + W.lse2);
    float* dk32 = (float*)(base + W.dk32);
    float* dv32 = (float*)(base + W.dv32);
    // (the dK/dV kernel puts 2 * nb key blocks on the grid's y axis)
    const bool mfma = c.dtype == SPARSEK_BF16 && (c.d == 64 || c.d == 128) && (uint64_t)c.n * c.d * 2 <= 0xFFFFFFFFull &&
                      2 * nb <= 65535;
    if (!mfma && (q_begin != 0 || first_valid || q_rows != 0)) return SPARSEK_ERR_UNSUPPORTED;
    if (q_begin % 128 != 0) return SPARSEK_ERR_INVALID_ARG;
    if (!mfma)  // the generic kernel accumulates dk, dv with atomics
        hipLaunchKernelGGL(abwd_zero_kernel, dim3(2048), dim3(256), 0, st, (uint4*)(base + W.dk32), (W.sk32 - W.dk32) / 16);
    ExtLists x{nullptr, nullptr, nullptr, 0};
    if (mfma) {
        x.pos = (int32_t*)(base + W.xpos);
        x.death = (int32_t*)(base + W.xdeath);
        x.u = (float*)(base + W.xu);
        x.KP = (int)ext_stride(c);
    }
    launch_block_lists_ext(c, death, lists, counts, u, x, st);
    dim3 grid(nb, c.B * c.H);
    if (c.dtype == SPARSEK_F32) {
        hipLaunchKernelGGL(abwd_delta_kernel<float>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, (const float*)o,
                           (const float*)dO, rows, c.d, delta);
        hipLaunchKernelGGL(attn_bwd_generic_kernel<float>, grid, dim3(256), 0, st, (const float*)q, (const float*)k,
                           (const float*)v, u, tau, death, lists, counts, lse, (const float*)dO, delta, (float*)dq, dk32,
                           dv32, c.H, c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale, nb);
        hipLaunchKernelGGL(abwd_convert_kernel<float>, dim3(2048), dim3(256), 0, st, dk32, dv32, (float*)dk, (float*)dv,
                           nelem);
    } else {
        if (c.d == 128)
            hipLaunchKernelGGL(abwd_delta_bf16_kernel<16>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st,
                               (const uint16_t*)o, (const uint16_t*)dO, rows, delta, lse, lse2);
        else if (c.d == 64)
            hipLaunchKernelGGL(abwd_delta_bf16_kernel<8>, dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, st,
                               (const uint16_t*)o, (const uint16_t*)dO, rows, delta, lse, lse2);
        else
            hipLaunchKernelGGL(abwd_delta_kernel<uint16_t>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st,
                               (const uint16_t*)o, (const uint16_t*)dO, rows, c.d, delta);
        if (mfma) {
            int32_t* elist = (int32_t*)(base + W.elist);
            int32_t* ecount = (int32_t*)(base + W.ecount);
            int32_t* eslot = (int32_t*)(base + W.eslot);
            float* sk32 = (float*)(base + W.sk32);
            float* sv32 = (float*)(base + W.sv32);
            hipLaunchKernelGGL(abwd_elist_kernel, dim3(c.B * c.Gu), dim3(1024), 0, st, death, c.n, q_begin, elist, ecount,
                               eslot);
            if (c.d == 64) {
                launch_dq_mfma<64>(c, q, k, v, u, tau, death, x, counts, lse, dO, delta, dq, nb, st, q_begin, first_valid,
                                   q_rows);
                launch_dkv_mfma<64>(c, q, k, v, u, tau, death, elist, ecount, lse2, dO, delta, dk32, dv32, sk32, sv32, eslot,
                                    dk, dv, nb, st, q_begin, q_rows);
            } else {
                launch_dq_mfma<128>(c, q, k, v, u, tau, death, x, counts, lse, dO, delta, dq, nb, st, q_begin, first_valid,
                                    q_rows);
                launch_dkv_mfma<128>(c, q, k, v, u, tau, death, elist, ecount, lse2, dO, delta, dk32, dv32, sk32, sv32, eslot,
                                     dk, dv, nb, st, q_begin, q_rows);
            }
            const int d4 = c.d / 4;
            const int gx = (int)std::min<size_t>(((size_t)c.n * d4 + 255) / 256, 1024);
            hipLaunchKernelGGL(abwd_merge_kernel, dim3(gx, c.B * c.H), dim3(256), 0, st, dk32, dv32, sk32, sv32, elist,
                               ecount, c.H, c.Gu, c.n, d4, (uint16_t*)dk, (uint16_t*)dv, q_begin, q_rows);
        } else {
            hipLaunchKernelGGL(attn_bwd_generic_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)q,
                               (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, lse,
                               (const uint16_t*)dO, delta, (uint16_t*)dq, dk32, dv32, c.H, c.Gu, c.n, c.d, c.k, c.w,
                               c.gate_mode, c.softmax_scale, nb);
            hipLaunchKernelGGL(abwd_convert_kernel<uint16_t>, dim3(2048), dim3(256), 0, st, dk32, dv32, (uint16_t*)dk,
                               (uint16_t*)dv, nelem);
        }
    }
    return launch_status();
}

}  // namespace spk

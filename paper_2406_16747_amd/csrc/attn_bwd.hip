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
    size_t lists, counts, delta, dk32, dv32, total;
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
    W.delta = off; off += align_up(BH * c.n * 4, 256);
    W.dk32 = off; off += align_up(BH * c.n * c.d * 4, 256);
    W.dv32 = off; off += align_up(BH * c.n * c.d * 4, 256);
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
        if (lane < d) stg(dq + hb + (size_t)i * d + lane, dq0);
        if (lane + 64 < d) stg(dq + hb + (size_t)i * d + lane + 64, dq1);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    }
}

int launch_attn_bwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, const void* o, const float* lse, const void* dO, void* dq,
                    void* dk, void* dv, void* ws, hipStream_t st)
{
    const AbwdWs W = abwd_ws(c);
    char* base = (char*)ws;
    const int nb = (c.n + QB - 1) / QB;
    const size_t BH = (size_t)c.B * c.H, rows = BH * c.n, nelem = rows * c.d;
    int32_t* lists = (int32_t*)(base + W.lists);
    int32_t* counts = (int32_t*)(base + W.counts);
    float* delta = (float*)(base + W.delta);
    float* dk32 = (float*)(base + W.dk32);
    float* dv32 = (float*)(base + W.dv32);
    hipLaunchKernelGGL(abwd_zero_kernel, dim3(2048), dim3(256), 0, st, (uint4*)(base + W.dk32), (W.total - W.dk32) / 16);
    launch_block_lists(c, death, lists, counts, st);
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
        hipLaunchKernelGGL(abwd_delta_kernel<uint16_t>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st,
                           (const uint16_t*)o, (const uint16_t*)dO, rows, c.d, delta);
        hipLaunchKernelGGL(attn_bwd_generic_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)q,
                           (const uint16_t*)k, (const uint16_t*)v, u, tau, death, lists, counts, lse, (const uint16_t*)dO,
                           delta, (uint16_t*)dq, dk32, dv32, c.H, c.Gu, c.n, c.d, c.k, c.w, c.gate_mode, c.softmax_scale,
                           nb);
        hipLaunchKernelGGL(abwd_convert_kernel<uint16_t>, dim3(2048), dim3(256), 0, st, dk32, dv32, (uint16_t*)dk,
                           (uint16_t*)dv, nelem);
    }
    return launch_status();
}

}  // namespace spk

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

namespace spk {

constexpr int QB = 128;  // queries per block (shared by the list builder and the kernels)

static inline int nblocks(int n) { return (n + QB - 1) / QB; }

size_t attn_fwd_ws_bytes(const sparsek_cfg& c)
{
    size_t rows = (size_t)c.B * c.Gu;
    size_t nb = nblocks(c.n);
    size_t lists = align_up(rows * nb * (size_t)(c.k > 0 ? c.k : 1) * sizeof(int32_t), 256);
    size_t counts = align_up(rows * nb * sizeof(int32_t), 256);
    return lists + counts;
}

// ---------------------------------------------------------------------------------
// Per (row, block): ascending positions of the top-k of prefix T0 = blk*QB - w.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void block_lists_kernel(const int32_t* __restrict__ death, int n, int k,
                                                          int w, int nb, int32_t* __restrict__ lists,
                                                          int32_t* __restrict__ counts)
{
    __shared__ int wcount[4];
    __shared__ int base;
    const int blk = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int T0 = blk * QB - w;
    int32_t* lo = lists + ((size_t)row * nb + blk) * (size_t)(k > 0 ? k : 1);
    if (T0 < 0 || k == 0) {
        if (tid == 0) counts[(size_t)row * nb + blk] = 0;
        return;
    }
    const int32_t* dr = death + (size_t)row * n;
    if (tid == 0) base = 0;
    __syncthreads();
    for (int j0 = 0; j0 <= T0; j0 += 256) {
        int j = j0 + tid;
        bool p = (j <= T0) && (dr[j] > T0);
        unsigned long long ball = __ballot(p);
        if (lane == 0) wcount[wv] = __popcll(ball);
        __syncthreads();
        int off = base;
        for (int i = 0; i < wv; i++) off += wcount[i];
        if (p) {
            int o = off + __popcll(ball & ((1ull << lane) - 1ull));
            if (o < k) lo[o] = j;
        }
        __syncthreads();
        if (tid == 0) base += wcount[0] + wcount[1] + wcount[2] + wcount[3];
        __syncthreads();
    }
    if (tid == 0) counts[(size_t)row * nb + blk] = min(base, k);
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

int launch_attn_fwd(const sparsek_cfg& c, const void* q, const void* k, const void* v, const float* u,
                    const float* tau, const int32_t* death, void* o, float* lse, void* ws,
                    hipStream_t st)
{
    const int rows = c.B * c.Gu;
    const int nb = nblocks(c.n);
    int32_t* lists = (int32_t*)ws;
    int32_t* counts =
        (int32_t*)((char*)ws + align_up((size_t)rows * nb * (size_t)(c.k > 0 ? c.k : 1) * sizeof(int32_t), 256));
    hipLaunchKernelGGL(block_lists_kernel, dim3(nb, rows), dim3(256), 0, st, death, c.n, c.k, c.w, nb, lists,
                       counts);
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

// Importance scores of the key-value pairs (Sec. 3.2: scoring network with position slope;
// Sec. 3.5: score normalisation):
//     raw_t = x_t . w + t * slope                                  (t counted from 0)
//     u_t   = raw_t                                                (norm == 0)
//     u_t   = (raw_t - mean_t) / sqrt(var_t + norm_eps)            (norm == 1)
// with the running mean and population variance of raw_0 .. raw_t.
//
// scores_dot_kernel streams the hidden states once (the only traffic that matters: B*n*D elements
// against 4 bytes of output per position, roofline "hbm").  A wave owns 8 positions and walks the
// feature dimension with 16-byte loads; the scorer sits in LDS as fp64 and one read of it serves
// all 8 positions.  Products and sums are fp64 (exact products, the reduction is the only
// rounding), so the normalised scores stay accurate where early timesteps nearly cancel.
// The normalisation works on shifted scores z = raw - raw_0, which keeps E[z^2] - E[z]^2 free of
// cancellation whatever offset the scores carry: scores_partial_kernel sums z and z^2 over blocks
// of 256 positions, scores_norm_kernel adds up the blocks before its own, scans its 256 positions
// and writes u.
#include "common.hpp"

namespace spk {

constexpr int SC_POS_PER_WAVE = 8;
constexpr int SC_POS_PER_BLOCK = 4 * SC_POS_PER_WAVE;
constexpr int SC_NORM_BLOCK = 256;

template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&x)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&x)[8])
{
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, float (&x)[8])
{
    const uint4 a = *(const uint4*)p;
    const uint32_t r[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
        x[2 * i] = __uint_as_float(r[i] << 16);
        x[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void scores_dot_kernel(const T* __restrict__ x, const float* __restrict__ w,
                                                         int n, int D, double slope, double* __restrict__ raw,
                                                         float* __restrict__ u_out)
{
    // the scorer, widened once; element c sits at [c % 8][c / 8] so that the lanes of a wave,
    // which own consecutive groups of 8 features, read consecutive doubles (no bank conflicts)
    extern __shared__ double wd[];
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int D8 = D >> 3;
    for (int c = tid; c < D; c += 256) wd[(c & 7) * D8 + (c >> 3)] = (double)w[c];
    __syncthreads();
    const int t0 = blockIdx.x * SC_POS_PER_BLOCK + wv * SC_POS_PER_WAVE;
    if (t0 >= n) return;
    const T* rows[SC_POS_PER_WAVE];
#pragma unroll
    for (int p = 0; p < SC_POS_PER_WAVE; p++) rows[p] = x + ((size_t)b * n + min(t0 + p, n - 1)) * D;
    double acc[SC_POS_PER_WAVE];
#pragma unroll
    for (int p = 0; p < SC_POS_PER_WAVE; p++) acc[p] = 0.0;
    for (int c0 = 8 * lane; c0 < D; c0 += 512) {
        float xv[SC_POS_PER_WAVE][8];
#pragma unroll
        for (int p = 0; p < SC_POS_PER_WAVE; p++) load8<T>(rows[p] + c0, xv[p]);
        double wv8[8];
#pragma unroll
        for (int e = 0; e < 8; e++) wv8[e] = wd[e * D8 + (c0 >> 3)];
#pragma unroll
        for (int e = 0; e < 8; e++)
#pragma unroll
            for (int p = 0; p < SC_POS_PER_WAVE; p++) acc[p] = fma((double)xv[p][e], wv8[e], acc[p]);
    }
#pragma unroll
    for (int p = 0; p < SC_POS_PER_WAVE; p++) {
        const double s = wave_sum_f64(acc[p]);
        const int t = t0 + p;
        if (lane == 0 && t < n) {
            const double r = s + (double)t * slope;
            if (raw) raw[(size_t)b * n + t] = r;
            else u_out[(size_t)b * n + t] = (float)r;
        }
    }
}

// Inclusive prefix sums of (a, b) over the 256 threads of a workgroup, in place; tot = block totals.
__device__ __forceinline__ void block_inclusive_scan2_256(double& a, double& b, double (*wt)[4] /* [2][4] LDS */,
                                                          double& tot_a, double& tot_b)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double ya = __shfl_up(a, o, 64), yb = __shfl_up(b, o, 64);
        if (lane >= o) { a += ya; b += yb; }
    }
    if (lane == 63) { wt[0][wv] = a; wt[1][wv] = b; }
    __syncthreads();
    tot_a = 0.0; tot_b = 0.0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        if (i < wv) { a += wt[0][i]; b += wt[1][i]; }
        tot_a += wt[0][i]; tot_b += wt[1][i];
    }
}

// partial[b][blk] = (sum z, sum z^2) over the positions of block blk, z = raw - raw_0
__global__ __launch_bounds__(SC_NORM_BLOCK) void scores_partial_kernel(const double* __restrict__ raw, int n,
                                                                        double2* __restrict__ partial)
{
    __shared__ double red[2][4];
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const double* r = raw + (size_t)b * n;
    const int t = blockIdx.x * SC_NORM_BLOCK + tid;
    const double z = t < n ? r[t] - r[0] : 0.0;
    const double s1 = wave_sum_f64(z), s2 = wave_sum_f64(z * z);
    if (lane == 0) { red[0][wv] = s1; red[1][wv] = s2; }
    __syncthreads();
    if (tid == 0)
        partial[(size_t)b * gridDim.x + blockIdx.x] =
            make_double2(red[0][0] + red[0][1] + red[0][2] + red[0][3], red[1][0] + red[1][1] + red[1][2] + red[1][3]);
}

__global__ __launch_bounds__(SC_NORM_BLOCK) void scores_norm_kernel(const double* __restrict__ raw,
                                                                     const double2* __restrict__ partial, int n,
                                                                     double norm_eps, float* __restrict__ u)
{
    __shared__ double red[2][4];
    __shared__ double wt[2][4];
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const double* r = raw + (size_t)b * n;
    const int start = blockIdx.x * SC_NORM_BLOCK;
    const double shift = r[0];
    // everything before this workgroup's positions
    double s1 = 0.0, s2 = 0.0;
    for (int i = tid; i < (int)blockIdx.x; i += SC_NORM_BLOCK) {
        const double2 p = partial[(size_t)b * gridDim.x + i];
        s1 += p.x;
        s2 += p.y;
    }
    s1 = wave_sum_f64(s1);
    s2 = wave_sum_f64(s2);
    if (lane == 0) { red[0][wv] = s1; red[1][wv] = s2; }
    __syncthreads();
    const double before1 = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    const double before2 = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    const int t = start + tid;
    const double z = t < n ? r[t] - shift : 0.0;
    double c1 = z, c2 = z * z, tot1, tot2;
    block_inclusive_scan2_256(c1, c2, wt, tot1, tot2);
    if (t < n) {
        const double cnt = (double)(t + 1);
        const double mean = (before1 + c1) / cnt;
        const double var = fmax((before2 + c2) / cnt - mean * mean, 0.0);
        u[(size_t)b * n + t] = (float)((z - mean) / sqrt(var + norm_eps));
    }
}

static size_t scores_raw_bytes(int B, int n) { return align_up((size_t)B * n * sizeof(double), 256); }
size_t scores_ws_bytes(int B, int n)
{
    const size_t nblk = (n + SC_NORM_BLOCK - 1) / SC_NORM_BLOCK;
    return scores_raw_bytes(B, n) + align_up((size_t)B * nblk * sizeof(double2), 256);
}

int launch_scores(int B, int n, int D, int dtype, int norm, double slope, double norm_eps, const void* x,
                  const float* w, float* u, void* ws, hipStream_t st)
{
    double* raw = norm ? (double*)ws : nullptr;
    dim3 grid((n + SC_POS_PER_BLOCK - 1) / SC_POS_PER_BLOCK, B);
    const size_t lds = (size_t)D * sizeof(double);
    if (dtype == SPARSEK_BF16)
        hipLaunchKernelGGL(scores_dot_kernel<uint16_t>, grid, dim3(256), lds, st, (const uint16_t*)x, w, n, D, slope, raw,
                           u);
    else
        hipLaunchKernelGGL(scores_dot_kernel<float>, grid, dim3(256), lds, st, (const float*)x, w, n, D, slope, raw, u);
    if (norm) {
        double2* partial = (double2*)((char*)ws + scores_raw_bytes(B, n));
        dim3 g2((n + SC_NORM_BLOCK - 1) / SC_NORM_BLOCK, B);
        hipLaunchKernelGGL(scores_partial_kernel, g2, dim3(SC_NORM_BLOCK), 0, st, raw, n, partial);
        hipLaunchKernelGGL(scores_norm_kernel, g2, dim3(SC_NORM_BLOCK), 0, st, raw, partial, n, norm_eps, u);
    }
    return launch_status();
}

}  // namespace spk

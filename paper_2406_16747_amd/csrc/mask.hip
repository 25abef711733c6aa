// Stages 1+2: SPARSEK thresholds tau_t for every causal prefix and per-key lifetimes.
//
// The paper evaluates the prefixes one after another with two heaps on the CPU
// (Sec. 3.3, incremental algorithm; App. B.3).  Here the sequence is cut into chunks of
// CHUNK prefixes that are solved independently, one workgroup each:
//   * tau_t and the k-th largest score theta_t never decrease once the prefix holds k
//     entries (Sec. 3.2, irreversibility), so for a chunk starting at t0 only the scores
//     above a lower bound lo <= tau_{t0-1} can matter; a first kernel finds such a bound
//     at coarse boundaries, the chunk kernel compacts those candidates into LDS;
//   * inside a chunk every wave owns a few consecutive prefixes.  tau_t is the root of
//     f_t(x) = sum clip(z - x, 0, 1) = k, found by repeating the closed form of the
//     solution equation (tau from u*, w* and the fractional sum) until the pair (u*, w*)
//     reproduces itself -- exact, not an iteration to a tolerance; a bracket guards it.
//     Sums are fp64.  theta_t follows by "newcomer in, smallest out";
//   * death[j] is the first t with sel_key(j) < theta_t: a binary search in the chunk.
#include "common.hpp"

namespace spk {

constexpr int CHUNK = 128;        // prefixes per workgroup of the chunk kernel
constexpr int NT_CHUNK = 512;     // threads of the chunk kernel (8 waves, 16 prefixes each)
constexpr int NW_CHUNK = NT_CHUNK / 64;
constexpr int TPW = CHUNK / NW_CHUNK;
constexpr int SUPER = 2048;       // spacing of the coarse lower bounds
constexpr int CAP = 8192;         // candidate capacity in LDS (scores + positions: 64 KB)
constexpr int NT_COARSE = 1024;
constexpr int NPROBE = 15;
constexpr int NPASS = 3;
constexpr int MAX_ITERS = 4096;

size_t mask_ws_bytes(const sparsek_cfg& c)
{
    size_t rows = (size_t)c.B * c.Gu;
    size_t nsuper = ((size_t)c.n + SUPER - 1) / SUPER;
    return align_up(rows * nsuper * sizeof(float), 256) + 256;
}

// ---------------------------------------------------------------------------------
// Prefixes with at most k entries: tau_t = min(u[0..t]) - 1.  k == 0: tau_t = max, death = j.
// One workgroup per row; a three-phase scan over `upto` entries.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void mask_short_prefix_kernel(const float* __restrict__ u,
                                                                  float* __restrict__ tau,
                                                                  int32_t* __restrict__ death, int n,
                                                                  int k)
{
    __shared__ float part[1024];
    const int row = blockIdx.x;
    const float* ur = u + (size_t)row * n;
    float* tr = tau + (size_t)row * n;
    const bool use_max = (k == 0);
    const int upto = use_max ? n : (k < n ? k : n);
    const int per = (upto + 1023) / 1024;
    const int b = threadIdx.x * per;
    const int e = min(b + per, upto);
    float acc = use_max ? -INFINITY : INFINITY;
    for (int i = b; i < e; i++) acc = use_max ? fmaxf(acc, ur[i]) : fminf(acc, ur[i]);
    part[threadIdx.x] = acc;
    __syncthreads();
    float run = use_max ? -INFINITY : INFINITY;
    for (int i = 0; i < (int)threadIdx.x; i++) run = use_max ? fmaxf(run, part[i]) : fminf(run, part[i]);
    for (int i = b; i < e; i++) {
        run = use_max ? fmaxf(run, ur[i]) : fminf(run, ur[i]);
        tr[i] = use_max ? run : run - 1.0f;
    }
    if (use_max) {
        int32_t* dr = death + (size_t)row * n;
        for (int i = threadIdx.x; i < n; i += 1024) dr[i] = i;
    }
}

// ---------------------------------------------------------------------------------
// Coarse lower bounds.  Block (s, row) looks at the prefix of length L = s*SUPER and, if
// L >= k, narrows a bracket around the root of f_L(x) = k with NPASS passes of NPROBE probes;
// lo_out = a point with f(lo) >= k + 1/4 (so lo <= tau of that prefix despite fp32 partial
// sums).  It also presets death[] = n on its slice.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(NT_COARSE) void mask_coarse_kernel(const float* __restrict__ u,
                                                                 float* __restrict__ lo_out,
                                                                 int32_t* __restrict__ death, int n,
                                                                 int k, int nsuper)
{
    __shared__ double red[NT_COARSE / 64][NPROBE + 1];
    __shared__ float bracket[2];
    const int s = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float* ur = u + (size_t)row * n;
    int32_t* dr = death + (size_t)row * n;
    for (int i = s * SUPER + tid; i < min(n, (s + 1) * SUPER); i += NT_COARSE) dr[i] = n;
    const int L = s * SUPER;
    float* out = lo_out + (size_t)row * nsuper + s;
    if (L < k || L == 0) {
        if (tid == 0) *out = -INFINITY;
        return;
    }
    // pass 0: range of the prefix
    float mn = INFINITY, mx = -INFINITY;
    for (int i = tid; i < L; i += NT_COARSE) {
        float z = ur[i];
        mn = fminf(mn, z);
        mx = fmaxf(mx, z);
    }
    mn = wave_min_f32(mn);
    mx = wave_max_f32(mx);
    if (lane == 0) { red[wv][0] = mn; red[wv][1] = mx; }
    __syncthreads();
    if (tid == 0) {
        float a = INFINITY, b = -INFINITY;
        for (int i = 0; i < NT_COARSE / 64; i++) { a = fminf(a, (float)red[i][0]); b = fmaxf(b, (float)red[i][1]); }
        bracket[0] = a - 1.0f;  // f = L >= k here
        bracket[1] = b;         // f = 0 < k here
    }
    __syncthreads();
    for (int pass = 0; pass < NPASS; pass++) {
        const float lo = bracket[0], hi = bracket[1];
        const float step = (hi - lo) / (float)(NPROBE + 1);
        float acc[NPROBE];
#pragma unroll
        for (int p = 0; p < NPROBE; p++) acc[p] = 0.0f;
        for (int i = tid; i < L; i += NT_COARSE) {
            float z = ur[i];
#pragma unroll
            for (int p = 0; p < NPROBE; p++) acc[p] += clip01(z - (lo + step * (float)(p + 1)));
        }
#pragma unroll
        for (int p = 0; p < NPROBE; p++) {
            double t = wave_sum_f64((double)acc[p]);
            if (lane == 0) red[wv][p] = t;
        }
        __syncthreads();
        if (tid == 0) {
            float nlo = lo, nhi = hi;
            for (int p = 0; p < NPROBE; p++) {
                double f = 0.0;
                for (int i = 0; i < NT_COARSE / 64; i++) f += red[i][p];
                float x = lo + step * (float)(p + 1);
                if (f >= (double)k + 0.25) nlo = x;
                else { nhi = x; break; }
            }
            bracket[0] = nlo;
            bracket[1] = nhi;
        }
        __syncthreads();
    }
    if (tid == 0) *out = bracket[0];
}

// ---------------------------------------------------------------------------------
// Candidate lists: compacted in LDS, or (overflow fallback) the raw prefix in global memory.
// ---------------------------------------------------------------------------------
struct ListLds {
    const float* v;
    const int* idx;
    int M;
    __device__ __forceinline__ float val(int i) const { return v[i]; }
    __device__ __forceinline__ int pos(int i) const { return idx[i]; }
};
struct ListGlobal {
    const float* u;
    int M;
    __device__ __forceinline__ float val(int i) const { return u[i]; }
    __device__ __forceinline__ int pos(int i) const { return i; }
};

// Right-limit counts of the piece of f_t that starts at x: F = #{z > x+1}, S = #{z > x},
// fsum = sum of the z in (x, x+1], minF = min{z > x+1}; over list entries at positions <= t.
template <class List>
__device__ __forceinline__ void eval_piece(const List& L, int t, double x, int lane, int& F, int& S,
                                           double& fsum, float& minF)
{
    int f = 0, s = 0;
    double sum = 0.0;
    float mf = INFINITY;
    const double x1 = x + 1.0;
    for (int i = lane; i < L.M; i += 64) {
        float v = L.val(i);
        if (L.pos(i) <= t) {
            double dv = (double)v;
            if (dv > x) {
                s++;
                if (dv > x1) { f++; mf = fminf(mf, v); }
                else sum += dv;
            }
        }
    }
    unsigned long long packed = wave_sum_u64(((unsigned long long)f << 32) | (unsigned long long)s);
    F = (int)(packed >> 32);
    S = (int)(packed & 0xFFFFFFFFull);
    fsum = wave_sum_f64(sum);
    minF = wave_min_f32(mf);
}

// tau of prefix t (t+1 > k >= 1) starting from a point `start` with f_t(start) >= k.
// Repeats tau <- (fsum + F - k)/(S - F) (solution equation of Sec. 3.3 with u* = F, w* = S)
// until (F, S) at the new point equal those it was computed from; then that point is the
// exact root of its linear piece.  Overshoots fall back to bisection of the bracket.
template <class List>
__device__ double solve_tau(const List& L, int t, int k, double start, int lane, int* status)
{
    double lo_b = start, hi_b = INFINITY, x = start;
    int pF = -1, pS = -1;
    for (int it = 0; it < MAX_ITERS; it++) {
        int F, S;
        double fsum;
        float minF;
        eval_piece(L, t, x, lane, F, S, fsum, minF);
        if (F == pF && S == pS) return x;
        const double f = (double)F + fsum - (double)(S - F) * x;
        if (f < (double)k) {  // overshoot: x is right of the root
            hi_b = x;
            pF = pS = -1;
            double mid = 0.5 * (lo_b + hi_b);
            if (!(mid > lo_b && mid < hi_b)) return lo_b;
            x = mid;
            continue;
        }
        lo_b = x;
        if (S == F) {  // flat to the right of x, f == F there
            if (F == k) return (double)minF - 1.0;  // sup of the level set f == k
            x = (double)minF - 1.0;                  // F > k: next breakpoint
            pF = pS = -1;
            continue;
        }
        const double xn = (fsum + (double)F - (double)k) / (double)(S - F);
        if (!(xn > x)) return x;  // f(x) == k up to rounding
        if (xn >= hi_b) {
            pF = pS = -1;
            double mid = 0.5 * (lo_b + hi_b);
            if (!(mid > lo_b && mid < hi_b)) return lo_b;
            x = mid;
            continue;
        }
        pF = F;
        pS = S;
        x = xn;
    }
    if (lane == 0) atomicOr(status, 1);
    return x;
}

// k-th largest selection key among list entries at positions < tlim (at least k of them
// exist).  MSB-first radix select, 8 bits a round, one 256-bin LDS histogram per wave.
template <class List>
__device__ unsigned long long kth_largest(const List& L, int tlim, int k, int lane, unsigned* hist)
{
    unsigned long long prefix = 0;  // decided high bits
    int r = k;                      // rank wanted among the entries matching the prefix
    for (int round = 0; round < 8; round++) {
        const int shift = 56 - 8 * round;
        for (int b = lane; b < 256; b += 64) hist[b] = 0;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        for (int i = lane; i < L.M; i += 64) {
            int p = L.pos(i);
            if (p < tlim) {
                unsigned long long key = sel_key(L.val(i), p);
                bool match = (round == 0) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
                if (match) atomicAdd(&hist[(unsigned)(key >> shift) & 255u], 1u);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        // lane l owns bins 4l..4l+3; suffix sums from the top bin down
        unsigned h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2],
                 h3 = hist[4 * lane + 3];
        unsigned lsum = h0 + h1 + h2 + h3;
        unsigned suf = lsum;  // inclusive suffix sum over lanes >= this one
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            unsigned y = __shfl_down(suf, o, 64);
            if (lane + o < 64) suf += y;
        }
        unsigned long long ball = __ballot(suf >= (unsigned)r);
        if (ball == 0) return 0;  // fewer than k entries: caller's precondition broken
        int ls = 63 - __builtin_clzll(ball);  // highest lane whose suffix reaches r
        unsigned above = __shfl(suf - lsum, ls, 64);  // entries in bins above that lane
        unsigned b3 = __shfl(h3, ls, 64), b2 = __shfl(h2, ls, 64), b1 = __shfl(h1, ls, 64),
                 b0 = __shfl(h0, ls, 64);
        int digit;
        unsigned cnt;
        if (above + b3 >= (unsigned)r) { digit = 4 * ls + 3; cnt = b3; }
        else if (above + b3 + b2 >= (unsigned)r) { digit = 4 * ls + 2; above += b3; cnt = b2; }
        else if (above + b3 + b2 + b1 >= (unsigned)r) { digit = 4 * ls + 1; above += b3 + b2; cnt = b1; }
        else { digit = 4 * ls; above += b3 + b2 + b1; cnt = b0; }
        r -= (int)above;
        prefix |= (unsigned long long)digit << shift;
        if (cnt == 1 && shift > 0) {  // a single entry carries this prefix: fetch it
            unsigned long long best = 0;
            for (int i = lane; i < L.M; i += 64) {
                int p = L.pos(i);
                if (p < tlim) {
                    unsigned long long key = sel_key(L.val(i), p);
                    if ((key >> shift) == (prefix >> shift)) best = key;
                }
            }
            return wave_max_u64(best);
        }
    }
    return prefix;
}

// Smallest key strictly above `theta` among entries at positions < tlim (all-ones if none).
template <class List>
__device__ __forceinline__ unsigned long long succ_key(const List& L, int tlim, unsigned long long theta,
                                                        int lane)
{
    unsigned long long best = ~0ull;
    for (int i = lane; i < L.M; i += 64) {
        int p = L.pos(i);
        if (p < tlim) {
            unsigned long long key = sel_key(L.val(i), p);
            if (key > theta && key < best) best = key;
        }
    }
    return wave_min_u64(best);
}

template <class List>
__device__ __forceinline__ unsigned long long min_key(const List& L, int tlim, int lane)
{
    unsigned long long best = ~0ull;
    for (int i = lane; i < L.M; i += 64) {
        int p = L.pos(i);
        if (p < tlim) {
            unsigned long long key = sel_key(L.val(i), p);
            if (key < best) best = key;
        }
    }
    return wave_min_u64(best);
}

// One wave, prefixes [ta, tb): writes tau (for t >= k) and theta keys into th[t - t0].
template <class List>
__device__ void wave_prefixes(const List& L, const float* __restrict__ ur, float* __restrict__ tr,
                              int t0, int ta, int tb, int k, float lo, int lane, unsigned* hist,
                              unsigned long long* th, unsigned long long* th_start, int* status)
{
    // ---- tau ----
    bool have_prev = false;
    double tau_prev = 0.0;
    for (int t = ta; t < tb; t++) {
        if (t + 1 <= k) continue;  // written by the short-prefix kernel
        const double ut = (double)ur[t];
        double tau;
        if (have_prev && !(ut > tau_prev)) {
            tau = tau_prev;  // the new score is below the threshold: nothing changes
        } else {
            double start;
            if (have_prev) start = tau_prev;
            else if (lo > -INFINITY) start = (double)lo;
            else {  // no bound yet: min(prefix) - 1 has f = t+1 >= k
                float mn = INFINITY;
                for (int i = lane; i < L.M; i += 64)
                    if (L.pos(i) <= t) mn = fminf(mn, L.val(i));
                start = (double)wave_min_f32(mn) - 1.0;
            }
            tau = solve_tau(L, t, k, start, lane, status);
        }
        tau_prev = tau;
        have_prev = true;
        if (lane == 0) tr[t] = (float)tau;
    }
    // ---- theta: k-th largest selection key of each prefix (0 while the prefix is shorter than k) ----
    unsigned long long theta = 0;
    if (ta >= k) theta = kth_largest(L, ta, k, lane, hist);
    if (ta == t0 && lane == 0) *th_start = theta;
    for (int t = ta; t < tb; t++) {
        const int len = t + 1;
        if (len == k) {
            theta = min_key(L, t + 1, lane);
        } else if (len > k) {
            unsigned long long e = sel_key(ur[t], t);
            if (e > theta) {
                unsigned long long sc = succ_key(L, t, theta, lane);
                theta = e < sc ? e : sc;
            }
        }
        if (lane == 0) th[t - t0] = theta;
    }
}

// death of one list entry given the chunk's theta sequence (non-decreasing).
__device__ __forceinline__ void write_death(float v, int j, int t0, int t1, int k,
                                            const unsigned long long* th, unsigned long long th_start,
                                            int32_t* __restrict__ dr)
{
    const unsigned long long key = sel_key(v, j);
    int first;
    if (j < t0) {
        if (t0 >= k && key < th_start) return;  // already out before this chunk
        first = t0;
    } else {
        first = j;
    }
    // first t in [first, t1) with th[t - t0] > key
    int a = first - t0, b = t1 - t0;  // answer in [a, b]
    while (a < b) {
        int m = (a + b) >> 1;
        if (th[m] > key) b = m;
        else a = m + 1;
    }
    if (a < t1 - t0) dr[j] = t0 + a;
}

__global__ __launch_bounds__(NT_CHUNK) void mask_chunk_kernel(const float* __restrict__ u,
                                                               const float* __restrict__ lo_in,
                                                               float* __restrict__ tau,
                                                               int32_t* __restrict__ death, int n, int k,
                                                               int nsuper, int* __restrict__ status)
{
    __shared__ float cand_val[CAP];
    __shared__ int cand_idx[CAP];
    __shared__ unsigned long long th[CHUNK];
    __shared__ unsigned hist[NW_CHUNK][256];
    __shared__ int wcount[NW_CHUNK + 1];
    __shared__ unsigned long long th_start;

    const int c = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int t0 = c * CHUNK, t1 = min(n, t0 + CHUNK);
    if (t1 <= k) return;  // no prefix here is longer than k: tau is written elsewhere, nothing dies
    const float* ur = u + (size_t)row * n;
    float* tr = tau + (size_t)row * n;
    int32_t* dr = death + (size_t)row * n;
    const float lo = lo_in[(size_t)row * nsuper + t0 / SUPER];

    // ---- ordered compaction of {j < t0 : u_j > lo}: each wave owns a contiguous slice ----
    const int per = ((t0 + NW_CHUNK - 1) / NW_CHUNK + 63) / 64 * 64;
    const int sb = min(t0, wv * per), se = min(t0, sb + per);
    const int iters = (se - sb + 63) / 64;
    int cnt = 0;
    for (int it = 0; it < iters; it++) {
        const int i = sb + it * 64 + lane;
        bool p = (i < se) && (ur[i] > lo);
        cnt += __popcll(__ballot(p));
    }
    if (lane == 0) wcount[wv] = cnt;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int i = 0; i < NW_CHUNK; i++) { int x = wcount[i]; wcount[i] = run; run += x; }
        wcount[NW_CHUNK] = run;
    }
    __syncthreads();
    const int m_old = wcount[NW_CHUNK];
    const bool fits = (m_old + (t1 - t0) <= CAP);
    if (fits) {
        int off = wcount[wv];
        for (int it = 0; it < iters; it++) {
            const int i = sb + it * 64 + lane;
            float v = (i < se) ? ur[i] : 0.0f;
            bool p = (i < se) && (v > lo);
            unsigned long long ball = __ballot(p);
            if (p) {
                int o = off + __popcll(ball & ((1ull << lane) - 1ull));
                cand_val[o] = v;
                cand_idx[o] = i;
            }
            off += __popcll(ball);
        }
        for (int i = tid; i < t1 - t0; i += NT_CHUNK) {
            cand_val[m_old + i] = ur[t0 + i];
            cand_idx[m_old + i] = t0 + i;
        }
    }
    __syncthreads();

    const int ta = min(t1, t0 + wv * TPW), tb = min(t1, ta + TPW);
    if (fits) {
        ListLds L{cand_val, cand_idx, m_old + (t1 - t0)};
        wave_prefixes(L, ur, tr, t0, ta, tb, k, lo, lane, hist[wv], th, &th_start, status);
    } else {
        ListGlobal L{ur, t1};
        wave_prefixes(L, ur, tr, t0, ta, tb, k, -INFINITY, lane, hist[wv], th, &th_start, status);
    }
    __syncthreads();
    const unsigned long long ths = th_start;
    if (fits) {
        const int M = m_old + (t1 - t0);
        for (int i = tid; i < M; i += NT_CHUNK) write_death(cand_val[i], cand_idx[i], t0, t1, k, th, ths, dr);
    } else {
        for (int i = tid; i < t1; i += NT_CHUNK) write_death(ur[i], i, t0, t1, k, th, ths, dr);
    }
}

// ---------------------------------------------------------------------------------
// Explicit top-k lists (verification aid): one workgroup per (prefix, row).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void materialize_kernel(const float* __restrict__ u,
                                                          const float* __restrict__ tau,
                                                          const int32_t* __restrict__ death, int n, int k,
                                                          int t_begin, int nt, int32_t* __restrict__ idx,
                                                          float* __restrict__ gate)
{
    __shared__ int wcount[4];
    __shared__ int base;
    const int t = t_begin + blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float* ur = u + (size_t)row * n;
    const int32_t* dr = death + (size_t)row * n;
    const float tt = tau[(size_t)row * n + t];
    int32_t* io = idx + ((size_t)row * nt + blockIdx.x) * k;
    float* go = gate ? gate + ((size_t)row * nt + blockIdx.x) * k : nullptr;
    if (tid == 0) base = 0;
    __syncthreads();
    for (int j0 = 0; j0 <= t; j0 += 256) {
        int j = j0 + tid;
        bool p = (j <= t) && (dr[j] > t);
        unsigned long long ball = __ballot(p);
        if (lane == 0) wcount[wv] = __popcll(ball);
        __syncthreads();
        int off = base;
        for (int i = 0; i < wv; i++) off += wcount[i];
        if (p) {
            int o = off + __popcll(ball & ((1ull << lane) - 1ull));
            if (o < k) {
                io[o] = j;
                if (go) go[o] = clip01(ur[j] - tt);
            }
        }
        __syncthreads();
        if (tid == 0) base += wcount[0] + wcount[1] + wcount[2] + wcount[3];
        __syncthreads();
    }
    for (int o = base + tid; o < k; o += 256) {
        io[o] = -1;
        if (go) go[o] = 0.0f;
    }
}

int launch_mask(const sparsek_cfg& c, const float* u, float* tau, int32_t* death, void* ws,
                hipStream_t st)
{
    const int rows = c.B * c.Gu;
    const int nsuper = (c.n + SUPER - 1) / SUPER;
    float* lo = (float*)ws;
    int* status = (int*)((char*)ws + align_up((size_t)rows * nsuper * sizeof(float), 256));
    hipLaunchKernelGGL(mask_short_prefix_kernel, dim3(rows), dim3(1024), 0, st, u, tau, death, c.n, c.k);
    if (c.k == 0) return launch_status();
    hipLaunchKernelGGL(mask_coarse_kernel, dim3(nsuper, rows), dim3(NT_COARSE), 0, st, u, lo, death, c.n,
                       c.k, nsuper);
    if (c.k < c.n) {
        const int nchunks = (c.n + CHUNK - 1) / CHUNK;
        hipLaunchKernelGGL(mask_chunk_kernel, dim3(nchunks, rows), dim3(NT_CHUNK), 0, st, u, lo, tau, death,
                           c.n, c.k, nsuper, status);
    }
    return launch_status();
}

int launch_materialize(const sparsek_cfg& c, const float* u, const float* tau, const int32_t* death,
                       int t_begin, int t_end, int32_t* idx, float* gate, hipStream_t st)
{
    const int rows = c.B * c.Gu;
    const int nt = t_end - t_begin;
    if (nt == 0 || c.k == 0) return SPARSEK_OK;
    hipLaunchKernelGGL(materialize_kernel, dim3(nt, rows), dim3(256), 0, st, u, tau, death, c.n, c.k,
                       t_begin, nt, idx, gate);
    return launch_status();
}

}  // namespace spk

// Stages 1+2: SPARSEK thresholds tau_t for every causal prefix and per-key lifetimes.
//
// The paper evaluates the prefixes one after another with two heaps on the CPU
// (Sec. 3.3, incremental algorithm; App. B.3).  Here the sequence is cut into chunks of
// CHUNK prefixes that are solved independently, one workgroup each:
//   * tau_t and the k-th largest score theta_t never decrease once the prefix holds k
//     entries (Sec. 3.2, irreversibility), so for a chunk starting at t0 only the scores
//     above a lower bound lo <= tau_{t0-1} can matter; a first kernel finds such a bound
//     at coarse boundaries, the chunk kernel compacts those candidates into LDS, sorts them
//     once (selection order, bitonic) and takes fp64 prefix sums of the sorted scores;
//   * inside a chunk every wave owns a few consecutive prefixes.  tau_t is the root of
//     f_t(x) = sum clip(z - x, 0, 1) = k, found by repeating the closed form of the
//     solution equation (tau from u*, w* and the fractional sum) until the pair (u*, w*)
//     reproduces itself -- exact, not an iteration to a tolerance; a bracket guards it.
//     One evaluation of (u*, w*, fractional sum) is two searches in the sorted list plus a
//     difference of prefix sums for the older scores, and a direct pass over the chunk's own
//     (at most CHUNK) scores, which enter one by one.  theta_t follows by "newcomer in,
//     smallest out" with a pointer into the sorted list;
//   * death[j] is the first t with sel_key(j) < theta_t: a binary search in the chunk.
#include "common.hpp"

namespace spk {

constexpr int CHUNK = 128;        // prefixes per workgroup of the chunk kernel
constexpr int NT_CHUNK = 1024;    // threads of the chunk kernel (16 waves, 8 prefixes each)
constexpr int NW_CHUNK = NT_CHUNK / 64;
constexpr int SUPER = 2048;       // spacing of the coarse lower bounds
constexpr int CAP = 8192;         // candidate capacity in LDS (64-bit keys: 64 KB, fp64 prefix sums: 64 KB);
                                  // CAP_SMALL halves it so that two workgroups share a compute unit
constexpr int NT_COARSE = 1024;
constexpr int NPROBE = 15;
constexpr int NPASS = 3;
constexpr int MAX_ITERS = 4096;

size_t mask_ws_bytes(const sparsek_cfg& c)
{
    size_t rows = (size_t)c.B * c.Gu;
    size_t nsuper = ((size_t)c.n + SUPER - 1) / SUPER;
    // lower bounds, the status word, one bit per 128-prefix chunk (chunks that the half-capacity kernel hands on)
    size_t nchunks = ((size_t)c.n + CHUNK - 1) / CHUNK;
    return align_up(rows * nsuper * sizeof(float), 256) + 256 + align_up((rows * nchunks + 31) / 32 * 4, 256);
}

// ---------------------------------------------------------------------------------
// Coarse kernel, grid (nsuper, rows), 1024 threads.
//  * every block presets death[] = n on its slice of SUPER positions;
//  * block s == 0 also writes the thresholds of the prefixes with at most k entries:
//    tau_t = min(u[0..t]) - 1 (k == 0: tau_t = max(u[0..t]) and death[j] = j) -- a block scan;
//  * block s >= 1 looks at the prefix of length L = s*SUPER and, if L >= k, narrows a bracket
//    around the root of f_L(x) = k with NPASS passes of NPROBE probes; lo_out = a point with
//    f(lo) >= k + 1/4 (so lo <= tau of that prefix despite fp32 partial sums).
// Scores are read once into registers (COARSE_REG per thread), in segments for very long rows.
// ---------------------------------------------------------------------------------
constexpr int COARSE_REG = 32;

__device__ void short_prefix_scan(const float* __restrict__ ur, float* __restrict__ tr, int32_t* __restrict__ dr,
                                  int n, int k, float* part /* [1024] LDS */)
{
    const int tid = threadIdx.x;
    const bool use_max = (k == 0);
    const int upto = use_max ? n : (k < n ? k : n);
    const int per = (upto + 1023) / 1024;
    const int b = tid * per, e = min(b + per, upto);
    float acc = use_max ? -INFINITY : INFINITY;
    for (int i = b; i < e; i++) acc = use_max ? fmaxf(acc, ur[i]) : fminf(acc, ur[i]);
    part[tid] = acc;
    __syncthreads();
    // inclusive Hillis-Steele scan of the 1024 partial extrema
    for (int off = 1; off < 1024; off <<= 1) {
        float other = (tid >= off) ? part[tid - off] : acc;
        __syncthreads();
        acc = use_max ? fmaxf(acc, other) : fminf(acc, other);
        part[tid] = acc;
        __syncthreads();
    }
    float run = (tid == 0) ? (use_max ? -INFINITY : INFINITY) : part[tid - 1];
    for (int i = b; i < e; i++) {
        run = use_max ? fmaxf(run, ur[i]) : fminf(run, ur[i]);
        tr[i] = use_max ? run : run - 1.0f;
    }
    if (use_max)
        for (int i = tid; i < n; i += 1024) dr[i] = i;
}

__global__ __launch_bounds__(NT_COARSE) void mask_coarse_kernel(const float* __restrict__ u,
                                                                 float* __restrict__ lo_out,
                                                                 float* __restrict__ tau,
                                                                 int32_t* __restrict__ death, int n,
                                                                 int k, int nsuper, int* __restrict__ status,
                                                                 unsigned* __restrict__ handed_on, int nwords)
{
    __shared__ double red[NT_COARSE / 64][NPROBE + 1];
    __shared__ double ftot[NPROBE];
    __shared__ float bracket[2];
    __shared__ float part[1024];
    const int s = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float* ur = u + (size_t)row * n;
    int32_t* dr = death + (size_t)row * n;
    // the call's status word starts at 0; the chunk kernel, which sets bits in it, runs after this one on the stream
    if (s == 0 && row == 0 && tid == 0) *status = 0;
    for (int i = (row * gridDim.x + s) * NT_COARSE + tid; i < nwords; i += gridDim.x * gridDim.y * NT_COARSE)
        handed_on[i] = 0u;
    if (k > 0)
        for (int i = s * SUPER + tid; i < min(n, (s + 1) * SUPER); i += NT_COARSE) dr[i] = n;
    const int L = s * SUPER;
    float* out = lo_out + (size_t)row * nsuper + s;
    if (s == 0) {
        short_prefix_scan(ur, tau + (size_t)row * n, dr, n, k, part);
        if (tid == 0) *out = -INFINITY;
        return;
    }
    if (L < k || k == 0) {
        if (tid == 0) *out = -INFINITY;
        return;
    }
    const int nseg = (L + NT_COARSE * COARSE_REG - 1) / (NT_COARSE * COARSE_REG);
    float z[COARSE_REG];
    auto load_seg = [&](int seg) {
#pragma unroll
        for (int r = 0; r < COARSE_REG; r++) {
            const int i = (seg * COARSE_REG + r) * NT_COARSE + tid;
            z[r] = (i < L) ? ur[i] : -INFINITY;  // -inf never counts in f; excluded from the min below
        }
    };
    load_seg(0);
    // pass 0: range of the prefix
    float mn = INFINITY, mx = -INFINITY;
    for (int seg = 0; seg < nseg; seg++) {
        if (nseg > 1) load_seg(seg);
#pragma unroll
        for (int r = 0; r < COARSE_REG; r++) {
            mx = fmaxf(mx, z[r]);
            mn = (z[r] > -INFINITY) ? fminf(mn, z[r]) : mn;
        }
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
        for (int seg = 0; seg < nseg; seg++) {
            if (nseg > 1) load_seg(seg);
#pragma unroll
            for (int r = 0; r < COARSE_REG; r++) {
#pragma unroll
                for (int p = 0; p < NPROBE; p++) acc[p] += clip01(z[r] - (lo + step * (float)(p + 1)));
            }
        }
#pragma unroll
        for (int p = 0; p < NPROBE; p++) {
            double t = wave_sum_f64((double)acc[p]);
            if (lane == 0) red[wv][p] = t;
        }
        __syncthreads();
        if (tid < NPROBE) {  // one thread per probe adds the 16 wave totals
            double f = 0.0;
            for (int i = 0; i < NT_COARSE / 64; i++) f += red[i][tid];
            ftot[tid] = f;
        }
        __syncthreads();
        if (tid == 0) {
            float nlo = lo, nhi = hi;
            for (int p = 0; p < NPROBE; p++) {
                float x = lo + step * (float)(p + 1);
                if (ftot[p] >= (double)k + 0.25) nlo = x;
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
// Sorted list: key[0, m_old) = selection keys (score, then older position) of the older
// candidates in descending order, pref[i] = sum of the scores of key[0, i) in fp64; the chunk's
// own scores live in registers, two per lane (entries `lane` and `lane + 64` of the chunk).
struct ListSorted {
    const unsigned long long* key;
    const double* pref;
    int m_old, t0;
    float nv0, nv1;  // this lane's chunk scores (-inf beyond the chunk)
};
__device__ __forceinline__ float key_score(unsigned long long key)
{
    return __uint_as_float(score_key_inv((uint32_t)(key >> 32)));
}
__device__ __forceinline__ int key_pos(unsigned long long key) { return (int)(0xFFFFFFFFu - (uint32_t)key); }
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

// The linear piece of f_t that contains x (right-limit counts), for the sorted list.
struct Piece {
    int F, S, a;      // a = older scores above x + 1
    double fsum;
    double next_old;  // smallest breakpoint of the older scores above x (+inf if none)
    double prev_old;  // largest breakpoint of the older scores at or below x (-inf if none)
};

// The fp64 thresholds are replaced by their round-down fp32 values: for an fp32 score v,
// v > x  <=>  v > rd(x).  The counts over the older scores are the results of two searches
// (32 probes a round; lanes 0..31 search x, lanes 32..63 search x + 1), their fractional sum is a
// difference of prefix sums, or a direct sum when at most 64 scores are fractional: a sum with a
// single fractional score has to stay exact, which the flat case (root exactly on a breakpoint,
// sup rule) relies on.  The chunk's own scores are added from registers.
__device__ __forceinline__ Piece eval_sorted(const ListSorted& L, int t, double x, int lane)
{
    const float xf = __double2float_rd(x), x1f = __double2float_rd(x + 1.0);
    const int hf = lane >> 5, l32 = lane & 31;
    const float thr = hf ? x1f : xf;
    int lo = 0, hi = L.m_old;  // the count lies in [lo, hi]: key[<lo] are above thr, key[>=hi] are not
    while (__any(lo < hi)) {
        const int stride = (hi - lo + 31) >> 5;
        const int p = lo + l32 * stride;
        const bool above = (p < hi) && (key_score(L.key[p]) > thr);
        const unsigned long long ball = __ballot(above);
        const int c = __popc(hf ? (unsigned)(ball >> 32) : (unsigned)ball);
        if (lo < hi) {
            if (c == 0) hi = lo;
            else {
                hi = min(hi, lo + c * stride);
                lo = lo + (c - 1) * stride + 1;
            }
        }
    }
    const int b = __builtin_amdgcn_readlane(lo, 0);   // older scores above x
    const int a = __builtin_amdgcn_readlane(lo, 32);  // older scores above x + 1
    Piece P;
    P.a = a;
    // neighbouring breakpoints of the older scores (uniform addresses: broadcast reads)
    P.next_old = INFINITY;
    P.prev_old = -INFINITY;
    if (b > 0) P.next_old = (double)key_score(L.key[b - 1]);
    if (a > 0) P.next_old = fmin(P.next_old, (double)key_score(L.key[a - 1]) - 1.0);
    if (b < L.m_old) P.prev_old = (double)key_score(L.key[b]);
    if (a < L.m_old) P.prev_old = fmax(P.prev_old, (double)key_score(L.key[a]) - 1.0);
    // the chunk's own scores inside prefix t
    const int nc = t - L.t0 + 1;
    const float v0 = (lane < nc) ? L.nv0 : -INFINITY, v1 = (lane + 64 < nc) ? L.nv1 : -INFINITY;
    const bool a0 = v0 > xf, b0 = v0 > x1f, a1 = v1 > xf, b1 = v1 > x1f;
    const int f = (b0 ? 1 : 0) + (b1 ? 1 : 0), sc = (a0 ? 1 : 0) + (a1 ? 1 : 0);
    double part = (double)((a0 && !b0) ? v0 : 0.0f) + (double)((a1 && !b1) ? v1 : 0.0f);
    double base = 0.0;
    if (b - a <= 64) {
        if (lane < b - a) part += (double)key_score(L.key[a + lane]);
    } else {
        base = L.pref[b] - L.pref[a];
    }
    const unsigned long long packed = wave_sum_u64(((unsigned long long)f << 32) | (unsigned long long)sc);
    P.F = a + (int)(packed >> 32);
    P.S = b + (int)(packed & 0xFFFFFFFFull);
    P.fsum = base + wave_sum_f64(part);
    return P;
}

// Smallest score above x + 1 in prefix t (the flat case needs it).
__device__ __forceinline__ float min_saturated(const ListSorted& L, int t, double x, int a, int lane)
{
    const float x1f = __double2float_rd(x + 1.0);
    const int nc = t - L.t0 + 1;
    const float v0 = (lane < nc) ? L.nv0 : -INFINITY, v1 = (lane + 64 < nc) ? L.nv1 : -INFINITY;
    float mf = fminf(v0 > x1f ? v0 : INFINITY, v1 > x1f ? v1 : INFINITY);
    if (a > 0) mf = fminf(mf, key_score(L.key[a - 1]));
    return wave_min_f32(mf);
}

// True if none of the chunk's own scores inside prefix t has a breakpoint (z or z - 1) in (lo, hi].
__device__ __forceinline__ bool own_piece_clear(const ListSorted& L, int t, double lo, double hi, int lane)
{
    const int nc = t - L.t0 + 1;
    const double v0 = (double)L.nv0, v1 = (double)L.nv1;
    const bool h0 = (lane < nc) && ((v0 > lo && v0 <= hi) || (v0 - 1.0 > lo && v0 - 1.0 <= hi));
    const bool h1 = (lane + 64 < nc) && ((v1 > lo && v1 <= hi) || (v1 - 1.0 > lo && v1 - 1.0 <= hi));
    return __ballot(h0 || h1) == 0ull;
}

// tau of prefix t (t+1 > k >= 1) starting from a point `start` with f_t(start) >= k.
// Repeats tau <- (fsum + F - k)/(S - F) (solution equation of Sec. 3.3 with u* = F, w* = S)
// until (F, S) at the new point equal those it was computed from; then that point is the
// exact root of its linear piece.  The step is the root of the linear piece through the current
// point, taken from whichever side of the root the point lies on (f_t is neither convex nor
// concave, so a one-sided iteration would creep); a bracket [lo_b, hi_b) of the root is kept and
// a step that leaves it is replaced by its midpoint.
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
        pF = pS = -1;
        const double f = (double)F + fsum - (double)(S - F) * x;
        double xn;
        bool have = false;
        if (f < (double)k) {
            hi_b = x;  // x is right of the root
            if (S > F) { xn = (fsum + (double)F - (double)k) / (double)(S - F); have = true; }
        } else {
            lo_b = x;
            if (S == F) {  // flat to the right of x, f == F there
                if (F == k) return (double)minF - 1.0;  // sup of the level set f == k
                xn = (double)minF - 1.0;                 // F > k: the next breakpoint, still left of the root
                if (xn < hi_b) { x = xn; continue; }
            } else {
                xn = (fsum + (double)F - (double)k) / (double)(S - F);
                if (!(xn > x)) return x;  // f(x) == k up to rounding
                have = true;
            }
        }
        if (have && xn > lo_b && xn < hi_b) {
            pF = F;
            pS = S;
            x = xn;
        } else {
            const double mid = 0.5 * (lo_b + hi_b);
            if (!(mid > lo_b && mid < hi_b)) return lo_b;
            x = mid;
        }
    }
    if (lane == 0) atomicOr(status, 1);
    return x;
}

// k-th largest selection key among list entries at positions < tlim (at least k of them exist;
// returns 0 otherwise).  Whole workgroup, MSB-first radix select, 8 bits a round, one 256-bin
// LDS histogram; every thread returns the same key.
template <class List>
__device__ unsigned long long block_kth_largest(const List& L, int tlim, int k, unsigned* hist, unsigned long long* bc)
{
    const int tid = threadIdx.x, lane = tid & 63;
    unsigned long long prefix = 0;  // decided high bits
    int r = k;                      // rank wanted among the entries matching the prefix
    for (int round = 0; round < 8; round++) {
        const int shift = 56 - 8 * round;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < L.M; i += NT_CHUNK) {
            const int p = L.pos(i);
            if (p < tlim) {
                const unsigned long long key = sel_key(L.val(i), p);
                const bool match = (round == 0) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
                if (match) atomicAdd(&hist[(unsigned)(key >> shift) & 255u], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {  // wave 0: lane l owns bins 4l..4l+3; suffix sums from the top bin down
            const unsigned h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
            const unsigned lsum = h0 + h1 + h2 + h3;
            unsigned suf = lsum;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned y = __shfl_down(suf, o, 64);
                if (lane + o < 64) suf += y;
            }
            const unsigned long long ball = __ballot(suf >= (unsigned)r);
            unsigned long long res = 0;  // digit | count << 16 | above << 32 ; 0xFFFF... = not enough entries
            if (ball == 0) res = ~0ull;
            else {
                const int ls = 63 - __builtin_clzll(ball);
                unsigned above = __shfl(suf - lsum, ls, 64);
                const unsigned b3 = __shfl(h3, ls, 64), b2 = __shfl(h2, ls, 64), b1 = __shfl(h1, ls, 64),
                               b0 = __shfl(h0, ls, 64);
                unsigned digit, cnt;
                if (above + b3 >= (unsigned)r) { digit = 4 * ls + 3; cnt = b3; }
                else if (above + b3 + b2 >= (unsigned)r) { digit = 4 * ls + 2; above += b3; cnt = b2; }
                else if (above + b3 + b2 + b1 >= (unsigned)r) { digit = 4 * ls + 1; above += b3 + b2; cnt = b1; }
                else { digit = 4 * ls; above += b3 + b2 + b1; cnt = b0; }
                res = (unsigned long long)digit | ((unsigned long long)min(cnt, 0xFFFFu) << 16) | ((unsigned long long)above << 32);
            }
            if (lane == 0) *bc = res;
        }
        __syncthreads();
        const unsigned long long res = *bc;
        if (res == ~0ull) return 0;
        r -= (int)(res >> 32);
        prefix |= (res & 0xFFull) << shift;
        if (((res >> 16) & 0xFFFFull) == 1 && shift > 0) {  // a single entry carries this prefix: fetch it
            __syncthreads();
            if (tid == 0) *bc = 0;
            __syncthreads();
            for (int i = tid; i < L.M; i += NT_CHUNK) {
                const int p = L.pos(i);
                if (p < tlim) {
                    const unsigned long long key = sel_key(L.val(i), p);
                    if ((key >> shift) == (prefix >> shift)) *bc = key;  // exactly one writer
                }
            }
            __syncthreads();
            return *bc;
        }
        __syncthreads();
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

// Smallest score of prefix t.
template <class List>
__device__ __forceinline__ float prefix_min(const List& L, int t, int lane)
{
    float m2 = INFINITY;
    for (int i = lane; i < L.M; i += 64)
        if (L.pos(i) <= t) m2 = fminf(m2, L.val(i));
    return wave_min_f32(m2);
}
__device__ __forceinline__ float prefix_min(const ListSorted& L, int t, int lane)
{
    const int nc = t - L.t0 + 1;
    float m2 = fminf((lane < nc) ? L.nv0 : INFINITY, (lane + 64 < nc) ? L.nv1 : INFINITY);
    if (L.m_old > 0) m2 = fminf(m2, key_score(L.key[L.m_old - 1]));
    return wave_min_f32(m2);
}

// One wave, thresholds of prefixes [ta, tb) (those longer than k).
template <class List>
__device__ void wave_tau(const List& L, const float* __restrict__ ur, float* __restrict__ tr, int ta, int tb,
                         int k, float start0, int lane, int* status)
{
    const float my_u = (ta + lane < tb) ? ur[ta + lane] : 0.0f;  // tb - ta <= 64
    bool have_prev = false;
    double tau_prev = 0.0;
    for (int t = ta; t < tb; t++) {
        if (t + 1 <= k) continue;  // written by the coarse kernel's short-prefix scan
        const double ut = (double)readlane_f32(my_u, t - ta);
        double tau;
        if (have_prev && !(ut > tau_prev)) {
            tau = tau_prev;  // the new score is below the threshold: nothing changes
        } else {
            double start;
            if (have_prev) start = tau_prev;
            else if (start0 > -INFINITY) start = (double)start0;
            else {  // no bound known: min(prefix) - 1 has f = t+1 >= k
                start = (double)prefix_min(L, t, lane) - 1.0;
            }
            tau = solve_tau(L, t, k, start, lane, status);
        }
        tau_prev = tau;
        have_prev = true;
        if (lane == 0) tr[t] = (float)tau;
    }
}

// The same for the sorted list, with the linear piece carried from prefix to prefix: a new score
// above the threshold changes the counts of the current piece by one, the root of that piece is
// the closed form, and it is final if no breakpoint lies between the old and the new threshold
// (the sorted neighbours and one ballot over the chunk's own scores tell).  Only otherwise the
// piece is evaluated again (eval_sorted), with the two-sided iteration of solve_tau.
__device__ void wave_tau(const ListSorted& L, const float* __restrict__ ur, float* __restrict__ tr, int ta,
                         int tb, int k, float start0, int lane, int* status)
{
    const float my_u = (ta + lane < tb) ? ur[ta + lane] : 0.0f;  // tb - ta <= 64
    bool started = false;  // x = tau of the previous prefix
    bool have = false;     // and P describes the piece of that prefix's f at x
    double x = 0.0;
    Piece P;
    for (int t = ta; t < tb; t++) {
        if (t + 1 <= k) continue;  // written by the coarse kernel's short-prefix scan
        const float utf = readlane_f32(my_u, t - ta);
        const double ut = (double)utf;
        if (started && !(ut > x)) {  // the new score is below the threshold: nothing changes
            if (lane == 0) tr[t] = (float)x;
            continue;
        }
        if (have) {
            if (ut > x + 1.0) { P.F++; P.S++; }
            else { P.S++; P.fsum += ut; }
        } else {
            if (!started) {
                if (start0 > -INFINITY) x = (double)start0;
                else x = (double)prefix_min(L, t, lane) - 1.0;  // no bound known: f = t+1 >= k there
            }
            P = eval_sorted(L, t, x, lane);  // tau only rises: f_t(x) >= k at the previous tau too
            have = true;
        }
        started = true;
        // two-sided iteration on f_t from the piece P at x
        double lo_b = x, hi_b = INFINITY;
        int it = 0;
        for (; it < MAX_ITERS; it++) {
            const double f = (double)P.F + P.fsum - (double)(P.S - P.F) * x;
            double xn = 0.0;
            bool step = false;
            if (f < (double)k) {
                hi_b = x;
                if (P.S > P.F) {
                    xn = (P.fsum + (double)P.F - (double)k) / (double)(P.S - P.F);
                    // still inside the piece (it starts at the largest breakpoint <= x): exact root
                    if (xn < x && xn >= P.prev_old && own_piece_clear(L, t, xn, x, lane)) { x = xn; break; }
                    step = xn > lo_b && xn < hi_b;
                }
            } else {
                lo_b = x;
                if (P.S == P.F) {  // flat to the right of x, f == F there
                    const double nb = (double)min_saturated(L, t, x, P.a, lane) - 1.0;  // next breakpoint
                    if (P.F == k) {  // sup of the level set f == k; the piece changes there
                        x = nb;
                        have = false;
                        break;
                    }
                    xn = nb;  // F > k: still left of the root
                    step = xn < hi_b;
                } else {
                    xn = (P.fsum + (double)P.F - (double)k) / (double)(P.S - P.F);
                    if (!(xn > x)) break;  // f(x) == k up to rounding
                    if (xn < P.next_old && own_piece_clear(L, t, x, xn, lane)) { x = xn; break; }
                    step = xn < hi_b;
                }
            }
            if (!step) {
                const double mid = 0.5 * (lo_b + hi_b);
                if (!(mid > lo_b && mid < hi_b)) { x = lo_b; have = false; break; }
                xn = mid;
            }
            x = xn;
            P = eval_sorted(L, t, x, lane);
        }
        if (it == MAX_ITERS && lane == 0) atomicOr(status, 1);
        if (lane == 0) tr[t] = (float)x;
    }
}

// One wave, the whole chunk: theta_t = k-th largest selection key of prefix t (0 while the
// prefix is shorter than k), by "newcomer in, smallest out" starting from theta_{t0-1}.
template <class List>
__device__ void wave_theta(const List& L, const float* __restrict__ ur, int t0, int t1, int k,
                           unsigned long long theta, int lane, unsigned long long* th)
{
    for (int tb = t0; tb < t1; tb += 64) {
        const float my_u = (tb + lane < t1) ? ur[tb + lane] : 0.0f;
        for (int t = tb; t < min(t1, tb + 64); t++) {
            const int len = t + 1;
            if (len == k) {
                theta = min_key(L, t + 1, lane);
            } else if (len > k) {
                const unsigned long long e = sel_key(readlane_f32(my_u, t - tb), t);
                if (e > theta) {
                    const unsigned long long sc = succ_key(L, t, theta, lane);
                    theta = e < sc ? e : sc;
                }
            }
            if (lane == 0) th[t - t0] = theta;
        }
    }
}

// The same walk on the sorted list: `na` older keys lie above theta, so the next older key above
// theta is key[na - 1]; the chunk's own keys are compared in registers.  This walk is the one
// sequential dependency of a chunk, so it is kept short: in a chunk whose prefixes all hold more
// than k entries only the newcomers above the starting theta are visited (the others can never
// enter the top-k: theta only rises), the next two older keys are held in registers, and the
// steps in between are filled in afterwards with a prefix maximum.
__device__ void wave_theta(const ListSorted& L, const float* __restrict__ ur, int t0, int t1, int k,
                           unsigned long long theta, int lane, unsigned long long* th)
{
    const unsigned long long k0 = sel_key(L.nv0, t0 + lane), k1 = sel_key(L.nv1, t0 + lane + 64);
    if (t0 >= k) {
        __builtin_amdgcn_s_setprio(3);  // the other waves of the workgroup wait for this one
        const unsigned long long th_start = theta;
        int na = k - 1;  // theta = key[k - 1]
        unsigned long long so0 = na > 0 ? L.key[na - 1] : ~0ull, so1 = na > 1 ? L.key[na - 2] : ~0ull;
        th[lane] = 0ull;
        th[lane + 64] = 0ull;
        const int cn = t1 - t0;
        unsigned long long m[2] = {__ballot(lane < cn && k0 > th_start), __ballot(lane + 64 < cn && k1 > th_start)};
        for (int h = 0; h < 2; h++) {
            unsigned long long todo = m[h];
            while (todo) {
                const int cl = __builtin_ctzll(todo);
                todo &= todo - 1;
                const int c = 64 * h + cl;  // chunk entries 0..c-1 are inside the prefix, entry c is the newcomer
                const unsigned long long e = h ? readlane_u64(k1, cl) : readlane_u64(k0, cl);
                if (e > theta) {
                    unsigned long long sc = ~0ull;
                    if (lane < c && k0 > theta) sc = k0;
                    if (lane + 64 < c && k1 > theta && k1 < sc) sc = k1;
                    sc = wave_min_u64(sc);
                    unsigned long long nt = e < sc ? e : sc;
                    if (so0 < nt) {
                        nt = so0;
                        na--;
                        so0 = so1;
                        so1 = na > 1 ? L.key[na - 2] : ~0ull;
                    }
                    theta = nt;
                    if (lane == 0) th[c] = theta;
                }
            }
        }
        // th[i] = max(th_start, th[0..i]): inclusive prefix maximum over the 128 entries
        unsigned long long a = th[lane], b = th[lane + 64];
        a = a > th_start ? a : th_start;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long y = __shfl_up(a, o, 64);
            if (lane >= o && y > a) a = y;
        }
        const unsigned long long top = readlane_u64(a, 63);
        b = b > top ? b : top;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long y = __shfl_up(b, o, 64);
            if (lane >= o && y > b) b = y;
        }
        th[lane] = a;
        th[lane + 64] = b;
        __builtin_amdgcn_s_setprio(0);
        return;
    }
    int na = 0;
    for (int t = t0; t < t1; t++) {
        const int len = t + 1, c = t - t0;  // chunk entries 0..c-1 are inside prefix t-1, entry c is the newcomer
        if (len == k) {
            // every entry of the prefix is selected: theta is the smallest key
            unsigned long long m = ~0ull;
            if (lane <= c) m = k0;
            if (lane + 64 <= c) m = k1 < m ? k1 : m;
            m = wave_min_u64(m);
            if (L.m_old > 0) m = L.key[L.m_old - 1] < m ? L.key[L.m_old - 1] : m;
            theta = m;
            na = L.m_old;
            // older keys above theta: all but the one that equals it, if that one is the minimum
            if (L.m_old > 0 && L.key[L.m_old - 1] == theta) na = L.m_old - 1;
        } else if (len > k) {
            const unsigned long long e = (c < 64) ? readlane_u64(k0, c) : readlane_u64(k1, c - 64);
            if (e > theta) {
                unsigned long long sc = ~0ull;
                if (lane < c && k0 > theta) sc = k0;
                if (lane + 64 < c && k1 > theta && k1 < sc) sc = k1;
                sc = wave_min_u64(sc);
                const unsigned long long so = (na > 0) ? L.key[na - 1] : ~0ull;
                unsigned long long nt = e < sc ? e : sc;
                if (so < nt) { nt = so; na--; }
                theta = nt;
            }
        }
        if (lane == 0) th[t - t0] = theta;
    }
}

// death of one list entry given the chunk's theta sequence (non-decreasing).
__device__ __forceinline__ void write_death(unsigned long long key, int j, int t0, int t1, int k,
                                            const unsigned long long* th, unsigned long long th_start,
                                            int32_t* __restrict__ dr)
{
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

constexpr int NW_TAU = NW_CHUNK - 1;                     // waves solving tau; the last wave walks theta
constexpr int TPW_TAU = (CHUNK + NW_TAU - 1) / NW_TAU;   // prefixes per tau wave
constexpr int SLICE_REG = 8;                             // compaction: scores cached per lane and segment

template <class List>
__device__ void chunk_body(const List& L, const float* __restrict__ ur, float* __restrict__ tr,
                           int32_t* __restrict__ dr, int t0, int t1, int k, float lo, unsigned* hist,
                           unsigned long long* bc, unsigned long long* th, int* status)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // theta at the chunk start, by the whole workgroup
    unsigned long long th_start = 0;
    if (t0 >= k) th_start = block_kth_largest(L, t0, k, hist, bc);
    // tau lies in [z_(k) - 1, z_(k)), and both ends only rise: theta_{t0-1} - 1 bounds every tau of the chunk
    float start0 = lo;
    if (t0 >= k) start0 = fmaxf(lo, __uint_as_float(score_key_inv((uint32_t)(th_start >> 32))) - 1.0f);
    if (wv < NW_TAU) {
        const int ta = min(t1, t0 + wv * TPW_TAU), tb = min(t1, ta + TPW_TAU);
        wave_tau(L, ur, tr, ta, tb, k, start0, lane, status);
    } else {
        wave_theta(L, ur, t0, t1, k, th_start, lane, th);
    }
    __syncthreads();
    for (int i = tid; i < L.M; i += NT_CHUNK) {
        const int p = L.pos(i);
        if (p < t1) write_death(sel_key(L.val(i), p), p, t0, t1, k, th, th_start, dr);
    }
}

// The same for the sorted list: theta at the chunk start is the k-th sorted key.
__device__ void chunk_body_sorted(const ListSorted& L, const float* __restrict__ ur, float* __restrict__ tr,
                                  int32_t* __restrict__ dr, int t0, int t1, int k, float lo,
                                  unsigned long long* th, int* status)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const unsigned long long th_start = (t0 >= k) ? L.key[k - 1] : 0ull;
    // tau lies in [z_(k) - 1, z_(k)), and both ends only rise: theta_{t0-1} - 1 bounds every tau of the chunk
    float start0 = lo;
    if (t0 >= k) start0 = fmaxf(lo, key_score(th_start) - 1.0f);
    if (wv < NW_TAU) {
        const int ta = min(t1, t0 + wv * TPW_TAU), tb = min(t1, ta + TPW_TAU);
        wave_tau(L, ur, tr, ta, tb, k, start0, lane, status);
    } else {
        wave_theta(L, ur, t0, t1, k, th_start, lane, th);
    }
    __syncthreads();
    for (int i = tid; i < L.m_old; i += NT_CHUNK) {
        const unsigned long long key = L.key[i];
        write_death(key, key_pos(key), t0, t1, k, th, th_start, dr);
    }
    if (tid < t1 - t0) write_death(sel_key(ur[t0 + tid], t0 + tid), t0 + tid, t0, t1, k, th, th_start, dr);
}

// Bitonic sort of key[0, N) in descending order, N a power of two >= 2048 (one or more pairs per
// thread).  Each wave owns a contiguous run of N/32 compare-exchange pairs, so passes whose
// stride fits into the wave's N/16 elements need no workgroup barrier: a wave's LDS accesses are
// performed in program order.
__device__ void bitonic_sort_desc(unsigned long long* key, int N)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int P = N / (2 * NW_CHUNK);  // pairs per wave
    for (int k2 = 2; k2 <= N; k2 <<= 1) {
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            if (j > P) __syncthreads();
            for (int m = lane; m < P; m += 64) {
                const int i = wv * P + m;
                const int a = 2 * i - (i & (j - 1)), b = a + j;
                const unsigned long long x = key[a], y = key[b];
                const bool desc = (a & k2) == 0;
                if ((x < y) == desc) {
                    key[a] = y;
                    key[b] = x;
                }
            }
            if (j > P) __syncthreads();
        }
    }
    __syncthreads();
}

// Sort key[0, m) in descending order by distribution: NB value buckets between the smallest and
// the largest score (one counting pass, one scan, one scatter into `tmp`), then every element
// finds its rank inside its bucket by reading the bucket (a handful of elements for spread-out
// scores) and goes to its final place in key[].  Returns false, with key[] untouched, when some
// bucket holds more than BUCKET_MAX elements (many equal or clustered scores): the caller then
// sorts by comparison.  The result depends on the keys only, not on the order of the atomics.
constexpr int NB = 2048;
constexpr int CAP_SMALL = 4096, NB_SMALL = 1024;   // the variant for k small enough that 4096 candidates suffice
constexpr int BUCKET_MAX = 96;

template <int NB>
__device__ bool bucket_sort_desc(unsigned long long* key, unsigned long long* tmp, int m, float vmin, float vmax,
                                 int* bcount /* [NB] */, int* boff /* [NB + 1] */, int* flag, int* wsum /* [NW_CHUNK] */)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float scale = (float)NB / (vmax - vmin);
    auto bucket = [&](unsigned long long kk) {
        const float v = key_score(kk);
        int b = (int)((v - vmin) * scale);
        b = max(0, min(NB - 1, b));
        return NB - 1 - b;  // larger scores first
    };
    for (int i = tid; i < NB; i += NT_CHUNK) bcount[i] = 0;
    if (tid == 0) *flag = 0;
    __syncthreads();
    for (int i = tid; i < m; i += NT_CHUNK) atomicAdd(&bcount[bucket(key[i])], 1);
    __syncthreads();
    // exclusive scan of the NB counts (NB / NT_CHUNK consecutive buckets per thread)
    constexpr int BPT = NB / NT_CHUNK;
    int c[BPT], tot = 0, big = 0;
#pragma unroll
    for (int r = 0; r < BPT; r++) {
        c[r] = bcount[tid * BPT + r];
        tot += c[r];
        big |= c[r] > BUCKET_MAX ? 1 : 0;
    }
    int inc = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(inc, o, 64);
        if (lane >= o) inc += y;
    }
    if (lane == 63) wsum[wv] = inc;
    if (big) *flag = 1;
    __syncthreads();
    if (*flag) return false;
    int before = inc - tot;
    for (int i = 0; i < wv; i++) before += wsum[i];
#pragma unroll
    for (int r = 0; r < BPT; r++) {
        boff[tid * BPT + r] = before;
        bcount[tid * BPT + r] = before;  // scatter cursor
        before += c[r];
    }
    if (tid == NT_CHUNK - 1) boff[NB] = before;
    __syncthreads();
    for (int i = tid; i < m; i += NT_CHUNK) {
        const unsigned long long kk = key[i];
        tmp[atomicAdd(&bcount[bucket(kk)], 1)] = kk;
    }
    __syncthreads();
    for (int i = tid; i < m; i += NT_CHUNK) {
        const unsigned long long kk = tmp[i];
        const int b = bucket(kk);
        const int b0 = boff[b], b1 = boff[b + 1];
        int rank = 0;
        for (int j = b0; j < b1; j++) rank += tmp[j] > kk ? 1 : 0;
        key[b0 + rank] = kk;
    }
    __syncthreads();
    return true;
}

// pref[i] = sum of the scores of key[0, i), i = 0..N, in fp64 (N a multiple of NT_CHUNK).
__device__ void sorted_prefix_sums(const unsigned long long* key, double* pref, int N, int m_old, double* wtot)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int per = N / NT_CHUNK;
    double run = 0.0;
    for (int r = 0; r < per; r++) {
        const int i = tid * per + r;
        run += (i < m_old) ? (double)key_score(key[i]) : 0.0;
    }
    // inclusive scan of the thread totals across the wave, then across the waves
    double inc = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double y = __shfl_up(inc, o, 64);
        if (lane >= o) inc += y;
    }
    if (lane == 63) wtot[wv] = inc;
    __syncthreads();
    double before = inc - run;
    for (int i = 0; i < wv; i++) before += wtot[i];
    for (int r = 0; r < per; r++) {
        const int i = tid * per + r;
        pref[i] = before;
        before += (i < m_old) ? (double)key_score(key[i]) : 0.0;
    }
    if (tid == NT_CHUNK - 1) pref[N] = before;
    __syncthreads();
}

template <int CAP, int NB>
__global__ __launch_bounds__(NT_CHUNK, CAP <= CAP_SMALL ? 8 : 4) void mask_chunk_kernel(
    const float* __restrict__ u, const float* __restrict__ lo_in, float* __restrict__ tau,
    int32_t* __restrict__ death, int n, int k, int nsuper, int* __restrict__ status, int t_begin,
    unsigned* __restrict__ handed_on, int only_handed_on)
{
    __shared__ __align__(16) unsigned long long skey[CAP];
    __shared__ __align__(16) double pref[CAP + 1];
    __shared__ unsigned long long th[CHUNK];
    __shared__ unsigned hist[256];
    __shared__ double wtot[NW_CHUNK];
    __shared__ int wcount[NW_CHUNK + 1];
    __shared__ float wmin[NW_CHUNK], wmax[NW_CHUNK];
    __shared__ int bcount[NB], boff[NB + 1], bflag, wsum[NW_CHUNK];
    __shared__ unsigned long long bc;

    const int c = blockIdx.x, row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int t0 = c * CHUNK, t1 = min(n, t0 + CHUNK);
    if (t1 <= k) return;  // no prefix here is longer than k: tau is written elsewhere, nothing dies
    if (t1 <= t_begin) return;  // the caller needs neither these thresholds nor the deaths that fall here
    // Two launches share the chunks when there are many: the half-capacity kernel (two workgroups per compute unit)
    // takes them all and hands on, through one bit each, those whose candidates do not fit its lists; the
    // full-capacity kernel then runs those alone.
    const int chunk_id = row * gridDim.x + c;
    if (only_handed_on && !((handed_on[chunk_id >> 5] >> (chunk_id & 31)) & 1u)) return;
    const float* ur = u + (size_t)row * n;
    float* tr = tau + (size_t)row * n;
    int32_t* dr = death + (size_t)row * n;
    const float lo = lo_in[(size_t)row * nsuper + t0 / SUPER];

    // ---- compaction of {j < t0 : u_j > lo} as selection keys, in one pass: each wave owns a contiguous slice, read
    // in segments of 64*SLICE_REG scores held in registers (independent loads, one latency); a segment reserves
    // its room in the list with one LDS atomic.  The order in which the segments land does not matter: the list
    // is sorted next, and the keys are distinct. ----
    const int per = ((t0 + NW_CHUNK - 1) / NW_CHUNK + 63) / 64 * 64;
    const int sb = min(t0, wv * per), se = min(t0, sb + per);
    constexpr int SEGN = 64 * SLICE_REG;
    if (tid == 0) wcount[NW_CHUNK] = 0;
    __syncthreads();
    float cmin = INFINITY, cmax = -INFINITY;  // range of the candidates
    for (int g0 = sb; g0 < se; g0 += SEGN) {
        float z[SLICE_REG];
#pragma unroll
        for (int r = 0; r < SLICE_REG; r++) {
            const int i = g0 + r * 64 + lane;
            z[r] = (i < se) ? ur[i] : -INFINITY;
        }
        int seg_cnt = 0;
#pragma unroll
        for (int r = 0; r < SLICE_REG; r++) {
            const bool p = z[r] > lo;
            seg_cnt += __popcll(__ballot(p));
            cmin = p ? fminf(cmin, z[r]) : cmin;
            cmax = p ? fmaxf(cmax, z[r]) : cmax;
        }
        int off = 0;
        if (lane == 0 && seg_cnt > 0) off = atomicAdd(&wcount[NW_CHUNK], seg_cnt);
        off = __builtin_amdgcn_readfirstlane(off);
#pragma unroll
        for (int r = 0; r < SLICE_REG; r++) {
            const bool p = z[r] > lo;
            const unsigned long long ball = __ballot(p);
            const int pos = off + __popcll(ball & ((1ull << lane) - 1ull));
            if (p && pos < CAP) skey[pos] = sel_key(z[r], g0 + r * 64 + lane);   // beyond CAP: the slow path below
            off += __popcll(ball);
        }
    }
    cmin = wave_min_f32(cmin);
    cmax = wave_max_f32(cmax);
    if (lane == 0) { wmin[wv] = cmin; wmax[wv] = cmax; }
    __syncthreads();
    const int m_old = wcount[NW_CHUNK];
    // the list must hold the whole top-k of every prefix of the chunk (it does when lo is a lower
    // bound of tau; checked, not assumed)
    const bool fits = (m_old <= CAP) && (t0 < k || m_old >= k);
    if (fits) {
        int npad = 2 * NT_CHUNK;
        while (npad < m_old) npad <<= 1;
        for (int i = m_old + tid; i < npad; i += NT_CHUNK) skey[i] = 0ull;  // below every real key
        __syncthreads();
        if (m_old > 0) {
            float vmin = INFINITY, vmax = -INFINITY;
            for (int i = 0; i < NW_CHUNK; i++) { vmin = fminf(vmin, wmin[i]); vmax = fmaxf(vmax, wmax[i]); }
            // pref[] is free until the prefix sums are taken: scratch of the distribution sort
            if (!bucket_sort_desc<NB>(skey, (unsigned long long*)pref, m_old, vmin, vmax, bcount, boff, &bflag, wsum))
                bitonic_sort_desc(skey, npad);
            sorted_prefix_sums(skey, pref, npad, m_old, wtot);
        }
        const int cn = t1 - t0;
        ListSorted L{skey, pref, m_old, t0, (lane < cn) ? ur[t0 + lane] : -INFINITY,
                     (lane + 64 < cn) ? ur[t0 + lane + 64] : -INFINITY};
        chunk_body_sorted(L, ur, tr, dr, t0, t1, k, lo, th, status);
    } else if (CAP <= CAP_SMALL && !only_handed_on) {
        if (tid == 0) atomicOr(&handed_on[chunk_id >> 5], 1u << (chunk_id & 31));
    } else {
        ListGlobal L{ur, t1};
        chunk_body(L, ur, tr, dr, t0, t1, k, -INFINITY, hist, &bc, th, status);
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
                hipStream_t st, int t_begin)
{
    const int rows = c.B * c.Gu;
    const int nsuper = (c.n + SUPER - 1) / SUPER;
    const int nchunks = (c.n + CHUNK - 1) / CHUNK;
    const size_t lo_bytes = align_up((size_t)rows * nsuper * sizeof(float), 256);
    float* lo = (float*)ws;
    int* status = (int*)((char*)ws + lo_bytes);
    unsigned* handed_on = (unsigned*)((char*)ws + lo_bytes + 256);
    const int nwords = (int)(((size_t)rows * nchunks + 31) / 32);
    hipLaunchKernelGGL(mask_coarse_kernel, dim3(c.k == 0 ? 1 : nsuper, rows), dim3(NT_COARSE), 0, st, u, lo, tau,
                       death, c.n, c.k, nsuper, status, handed_on, nwords);
    if (c.k == 0) return launch_status();
    if (c.k < c.n) {
        // The candidates of a chunk number about 2.5 k for scores of unit variance (the support of the threshold), so
        // up to k = 1280 the half-size lists usually do, and two workgroups then fit a compute unit: worth it when
        // the chunks outnumber the compute units several times (many score rows).  Chunks whose candidates do not
        // fit are handed on to the full-capacity kernel.  Not for the virtual sequences of the chunked prefill
        // (t_begin > 0), whose padding scores all count as candidates at first.
        const bool two_stage = c.k <= 1280 && t_begin == 0 && (long long)rows * nchunks >= 2048;
        if (two_stage)
            hipLaunchKernelGGL((mask_chunk_kernel<CAP_SMALL, NB_SMALL>), dim3(nchunks, rows), dim3(NT_CHUNK), 0, st, u, lo,
                               tau, death, c.n, c.k, nsuper, status, t_begin, handed_on, 0);
        hipLaunchKernelGGL((mask_chunk_kernel<CAP, NB>), dim3(nchunks, rows), dim3(NT_CHUNK), 0, st, u, lo, tau,
                           death, c.n, c.k, nsuper, status, t_begin, handed_on, two_stage ? 1 : 0);
    }
    return launch_status();
}

int mask_status(const sparsek_cfg& c, const void* ws, int32_t* host_flag, hipStream_t st)
{
    const size_t rows = (size_t)c.B * c.Gu, nsuper = ((size_t)c.n + SUPER - 1) / SUPER;
    const int* status = (const int*)((const char*)ws + align_up(rows * nsuper * sizeof(float), 256));
    if (hipMemcpyAsync(host_flag, status, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return SPARSEK_ERR_LAUNCH;
    return hipStreamSynchronize(st) == hipSuccess ? SPARSEK_OK : SPARSEK_ERR_LAUNCH;
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

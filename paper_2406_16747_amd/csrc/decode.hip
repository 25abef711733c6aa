// Constant-memory decode step (Sec. 3.2 irreversibility, Sec. 3.3 incremental SPARSEK).
//
// State per score row (b,g): the scores of the w window keys (a ring), of the <= k selected
// keys, and of every other key still above tau (the set S of the incremental algorithm minus
// the top-k), plus tau itself in fp64.  State per head (b,h): k+w key/value slots.  A key keeps
// its slot from the moment it is appended until it is dropped; selection only changes the
// per-slot gate score (+inf = window key, gate 1; finite = selected key, gate
// clip(u - tau, 0, 1); -inf = empty), so one step moves no K/V rows except the new token's.
//
// One step = two launches: (1) one workgroup per score row updates tau / top-k / candidates
// for the key that leaves the window and stores the new token's K/V rows; (2) one workgroup
// per head streams the k+w slots once (HBM-bound) with an online softmax.
#include "common.hpp"

namespace spk {

struct DecodeLayout {
    int rows, NS, cap, wlen, klen;
    size_t pos, nsel, ncand, status, nfree, new_slot, tau_d, tau_f;
    size_t win_u, win_slot, sel_u, sel_pos, sel_slot, cand_u, slot_u, free_stack, kslots, vslots, total;
};

__host__ __device__ inline DecodeLayout decode_layout(const sparsek_decode_cfg& c)
{
    DecodeLayout L;
    L.rows = c.B * c.Gu;
    L.NS = c.k + c.w;
    L.cap = c.cand_cap > 0 ? c.cand_cap : 4 * (c.k > 16 ? c.k : 16);
    L.wlen = c.w > 0 ? c.w : 1;
    L.klen = c.k > 0 ? c.k : 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = (off + bytes + 255) / 256 * 256;
        return o;
    };
    const size_t r = (size_t)L.rows;
    L.pos = take(r * 4);
    L.nsel = take(r * 4);
    L.ncand = take(r * 4);
    L.status = take(r * 4);
    L.nfree = take(r * 4);
    L.new_slot = take(r * 4);
    L.tau_d = take(r * 8);
    L.tau_f = take(r * 4);
    L.win_u = take(r * L.wlen * 4);
    L.win_slot = take(r * L.wlen * 4);
    L.sel_u = take(r * L.klen * 4);
    L.sel_pos = take(r * L.klen * 4);
    L.sel_slot = take(r * L.klen * 4);
    L.cand_u = take(r * (size_t)L.cap * 4);
    L.slot_u = take(r * (size_t)L.NS * 4);
    L.free_stack = take(r * (size_t)L.NS * 4);
    const size_t esz = c.dtype == SPARSEK_BF16 ? 2 : 4;
    const size_t kv = (size_t)c.B * c.H * L.NS * c.d * esz;
    L.kslots = take(kv);
    L.vslots = take(kv);
    L.total = off;
    return L;
}

size_t decode_state_bytes(const sparsek_decode_cfg& c) { return decode_layout(c).total; }

struct RowState {
    int *pos, *nsel, *ncand, *status, *nfree, *new_slot;
    double* tau_d;
    float* tau_f;
    float* win_u;
    int* win_slot;
    float* sel_u;
    int *sel_pos, *sel_slot;
    float *cand_u, *slot_u;
    int* free_stack;
};

__device__ inline RowState row_state(char* st, const DecodeLayout& L, int row)
{
    RowState R;
    R.pos = (int*)(st + L.pos) + row;
    R.nsel = (int*)(st + L.nsel) + row;
    R.ncand = (int*)(st + L.ncand) + row;
    R.status = (int*)(st + L.status) + row;
    R.nfree = (int*)(st + L.nfree) + row;
    R.new_slot = (int*)(st + L.new_slot) + row;
    R.tau_d = (double*)(st + L.tau_d) + row;
    R.tau_f = (float*)(st + L.tau_f) + row;
    R.win_u = (float*)(st + L.win_u) + (size_t)row * L.wlen;
    R.win_slot = (int*)(st + L.win_slot) + (size_t)row * L.wlen;
    R.sel_u = (float*)(st + L.sel_u) + (size_t)row * L.klen;
    R.sel_pos = (int*)(st + L.sel_pos) + (size_t)row * L.klen;
    R.sel_slot = (int*)(st + L.sel_slot) + (size_t)row * L.klen;
    R.cand_u = (float*)(st + L.cand_u) + (size_t)row * L.cap;
    R.slot_u = (float*)(st + L.slot_u) + (size_t)row * L.NS;
    R.free_stack = (int*)(st + L.free_stack) + (size_t)row * L.NS;
    return R;
}

constexpr int NT_ROW = 256;

// ---- block-wide reductions over NT_ROW threads (all threads get the result) ----
struct BlockRed {
    unsigned long long u64[NT_ROW / 64];
    double f64[NT_ROW / 64];
    float f32[NT_ROW / 64];
};

__device__ inline void block_eval(BlockRed& red, const float* a, int na, const float* b, int nb, bool with_z,
                                  float z, double x, int& F, int& S, double& fsum, float& minF)
{
    // right-limit counts of the piece of f that starts at x, over a[0..na) U b[0..nb) U {z}
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int f = 0, s = 0;
    double sum = 0.0;
    float mf = INFINITY;
    const double x1 = x + 1.0;
    auto add = [&](float v) {
        double dv = (double)v;
        if (dv > x) {
            s++;
            if (dv > x1) { f++; mf = fminf(mf, v); }
            else sum += dv;
        }
    };
    for (int i = tid; i < na; i += NT_ROW) add(a[i]);
    for (int i = tid; i < nb; i += NT_ROW) add(b[i]);
    if (with_z && tid == 0) add(z);
    unsigned long long packed = wave_sum_u64(((unsigned long long)f << 32) | (unsigned long long)s);
    double ws = wave_sum_f64(sum);
    float wm = wave_min_f32(mf);
    __syncthreads();
    if (lane == 0) { red.u64[wv] = packed; red.f64[wv] = ws; red.f32[wv] = wm; }
    __syncthreads();
    packed = 0;
    ws = 0.0;
    wm = INFINITY;
    for (int i = 0; i < NT_ROW / 64; i++) { packed += red.u64[i]; ws += red.f64[i]; wm = fminf(wm, red.f32[i]); }
    F = (int)(packed >> 32);
    S = (int)(packed & 0xFFFFFFFFull);
    fsum = ws;
    minF = wm;
}

// Same iteration as the prefill solver: tau <- (fsum + F - k)/(S - F), the root of the linear piece
// through the current point (from whichever side of the root it lies on), until (F, S) reproduce;
// a bracket of the root is kept and a step that leaves it is replaced by its midpoint.
__device__ double block_solve_tau(BlockRed& red, const float* a, int na, const float* b, int nb, bool with_z,
                                  float z, int k, double start, int* status)
{
    double lo_b = start, hi_b = INFINITY, x = start;
    int pF = -1, pS = -1;
    for (int it = 0; it < 4096; it++) {
        int F, S;
        double fsum;
        float minF;
        block_eval(red, a, na, b, nb, with_z, z, x, F, S, fsum, minF);
        if (F == pF && S == pS) return x;
        pF = pS = -1;
        const double f = (double)F + fsum - (double)(S - F) * x;
        double xn = 0.0;
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
    if (threadIdx.x == 0) atomicOr(status, 2);
    return x;
}

// In-place, order-preserving removal of candidates <= tau.  Returns the new count.
__device__ int block_prune(int* scan, float* cand, int n, float keep_above_as_double_hi, double tau)
{
    (void)keep_above_as_double_hi;
    const int tid = threadIdx.x;
    __shared__ int base_s;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n; i0 += NT_ROW) {
        const int i = i0 + tid;
        float v = (i < n) ? cand[i] : 0.0f;
        const bool keep = (i < n) && ((double)v > tau);
        const unsigned long long ball = __ballot(keep);
        const int lane = tid & 63, wv = tid >> 6;
        if (lane == 0) scan[wv] = __popcll(ball);
        __syncthreads();
        int off = base_s;
        for (int x = 0; x < wv; x++) off += scan[x];
        const int dst = off + __popcll(ball & ((1ull << lane) - 1ull));
        __syncthreads();  // all reads of this batch done before anyone writes (dst <= i always)
        if (keep) cand[dst] = v;
        if (tid == 0) base_s += scan[0] + scan[1] + scan[2] + scan[3];
        __syncthreads();
    }
    return base_s;
}

template <typename T>
__device__ __forceinline__ void copy_row(T* dst, const T* src, int d, int tid, int nt)
{
    for (int c = tid; c < d; c += nt) dst[c] = src[c];
}

// ---------------------------------------------------------------------------------
// (1) per score row: the key leaving the window joins the SPARSEK prefix; the new token is
// appended to the window; its K/V rows go to the freed slot.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT_ROW) void decode_update_kernel(sparsek_decode_cfg c, char* st,
                                                               const T* __restrict__ k_new,
                                                               const T* __restrict__ v_new,
                                                               const float* __restrict__ u_new)
{
    __shared__ BlockRed red;
    __shared__ int scan[NT_ROW / 64];
    __shared__ unsigned long long minkey_s[NT_ROW / 64];
    __shared__ int sh_i[4];
    const DecodeLayout L = decode_layout(c);
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    RowState R = row_state(st, L, row);
    const int k = c.k, w = c.w;
    const int t = *R.pos;
    int nsel = *R.nsel, ncand = *R.ncand;
    const int nfree0 = *R.nfree;
    const double tau_old = *R.tau_d;
    const float unew = u_new[row];
    // The new token's K/V rows of this score row's heads do not depend on the state: fetch the
    // first batch (16-byte vectors, 4 per thread and tensor) now, store it once the slot is known.
    const int b_ = row / c.Gu, g_ = row % c.Gu;
    const int h0 = (c.Gu == 1) ? 0 : g_, nh = (c.Gu == 1) ? c.H : 1;
    const int vpr = c.d * (int)sizeof(T) / 16;  // vectors per row
    const int nvec = nh * vpr;
    const uint4* ksrc = (const uint4*)(k_new + ((size_t)b_ * c.H + h0) * c.d);
    const uint4* vsrc = (const uint4*)(v_new + ((size_t)b_ * c.H + h0) * c.d);
    constexpr int VB = 4;
    uint4 kpre[VB], vpre[VB];
#pragma unroll
    for (int r = 0; r < VB; r++) {
        const int v = r * NT_ROW + tid;
        if (v < nvec) { kpre[r] = ksrc[v]; vpre[r] = vsrc[v]; }
    }
    __syncthreads();

    const bool leave = (w == 0) || (t >= w);
    int new_slot = -1;
    // Free-slot stack: at most one slot is pushed and at most one is popped per step, so the
    // step works on a local copy (count, the slot pushed in this step, the old top fetched
    // ahead) and writes the stack back once.
    int nfree = nfree0, pushed = -1;
    const int old_top = nfree0 > 0 ? R.free_stack[nfree0 - 1] : -1;
    auto pop_slot = [&]() -> int {
        if (pushed >= 0) { const int r = pushed; pushed = -1; return r; }
        nfree--;
        return old_top;
    };
    if (leave) {
        const int p = (w > 0) ? t - w : t;          // position joining the prefix (= prefix index T)
        const float z = (w > 0) ? R.win_u[p % w] : unew;
        const int zslot = (w > 0) ? R.win_slot[p % w] : -1;
        const int len = p + 1;
        // ---- (a) top-k decision (nothing is modified yet) ----
        bool selected = false;
        int e = -1;  // entry of the selected arrays that receives z
        bool evict = false;
        if (k > 0) {
            if (nsel < k) {
                selected = true;
                e = nsel;
            } else {
                unsigned long long mk = ~0ull;
                for (int i = tid; i < nsel; i += NT_ROW) {
                    unsigned long long key = sel_key(R.sel_u[i], R.sel_pos[i]);
                    mk = key < mk ? key : mk;
                }
                mk = wave_min_u64(mk);
                if (lane == 0) minkey_s[wv] = mk;
                __syncthreads();
                mk = minkey_s[0];
                for (int i = 1; i < NT_ROW / 64; i++) mk = minkey_s[i] < mk ? minkey_s[i] : mk;
                if (sel_key(z, p) > mk) {
                    selected = true;
                    evict = true;
                    for (int i = tid; i < nsel; i += NT_ROW)
                        if (sel_key(R.sel_u[i], R.sel_pos[i]) == mk) sh_i[0] = i;
                    __syncthreads();
                    e = sh_i[0];
                }
            }
        }
        // ---- (b) threshold of prefix p ----
        double tau_new;
        if (k == 0) {
            tau_new = (len == 1) ? (double)z : fmax(tau_old, (double)z);
        } else if (len <= k) {
            tau_new = (len == 1) ? (double)z - 1.0 : fmin(tau_old, (double)z - 1.0);
        } else if ((double)z > tau_old) {
            tau_new = block_solve_tau(red, R.sel_u, nsel, R.cand_u, ncand, true, z, k, tau_old, R.status);
        } else {
            tau_new = tau_old;
        }
        // ---- (c) candidates: scores above tau outside the top-k ----
        const float ev_u = evict ? R.sel_u[e] : 0.0f;
        const int ev_slot = evict ? R.sel_slot[e] : -1;
        __syncthreads();
        if (k > 0 && len > k) {
            // Candidates that fell to or below tau do no harm (they count nowhere); they are only
            // swept out when the set gets three quarters full, not at every rise of tau.
            if ((tau_new > tau_old && ncand + 2 > (L.cap / 4) * 3) || ncand + 2 > L.cap)
                ncand = block_prune(scan, R.cand_u, ncand, 0.0f, tau_new);
            if (tid == 0) {
                float add[2];
                int na = 0;
                if (!selected && (double)z > tau_new) add[na++] = z;
                if (evict && (double)ev_u > tau_new) add[na++] = ev_u;
                for (int i = 0; i < na; i++) {
                    if (ncand < L.cap) R.cand_u[ncand++] = add[i];
                    else {  // bounded set (Sec. 3.3): drop the smallest, flag the row
                        atomicOr(R.status, 1);
                        int mi = 0;
                        for (int x = 1; x < ncand; x++) if (R.cand_u[x] < R.cand_u[mi]) mi = x;
                        if (ncand > 0 && R.cand_u[mi] < add[i]) R.cand_u[mi] = add[i];
                    }
                }
                sh_i[1] = ncand;
            }
            __syncthreads();
            ncand = sh_i[1];
        }
        // ---- (d) slots ----
        if (tid == 0) {
            if (selected) {
                int slot = zslot;
                if (evict) {
                    R.slot_u[ev_slot] = -INFINITY;
                    pushed = ev_slot;
                }
                if (w == 0) slot = pop_slot();
                R.sel_u[e] = z;
                R.sel_pos[e] = p;
                R.sel_slot[e] = slot;
                R.slot_u[slot] = z;
                if (!evict) nsel++;
                if (w == 0) new_slot = slot;
            } else if (w > 0) {
                R.slot_u[zslot] = -INFINITY;
                pushed = zslot;
            }
            *R.nsel = nsel;
            *R.ncand = ncand;
            *R.tau_d = tau_new;
            *R.tau_f = (float)tau_new;
        }
    }
    // ---- (2) append the new token to the window ----
    if (tid == 0) {
        if (w > 0) {
            const int slot = pop_slot();
            R.win_u[t % w] = unew;
            R.win_slot[t % w] = slot;
            R.slot_u[slot] = INFINITY;
            new_slot = slot;
        }
        if (pushed >= 0) R.free_stack[nfree++] = pushed;
        *R.nfree = nfree;
        *R.new_slot = new_slot;
        *R.pos = t + 1;
        sh_i[2] = new_slot;
    }
    __syncthreads();
    new_slot = sh_i[2];
    if (new_slot >= 0) {
        T* ks = (T*)(st + L.kslots);
        T* vs = (T*)(st + L.vslots);
        auto dst = [&](T* slots, int v) -> uint4* {  // vector v of the rows -> its place in slot new_slot
            const size_t bh = (size_t)b_ * c.H + h0 + v / vpr;
            return (uint4*)(slots + (bh * L.NS + new_slot) * c.d) + v % vpr;
        };
#pragma unroll
        for (int r = 0; r < VB; r++) {
            const int v = r * NT_ROW + tid;
            if (v < nvec) { *dst(ks, v) = kpre[r]; *dst(vs, v) = vpre[r]; }
        }
        for (int v = VB * NT_ROW + tid; v < nvec; v += NT_ROW) {  // more heads than one batch holds
            *dst(ks, v) = ksrc[v];
            *dst(vs, v) = vsrc[v];
        }
    }
}

// ---------------------------------------------------------------------------------
// (2) attention of the one new query over the k+w slots of its head.
// LPR lanes share a slot row (8 elements each); 64/LPR rows per wave-load; 16 independent
// online-softmax streams per workgroup, merged through LDS at the end.
// ---------------------------------------------------------------------------------
template <typename T>
struct Ld8;
template <>
struct Ld8<uint16_t> {
    static __device__ __forceinline__ void ld(const uint16_t* p, float (&x)[8])
    {
        const uint4 r = *(const uint4*)p;
        x[0] = __uint_as_float(r.x << 16); x[1] = __uint_as_float(r.x & 0xFFFF0000u);
        x[2] = __uint_as_float(r.y << 16); x[3] = __uint_as_float(r.y & 0xFFFF0000u);
        x[4] = __uint_as_float(r.z << 16); x[5] = __uint_as_float(r.z & 0xFFFF0000u);
        x[6] = __uint_as_float(r.w << 16); x[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
};
template <>
struct Ld8<float> {
    static __device__ __forceinline__ void ld(const float* p, float (&x)[8])
    {
        const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
};
__device__ __forceinline__ void st1(uint16_t* p, float v) { *p = f32_to_bf16(v); }
__device__ __forceinline__ void st1(float* p, float v) { *p = v; }

template <typename T, int LPR, int MODE>
__global__ __launch_bounds__(256) void decode_attn_kernel(sparsek_decode_cfg c, const char* st,
                                                          const T* __restrict__ q_new, T* __restrict__ o)
{
    constexpr int D = LPR * 8;
    constexpr int RPW = 64 / LPR;        // rows per wave-load
    constexpr int NSTREAM = 4 * RPW;     // streams per workgroup
    __shared__ float part[NSTREAM][D + 2];
    const DecodeLayout L = decode_layout(c);
    const int bh = blockIdx.x;
    const int b = bh / c.H, h = bh % c.H;
    const int row = b * c.Gu + (c.Gu == 1 ? 0 : h);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int sub = lane % LPR, grp = lane / LPR;
    const int stream = wv * RPW + grp;
    const float* slot_u = (const float*)(st + L.slot_u) + (size_t)row * L.NS;
    const float tau = *((const float*)(st + L.tau_f) + row);
    const T* ks = (const T*)(st + L.kslots) + (size_t)bh * L.NS * D;
    const T* vs = (const T*)(st + L.vslots) + (size_t)bh * L.NS * D;
    float qf[8];
    Ld8<T>::ld(q_new + (size_t)bh * D + sub * 8, qf);
    const float c2 = c.softmax_scale * 1.4426950408889634f;
#pragma unroll
    for (int e = 0; e < 8; e++) qf[e] *= c2;

    float m_run = -INFINITY, l_run = 0.0f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] = 0.0f;

    constexpr int UNR = 4;
    for (int s0 = stream; s0 < L.NS; s0 += NSTREAM * UNR) {
        float kf[UNR][8], vf[UNR][8], su[UNR];
#pragma unroll
        for (int x = 0; x < UNR; x++) {
            const int s = s0 + x * NSTREAM;
            const bool in = s < L.NS;
            const int sc = in ? s : 0;
            su[x] = in ? slot_u[sc] : -INFINITY;
            Ld8<T>::ld(ks + (size_t)sc * D + sub * 8, kf[x]);
            Ld8<T>::ld(vs + (size_t)sc * D + sub * 8, vf[x]);
        }
#pragma unroll
        for (int x = 0; x < UNR; x++) {
            float dot = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; e++) dot += qf[e] * kf[x][e];
#pragma unroll
            for (int off = 1; off < LPR; off <<= 1) dot += __shfl_xor(dot, off, 64);
            const bool valid = su[x] > -INFINITY;
            const float g = clip01(su[x] - tau);  // +inf -> 1
            float s2 = (MODE == 0) ? dot * g : dot;
            s2 = valid ? s2 : -INFINITY;
            const float m_new = fmaxf(m_run, s2);
            const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
            const float alpha = exp2f(m_run - m_safe);
            const float p = exp2f(s2 - m_safe);
            const float pv = (MODE == 2) ? p : p * g;
            l_run = l_run * alpha + p;
#pragma unroll
            for (int e = 0; e < 8; e++) acc[e] = acc[e] * alpha + pv * vf[x][e];
            m_run = m_new;
        }
    }
    // ---- merge the streams ----
    if (sub == 0) { part[stream][D] = m_run; part[stream][D + 1] = l_run; }
#pragma unroll
    for (int e = 0; e < 8; e++) part[stream][sub * 8 + e] = acc[e];
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY;
        for (int s = 0; s < NSTREAM; s++) M = fmaxf(M, part[s][D]);
        float lsum = 0.0f, osum = 0.0f;
        for (int s = 0; s < NSTREAM; s++) {
            const float ms = part[s][D];
            const float f = (ms == -INFINITY) ? 0.0f : exp2f(ms - M);
            lsum += f * part[s][D + 1];
            osum += f * part[s][tid];
        }
        st1(o + (size_t)bh * D + tid, osum / lsum);
    }
}

// ---------------------------------------------------------------------------------
// init / load
// ---------------------------------------------------------------------------------
// Empty slots are skipped through their gate score (-inf) but their rows are still streamed and
// multiplied by a zero weight, so they must hold finite numbers: clear slots [first, NS) of every head.
__global__ __launch_bounds__(256) void decode_zero_slots_kernel(sparsek_decode_cfg c, char* st, int from_state)
{
    const DecodeLayout L = decode_layout(c);
    const int bh = blockIdx.x;
    const int b = bh / c.H, h = bh % c.H;
    const int row = b * c.Gu + (c.Gu == 1 ? 0 : h);
    const int first = from_state ? L.NS - *((const int*)(st + L.nfree) + row) : 0;
    const size_t esz = c.dtype == SPARSEK_BF16 ? 2 : 4;
    const size_t row_bytes = (size_t)c.d * esz;
    uint4* kd = (uint4*)(st + L.kslots + ((size_t)bh * L.NS + first) * row_bytes);
    uint4* vd = (uint4*)(st + L.vslots + ((size_t)bh * L.NS + first) * row_bytes);
    const size_t nchunk = (size_t)(L.NS - first) * row_bytes / 16;
    for (size_t x = threadIdx.x + (size_t)blockIdx.y * 256; x < nchunk; x += (size_t)gridDim.y * 256) {
        kd[x] = make_uint4(0, 0, 0, 0);
        vd[x] = make_uint4(0, 0, 0, 0);
    }
}

__global__ __launch_bounds__(NT_ROW) void decode_init_kernel(sparsek_decode_cfg c, char* st)
{
    const DecodeLayout L = decode_layout(c);
    const int row = blockIdx.x, tid = threadIdx.x;
    RowState R = row_state(st, L, row);
    for (int s = tid; s < L.NS; s += NT_ROW) {
        R.slot_u[s] = -INFINITY;
        R.free_stack[s] = L.NS - 1 - s;  // slot 0 is popped first
    }
    if (tid == 0) {
        *R.pos = 0; *R.nsel = 0; *R.ncand = 0; *R.status = 0; *R.nfree = L.NS; *R.new_slot = -1;
        *R.tau_d = 0.0; *R.tau_f = 0.0f;
    }
}

// State after positions 0..n_ctx-1: selected = top-k of prefix T = n_ctx-1-w, window = last w.
__global__ __launch_bounds__(NT_ROW) void decode_load_kernel(sparsek_decode_cfg c, char* st, int n_ctx,
                                                             const float* __restrict__ u,
                                                             const float* __restrict__ tau,
                                                             const int32_t* __restrict__ death)
{
    __shared__ BlockRed red;
    __shared__ int scan[NT_ROW / 64];
    __shared__ int base_s[2];
    const DecodeLayout L = decode_layout(c);
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    RowState R = row_state(st, L, row);
    const int k = c.k, w = c.w;
    const float* ur = u + (size_t)row * n_ctx;
    const int32_t* dr = death + (size_t)row * n_ctx;
    const int Tp = n_ctx - 1 - w;
    const float tau_f = (Tp >= 0) ? tau[(size_t)row * n_ctx + Tp] : 0.0f;
    // start a little below the fp32 threshold, then re-solve exactly in fp64
    const double tau_lo = (double)tau_f - 1e-5 * fmax(1.0, fabs((double)tau_f));
    const bool long_prefix = (k > 0) && (Tp + 1 > k);
    for (int s = tid; s < L.NS; s += NT_ROW) R.slot_u[s] = -INFINITY;
    if (tid == 0) { base_s[0] = 0; base_s[1] = 0; *R.status = 0; }
    __syncthreads();
    // ---- selected keys (ascending position -> slots 0..nsel-1) and candidates ----
    for (int j0 = 0; j0 <= Tp; j0 += NT_ROW) {
        const int j = j0 + tid;
        const bool in = j <= Tp;
        const float uj = in ? ur[j] : 0.0f;
        const bool sel = in && k > 0 && dr[j] > Tp;
        const bool cand = in && !sel && long_prefix && ((double)uj > tau_lo);
        const unsigned long long bs = __ballot(sel), bc = __ballot(cand);
        if (lane == 0) { scan[wv] = __popcll(bs) | (__popcll(bc) << 16); }
        __syncthreads();
        int os = base_s[0], oc = base_s[1];
        for (int x = 0; x < wv; x++) { os += scan[x] & 0xFFFF; oc += scan[x] >> 16; }
        if (sel) {
            const int e = os + __popcll(bs & ((1ull << lane) - 1ull));
            R.sel_u[e] = uj; R.sel_pos[e] = j; R.sel_slot[e] = e; R.slot_u[e] = uj;
        }
        if (cand) {
            const int e = oc + __popcll(bc & ((1ull << lane) - 1ull));
            if (e < L.cap) R.cand_u[e] = uj;
        }
        __syncthreads();
        if (tid == 0) {
            for (int x = 0; x < NT_ROW / 64; x++) { base_s[0] += scan[x] & 0xFFFF; base_s[1] += scan[x] >> 16; }
        }
        __syncthreads();
    }
    const int nsel = base_s[0];
    int ncand = base_s[1];
    if (ncand > L.cap) {  // keeps the first cap in position order; tau becomes approximate
        ncand = L.cap;
        if (tid == 0) atomicOr(R.status, 1);
    }
    __syncthreads();
    // ---- exact fp64 threshold of prefix Tp ----
    double tau_d = 0.0;
    if (Tp >= 0) {
        if (k == 0) tau_d = (double)tau_f;
        else if (!long_prefix) tau_d = (double)tau_f;  // min(prefix) - 1: exact in fp32
        else tau_d = block_solve_tau(red, R.sel_u, nsel, R.cand_u, ncand, false, 0.0f, k, tau_lo, R.status);
    }
    if (long_prefix) ncand = block_prune(scan, R.cand_u, ncand, 0.0f, tau_d);
    // ---- window: positions max(0, n_ctx-w) .. n_ctx-1 -> slots nsel.. ----
    const int wb = max(0, n_ctx - w);
    const int nwin = n_ctx - wb;
    for (int i = tid; i < nwin; i += NT_ROW) {
        const int p = wb + i;
        R.win_u[p % w] = ur[p];
        R.win_slot[p % w] = nsel + i;
        R.slot_u[nsel + i] = INFINITY;
    }
    const int used = nsel + nwin;
    for (int s = tid; s < L.NS - used; s += NT_ROW) R.free_stack[s] = L.NS - 1 - s;  // pops `used` first
    if (tid == 0) {
        *R.pos = n_ctx; *R.nsel = nsel; *R.ncand = ncand; *R.nfree = L.NS - used; *R.new_slot = -1;
        *R.tau_d = tau_d; *R.tau_f = (float)tau_d;
    }
}

// K/V rows of the loaded positions, one workgroup per head, 16-byte copies.
template <typename T>
__global__ __launch_bounds__(256) void decode_load_kv_kernel(sparsek_decode_cfg c, char* st, int n_ctx,
                                                             const T* __restrict__ kk, const T* __restrict__ vv)
{
    const DecodeLayout L = decode_layout(c);
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int b = bh / c.H, h = bh % c.H;
    const int row = b * c.Gu + (c.Gu == 1 ? 0 : h);
    RowState R = row_state(st, L, row);
    const int nsel = *R.nsel;
    const int used = L.NS - *R.nfree;
    const int wb = max(0, n_ctx - c.w);
    const int cpr = c.d * (int)sizeof(T) / 16;  // 16-byte chunks per row
    const uint4* ksrc = (const uint4*)(kk + (size_t)bh * n_ctx * c.d);
    const uint4* vsrc = (const uint4*)(vv + (size_t)bh * n_ctx * c.d);
    uint4* kdst = (uint4*)((T*)(st + L.kslots) + (size_t)bh * L.NS * c.d);
    uint4* vdst = (uint4*)((T*)(st + L.vslots) + (size_t)bh * L.NS * c.d);
    for (int x = tid; x < used * cpr; x += 256) {
        const int s = x / cpr, cc = x % cpr;
        const int p = (s < nsel) ? R.sel_pos[s] : wb + (s - nsel);
        kdst[(size_t)s * cpr + cc] = ksrc[(size_t)p * cpr + cc];
        vdst[(size_t)s * cpr + cc] = vsrc[(size_t)p * cpr + cc];
    }
}

// ---------------------------------------------------------------------------------
int launch_decode_init(const sparsek_decode_cfg& c, void* state, hipStream_t st)
{
    if (c.d != 32 && c.d != 64 && c.d != 128) return SPARSEK_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(decode_init_kernel, dim3(c.B * c.Gu), dim3(NT_ROW), 0, st, c, (char*)state);
    hipLaunchKernelGGL(decode_zero_slots_kernel, dim3(c.B * c.H, 4), dim3(256), 0, st, c, (char*)state, 0);
    return launch_status();
}

int launch_decode_load(const sparsek_decode_cfg& c, void* state, int n_ctx, const void* k, const void* v,
                       const float* u, const float* tau, const int32_t* death, hipStream_t st)
{
    if (c.d != 32 && c.d != 64 && c.d != 128) return SPARSEK_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(decode_load_kernel, dim3(c.B * c.Gu), dim3(NT_ROW), 0, st, c, (char*)state, n_ctx, u, tau,
                       death);
    if (c.dtype == SPARSEK_BF16)
        hipLaunchKernelGGL(decode_load_kv_kernel<uint16_t>, dim3(c.B * c.H), dim3(256), 0, st, c, (char*)state,
                           n_ctx, (const uint16_t*)k, (const uint16_t*)v);
    else
        hipLaunchKernelGGL(decode_load_kv_kernel<float>, dim3(c.B * c.H), dim3(256), 0, st, c, (char*)state,
                           n_ctx, (const float*)k, (const float*)v);
    hipLaunchKernelGGL(decode_zero_slots_kernel, dim3(c.B * c.H, 4), dim3(256), 0, st, c, (char*)state, 1);
    return launch_status();
}

template <typename T, int LPR>
static void launch_attn_t(const sparsek_decode_cfg& c, const void* state, const void* q, void* o, hipStream_t st)
{
    dim3 grid(c.B * c.H);
    if (c.gate_mode == 0)
        hipLaunchKernelGGL((decode_attn_kernel<T, LPR, 0>), grid, dim3(256), 0, st, c, (const char*)state,
                           (const T*)q, (T*)o);
    else if (c.gate_mode == 1)
        hipLaunchKernelGGL((decode_attn_kernel<T, LPR, 1>), grid, dim3(256), 0, st, c, (const char*)state,
                           (const T*)q, (T*)o);
    else
        hipLaunchKernelGGL((decode_attn_kernel<T, LPR, 2>), grid, dim3(256), 0, st, c, (const char*)state,
                           (const T*)q, (T*)o);
}

int launch_decode_step(const sparsek_decode_cfg& c, void* state, const void* q, const void* k, const void* v,
                       const float* u_new, void* o, hipStream_t st)
{
    if (c.d != 32 && c.d != 64 && c.d != 128) return SPARSEK_ERR_UNSUPPORTED;
    if (c.dtype == SPARSEK_BF16) {
        hipLaunchKernelGGL(decode_update_kernel<uint16_t>, dim3(c.B * c.Gu), dim3(NT_ROW), 0, st, c, (char*)state,
                           (const uint16_t*)k, (const uint16_t*)v, u_new);
        if (c.d == 128) launch_attn_t<uint16_t, 16>(c, state, q, o, st);
        else if (c.d == 64) launch_attn_t<uint16_t, 8>(c, state, q, o, st);
        else launch_attn_t<uint16_t, 4>(c, state, q, o, st);
    } else {
        hipLaunchKernelGGL(decode_update_kernel<float>, dim3(c.B * c.Gu), dim3(NT_ROW), 0, st, c, (char*)state,
                           (const float*)k, (const float*)v, u_new);
        if (c.d == 128) launch_attn_t<float, 16>(c, state, q, o, st);
        else if (c.d == 64) launch_attn_t<float, 8>(c, state, q, o, st);
        else launch_attn_t<float, 4>(c, state, q, o, st);
    }
    return launch_status();
}

int decode_status(const sparsek_decode_cfg& c, const void* state, int32_t* host_flags, hipStream_t st)
{
    const DecodeLayout L = decode_layout(c);
    if (hipMemcpyAsync(host_flags, (const char*)state + L.status, (size_t)L.rows * 4, hipMemcpyDeviceToHost, st) !=
        hipSuccess)
        return SPARSEK_ERR_LAUNCH;
    if (hipStreamSynchronize(st) != hipSuccess) return SPARSEK_ERR_LAUNCH;
    return SPARSEK_OK;
}

}  // namespace spk

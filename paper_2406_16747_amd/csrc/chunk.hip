// Chunk-wise recurrent prefill with a fixed-size scored cache (Sec. 3.4, "training with
// fixed-size truncation-free cache": attend the chunk against the cache, add the chunk's
// key-value pairs and scores, prune by score).  The result equals the unchunked computation.
//
// What must survive a chunk is decided by the SPARSEK threshold, which never decreases: a key
// whose score is not above the threshold of the last prefix used so far can neither be selected
// again nor enter the support of a later threshold.  So the state keeps, per score row and in
// position order, the scores of (a) every key older than the window that is still above that
// threshold (the top-k are among them) and (b) the last w keys, together with their K/V rows:
// at most R_cap = k + w + cand_cap entries, independent of the sequence length.
//
// A call builds a "virtual sequence"  [ padding | retained entries | chunk ]  of fixed length
// R_cap + c, runs the ordinary mask and attention kernels on it (only the chunk's queries are
// evaluated) and compacts the survivors back into the state.  Inside the virtual sequence
// distances of at most w are preserved (the last w retained entries are the true window), and
// dropped keys cannot change any threshold or selection, so every chunk query sees exactly the
// keys and gates of the unchunked run.  The padding carries scores 2 below every real one: it
// never enters a support once k real keys exist; while fewer exist the real gates are all 1, as
// they must be, and the padding itself is kept out of every query's key set (lifetimes cleared,
// and the attention kernel is told the first real position, so its window stops there).
#include "common.hpp"

namespace spk {

struct ChunkLayout {
    int rcap;                              // capacity of the retained set (multiple of 128)
    size_t count, flags, ret_u, ret_sel, ret_k, ret_v, total;
};

static int chunk_rcap(const sparsek_chunk_cfg& c)
{
    const int cand = c.cand_cap > 0 ? c.cand_cap : 4 * (c.k > 16 ? c.k : 16);
    return (c.k + c.w + cand + 127) / 128 * 128;
}

static size_t esize(int dtype) { return dtype == SPARSEK_BF16 ? 2 : 4; }

static ChunkLayout chunk_layout(const sparsek_chunk_cfg& c)
{
    ChunkLayout L;
    L.rcap = chunk_rcap(c);
    const size_t rows = (size_t)c.B * c.Gu, BH = (size_t)c.B * c.H;
    size_t off = 0;
    L.count = off; off += align_up(rows * 4, 256);
    L.flags = off; off += align_up(rows * 4, 256);
    L.ret_u = off; off += align_up(rows * L.rcap * 4, 256);
    L.ret_sel = off; off += align_up(rows * L.rcap * 4, 256);
    L.ret_k = off; off += align_up(BH * L.rcap * c.d * esize(c.dtype), 256);
    L.ret_v = off; off += align_up(BH * L.rcap * c.d * esize(c.dtype), 256);
    L.total = off;
    return L;
}

size_t chunk_state_bytes(const sparsek_chunk_cfg& c) { return chunk_layout(c).total; }

static sparsek_cfg virtual_cfg(const sparsek_chunk_cfg& c, int nv)
{
    sparsek_cfg v;
    v.B = c.B; v.H = c.H; v.Gu = c.Gu; v.n = nv; v.d = c.d; v.k = c.k; v.w = c.w;
    v.dtype = c.dtype;
    v.gate_mode = c.gate_mode == 3 ? 2 : c.gate_mode;
    v.softmax_scale = c.softmax_scale;
    return v;
}

struct ChunkWs {
    size_t u, tau, death, map, first, lse, k, v, mask, attn, total;
};
static ChunkWs chunk_ws(const sparsek_chunk_cfg& c, int clen)
{
    const ChunkLayout L = chunk_layout(c);
    const int nv = L.rcap + clen;
    const size_t rows = (size_t)c.B * c.Gu, BH = (size_t)c.B * c.H;
    const sparsek_cfg v = virtual_cfg(c, nv);
    ChunkWs W;
    size_t off = 0;
    W.u = off; off += align_up(rows * nv * 4, 256);
    W.tau = off; off += align_up(rows * nv * 4, 256);
    W.death = off; off += align_up(rows * nv * 4, 256);
    W.map = off; off += align_up(rows * L.rcap * 4, 256);
    W.first = off; off += align_up(rows * 4, 256);
    W.lse = off; off += align_up(BH * (size_t)clen * 4, 256);
    const size_t tens = align_up(BH * nv * c.d * esize(c.dtype), 256);
    W.k = off; off += tens;
    W.v = off; off += tens;
    W.mask = off; off += align_up(mask_ws_bytes(v), 256);
    W.attn = off; off += align_up(attn_fwd_ws_bytes(v), 256);
    W.total = off;
    return W;
}
size_t chunk_ws_bytes(const sparsek_chunk_cfg& c) { return chunk_ws(c, c.chunk_max).total; }

__global__ void chunk_init_kernel(int32_t* count, int32_t* flags, int rows)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) { count[i] = 0; flags[i] = 0; }
}

// Scores of the virtual sequence of one row: padding (min - 2), retained, chunk.
__global__ __launch_bounds__(1024) void chunk_assemble_scores_kernel(const int32_t* __restrict__ count,
                                                                     const float* __restrict__ ret_u,
                                                                     const float* __restrict__ u_chunk, int rcap,
                                                                     int clen, float* __restrict__ u_v,
                                                                     int32_t* __restrict__ first_valid)
{
    __shared__ float red[16];
    const int row = blockIdx.x, tid = threadIdx.x;
    const int R = count[row];
    const int pad = rcap - R, nv = rcap + clen;
    if (tid == 0) first_valid[row] = pad;
    const float* ru = ret_u + (size_t)row * rcap;
    const float* cu = u_chunk + (size_t)row * clen;
    float mn = INFINITY;
    for (int i = tid; i < R; i += 1024) mn = fminf(mn, ru[i]);
    for (int i = tid; i < clen; i += 1024) mn = fminf(mn, cu[i]);
    mn = wave_min_f32(mn);
    if ((tid & 63) == 0) red[tid >> 6] = mn;
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int i = 1; i < 16; i++) m = fminf(m, red[i]);
    const float dummy = m - 2.0f;
    float* out = u_v + (size_t)row * nv;
    for (int e = tid; e < nv; e += 1024) out[e] = e < pad ? dummy : e < rcap ? ru[e - pad] : cu[e - rcap];
}

// K and V rows of the virtual sequence of one head (16 bytes per thread and step).  Padding rows
// are zero.  (Q and O stay in the caller's chunk tensors: the attention kernel addresses them from
// its first query.)
__global__ __launch_bounds__(256) void chunk_assemble_rows_kernel(
    const int32_t* __restrict__ count, const uint4* __restrict__ ret_k, const uint4* __restrict__ ret_v,
    const uint4* __restrict__ k_c, const uint4* __restrict__ v_c, int H, int Gu, int rcap, int clen,
    int row16 /* 16-byte units per row */, uint4* __restrict__ k_v, uint4* __restrict__ v_v)
{
    const int bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const int pad = rcap - count[row], nv = rcap + clen;
    const size_t total = (size_t)nv * row16;
    for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < total; x += (size_t)gridDim.x * 256) {
        const int e = (int)(x / row16), c16 = (int)(x % row16);
        const size_t dst = ((size_t)bh * nv + e) * row16 + c16;
        uint4 kk = make_uint4(0, 0, 0, 0), vv = kk;
        if (e >= rcap) {
            const size_t src = ((size_t)bh * clen + (e - rcap)) * row16 + c16;
            kk = k_c[src];
            vv = v_c[src];
        } else if (e >= pad) {
            const size_t src = ((size_t)bh * rcap + (e - pad)) * row16 + c16;
            kk = ret_k[src];
            vv = ret_v[src];
        }
        k_v[dst] = kk;
        v_v[dst] = vv;
    }
}

// Padding entries are never selected: death[e] = e.  The same holds for retained keys that were
// kept only because their score is above the threshold: they left the top-k in an earlier chunk, at
// a prefix whose block the mask skips, so their lifetime is still at its preset.
__global__ void chunk_clear_padding_kernel(const int32_t* __restrict__ count, const int32_t* __restrict__ ret_sel,
                                           int rcap, int nv, int32_t* __restrict__ death)
{
    const int row = blockIdx.y;
    const int pad = rcap - count[row];
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rcap) return;
    if (e < pad || !ret_sel[(size_t)row * rcap + (e - pad)]) death[(size_t)row * nv + e] = e;
}

// Exclusive prefix sums of two counters over the 1024 threads of a workgroup.
__device__ __forceinline__ void block_scan2_1024(int a, int b, int (*wt)[16], int& ea, int& eb, int& ta, int& tb)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int ia = a, ib = b;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int ya = __shfl_up(ia, o, 64), yb = __shfl_up(ib, o, 64);
        if (lane >= o) { ia += ya; ib += yb; }
    }
    __syncthreads();
    if (lane == 63) { wt[0][wv] = ia; wt[1][wv] = ib; }
    __syncthreads();
    ea = ia - a; eb = ib - b; ta = 0; tb = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) {
        if (i < wv) { ea += wt[0][i]; eb += wt[1][i]; }
        ta += wt[0][i]; tb += wt[1][i];
    }
}

// The survivors of one row, in position order: the last w entries, the keys still selected for the
// last prefix used so far (T = nv - 1 - w) and every other real key whose score is above that
// prefix's threshold.  The first two classes always fit; if the third does not, its oldest members
// are dropped and bit 0 of the row's flag word is set (later thresholds are then approximate).
constexpr int RETAIN_LDS = 48 * 1024;  // classes of up to this many virtual positions are cached in LDS

__global__ __launch_bounds__(1024) void chunk_retain_kernel(int32_t* __restrict__ count, int32_t* __restrict__ flags,
                                                            const float* __restrict__ u_v,
                                                            const float* __restrict__ tau_v,
                                                            const int32_t* __restrict__ death_v, int rcap, int clen,
                                                            int w, int32_t* __restrict__ map, float* __restrict__ ret_u,
                                                            int32_t* __restrict__ ret_sel)
{
    __shared__ int wt[2][16];
    __shared__ unsigned char cls[RETAIN_LDS];
    const int row = blockIdx.x, tid = threadIdx.x;
    const int nv = rcap + clen;
    const int pad = rcap - count[row];
    const int T = nv - 1 - w;  // last prefix any query has used
    const bool cached = nv <= RETAIN_LDS;
    const float* ur = u_v + (size_t)row * nv;
    const int32_t* dr = death_v + (size_t)row * nv;
    const float thr = T >= pad ? tau_v[(size_t)row * nv + T] : -INFINITY;
    // class 1: mandatory (window, or selected for prefix T); class 2: other keys above the threshold
    auto classify = [&](int e) -> int {
        if (e < pad || e >= nv) return 0;
        if (e > T) return 1;
        if (dr[e] > T) return 1;
        return ur[e] > thr ? 2 : 0;
    };
    int n1 = 0, n2 = 0;
    for (int e = tid; e < nv; e += 1024) {
        const int c = classify(e);
        if (cached) cls[e] = (unsigned char)c;
        n1 += c == 1;
        n2 += c == 2;
    }
    int e1, e2, t1, t2;
    block_scan2_1024(n1, n2, wt, e1, e2, t1, t2);  // (its barriers also publish cls[])
    const int allowed = rcap - t1;        // >= 0: the mandatory classes hold at most k + w entries
    const int drop = t2 > allowed ? t2 - allowed : 0;  // the oldest `drop` members of class 2 go
    // second pass in position order: contiguous slices per thread keep the order
    const int per = (nv + 1023) / 1024;
    const int b0 = min(tid * per, nv), b1 = min(b0 + per, nv);
    int c1 = 0, c2 = 0;
    for (int e = b0; e < b1; e++) {
        const int c = cached ? cls[e] : classify(e);
        c1 += c == 1;
        c2 += c == 2;
    }
    int p1, p2, u1, u2;
    block_scan2_1024(c1, c2, wt, p1, p2, u1, u2);
    for (int e = b0; e < b1; e++) {
        const int c = cached ? cls[e] : classify(e);
        if (c == 0) continue;
        const bool keep = c == 1 || p2 >= drop;
        if (keep) {
            const int kept2 = p2 > drop ? p2 - drop : 0;  // class-2 survivors before e
            const int j = p1 + kept2;
            map[(size_t)row * rcap + j] = e;
            ret_u[(size_t)row * rcap + j] = ur[e];
            ret_sel[(size_t)row * rcap + j] = c == 1;
        }
        p1 += c == 1;
        p2 += c == 2;
    }
    if (tid == 0) {  // every thread has read the old count (before the first scan's barriers)
        count[row] = t1 + t2 - drop;
        if (drop > 0) flags[row] |= 1;
    }
}

__global__ __launch_bounds__(256) void chunk_retain_rows_kernel(const int32_t* __restrict__ count,
                                                                const int32_t* __restrict__ map,
                                                                const uint4* __restrict__ k_v,
                                                                const uint4* __restrict__ v_v, int H, int Gu, int rcap,
                                                                int nv, int row16, uint4* __restrict__ ret_k,
                                                                uint4* __restrict__ ret_v)
{
    const int bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int row = b * Gu + (Gu == 1 ? 0 : h);
    const size_t total = (size_t)count[row] * row16;
    for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < total; x += (size_t)gridDim.x * 256) {
        const int j = (int)(x / row16), c16 = (int)(x % row16);
        const int e = map[(size_t)row * rcap + j];
        const size_t src = ((size_t)bh * nv + e) * row16 + c16;
        const size_t dst = ((size_t)bh * rcap + j) * row16 + c16;
        ret_k[dst] = k_v[src];
        ret_v[dst] = v_v[src];
    }
}

int launch_chunk_init(const sparsek_chunk_cfg& c, void* state, hipStream_t st)
{
    const ChunkLayout L = chunk_layout(c);
    const int rows = c.B * c.Gu;
    char* s = (char*)state;
    hipLaunchKernelGGL(chunk_init_kernel, dim3((rows + 255) / 256), dim3(256), 0, st, (int32_t*)(s + L.count),
                       (int32_t*)(s + L.flags), rows);
    return launch_status();
}

int launch_chunk_prefill(const sparsek_chunk_cfg& c, void* state, int clen, const void* q, const void* k,
                         const void* v, const float* u, void* o, void* ws, hipStream_t st)
{
    const ChunkLayout L = chunk_layout(c);
    const ChunkWs W = chunk_ws(c, clen);
    const int rows = c.B * c.Gu, BH = c.B * c.H;
    const int nv = L.rcap + clen;
    const int row16 = (int)(c.d * esize(c.dtype) / 16);
    char* s = (char*)state;
    char* w = (char*)ws;
    int32_t* count = (int32_t*)(s + L.count);
    int32_t* flags = (int32_t*)(s + L.flags);
    float* ret_u = (float*)(s + L.ret_u);
    uint4* ret_k = (uint4*)(s + L.ret_k);
    uint4* ret_v = (uint4*)(s + L.ret_v);
    float* u_v = (float*)(w + W.u);
    float* tau_v = (float*)(w + W.tau);
    int32_t* death_v = (int32_t*)(w + W.death);
    int32_t* map = (int32_t*)(w + W.map);
    int32_t* first_valid = (int32_t*)(w + W.first);
    uint4* k_v = (uint4*)(w + W.k);
    uint4* v_v = (uint4*)(w + W.v);
    const sparsek_cfg cv = virtual_cfg(c, nv);

    hipLaunchKernelGGL(chunk_assemble_scores_kernel, dim3(rows), dim3(1024), 0, st, count, ret_u, u, L.rcap, clen, u_v,
                       first_valid);
    const int gx = (int)std::min<size_t>(((size_t)nv * row16 + 255) / 256, 2048);
    hipLaunchKernelGGL(chunk_assemble_rows_kernel, dim3(gx, BH), dim3(256), 0, st, count, ret_k, ret_v, (const uint4*)k,
                       (const uint4*)v, c.H, c.Gu, L.rcap, clen, row16, k_v, v_v);
    // thresholds are needed from prefix R_cap - w - 1 on (the last one the previous call used)
    int rc = launch_mask(cv, u_v, tau_v, death_v, w + W.mask, st, std::max(0, L.rcap - c.w - 1));
    if (rc) return rc;
    hipLaunchKernelGGL(chunk_clear_padding_kernel, dim3((L.rcap + 255) / 256, rows), dim3(256), 0, st, count,
                       (const int32_t*)(s + L.ret_sel), L.rcap, nv, death_v);
    rc = launch_attn_fwd(cv, q, k_v, v_v, u_v, tau_v, death_v, o, (float*)(w + W.lse), w + W.attn, st, L.rcap,
                         first_valid, clen);
    if (rc) return rc;
    hipLaunchKernelGGL(chunk_retain_kernel, dim3(rows), dim3(1024), 0, st, count, flags, u_v, tau_v, death_v, L.rcap,
                       clen, c.w, map, ret_u, (int32_t*)(s + L.ret_sel));
    const int gr = (int)std::min<size_t>(((size_t)L.rcap * row16 + 255) / 256, 2048);
    hipLaunchKernelGGL(chunk_retain_rows_kernel, dim3(gr, BH), dim3(256), 0, st, count, map, k_v, v_v, c.H, c.Gu,
                       L.rcap, nv, row16, ret_k, ret_v);
    return launch_status();
}

// Backward of one chunk with the cache's gradient stopped (training with chunk-wise recurrence, Algorithm 3):
// the gradients of L = sum(dO * O_chunk) with respect to the chunk's own q, k, v and scores, the retained keys
// being constants.  The forward call left the virtual sequence (scores, thresholds, lifetimes, K and V rows, lse)
// in its workspace; the ordinary backward kernels run on it with the queries offset to the chunk, and only
// keys from the chunk on receive dk, dv, du.
struct ChunkBwdWs {
    size_t du, attn, mask, total;
};
static ChunkBwdWs chunk_bwd_ws(const sparsek_chunk_cfg& c, int clen)
{
    const ChunkLayout L = chunk_layout(c);
    const int nv = L.rcap + clen;
    sparsek_cfg v = virtual_cfg(c, nv);
    ChunkBwdWs W;
    size_t off = 0;
    W.du = off; off += align_up((size_t)c.B * c.Gu * nv * 4, 256);
    W.attn = off; off += align_up(attn_bwd_ws_bytes(v), 256);
    v.gate_mode = c.gate_mode;
    W.mask = off; off += align_up(mask_bwd_ws_bytes(v), 256);
    W.total = off;
    return W;
}
size_t chunk_bwd_ws_bytes(const sparsek_chunk_cfg& c) { return chunk_bwd_ws(c, c.chunk_max).total; }

__global__ void chunk_slice_du_kernel(const float* __restrict__ du_v, int nv, int rcap, int clen, float* __restrict__ du)
{
    const int row = blockIdx.y;
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < clen; x += gridDim.x * blockDim.x)
        du[(size_t)row * clen + x] = du_v[(size_t)row * nv + rcap + x];
}

int launch_chunk_bwd(const sparsek_chunk_cfg& c, int clen, const void* q, const void* o, const void* dO,
                     const void* fwd_ws, void* dq, void* dk, void* dv, float* du, void* ws, hipStream_t st)
{
    const ChunkLayout L = chunk_layout(c);
    const ChunkWs W = chunk_ws(c, clen);
    const ChunkBwdWs Bw = chunk_bwd_ws(c, clen);
    const int rows = c.B * c.Gu;
    const int nv = L.rcap + clen;
    const char* w = (const char*)fwd_ws;
    char* b = (char*)ws;
    const float* u_v = (const float*)(w + W.u);
    const float* tau_v = (const float*)(w + W.tau);
    const int32_t* death_v = (const int32_t*)(w + W.death);
    const int32_t* first_valid = (const int32_t*)(w + W.first);
    const float* lse = (const float*)(w + W.lse);
    const void* k_v = w + W.k;
    const void* v_v = w + W.v;
    sparsek_cfg cv = virtual_cfg(c, nv);  // hard gates for gate_mode 3: what the forward computed
    int rc = launch_attn_bwd(cv, q, k_v, v_v, u_v, tau_v, death_v, o, lse, dO, dq, dk, dv, b + Bw.attn, st, L.rcap,
                             first_valid, clen);
    if (rc) return rc;
    cv.gate_mode = c.gate_mode;  // the straight-through mode has its own score gradient
    float* du_v = (float*)(b + Bw.du);
    rc = launch_mask_bwd(cv, q, k_v, v_v, u_v, tau_v, death_v, o, lse, dO, du_v, b + Bw.mask, st, L.rcap, clen,
                         std::max(0, L.rcap - c.w - 1));
    if (rc) return rc;
    hipLaunchKernelGGL(chunk_slice_du_kernel, dim3((clen + 255) / 256, rows), dim3(256), 0, st, du_v, nv, L.rcap, clen, du);
    return launch_status();
}

// Decode state after the tokens consumed so far: the retained entries alone (no chunk) form a
// virtual history whose last prefix has the true threshold and top-k, which is all the decode
// state is built from.  Needs at least k + w consumed tokens: with fewer, the padding would make
// a short prefix look long to the loader.
int launch_decode_load(const sparsek_decode_cfg& c, void* state, int n_ctx, const void* k, const void* v,
                       const float* u, const float* tau, const int32_t* death, hipStream_t st);

int launch_chunk_to_decode(const sparsek_chunk_cfg& c, void* state, void* ws, const sparsek_decode_cfg& dc,
                           void* dstate, hipStream_t st)
{
    const ChunkLayout L = chunk_layout(c);
    const ChunkWs W = chunk_ws(c, 0);
    const int rows = c.B * c.Gu, BH = c.B * c.H;
    const int nv = L.rcap;
    const int row16 = (int)(c.d * esize(c.dtype) / 16);
    char* s = (char*)state;
    char* w = (char*)ws;
    int32_t* count = (int32_t*)(s + L.count);
    float* u_v = (float*)(w + W.u);
    float* tau_v = (float*)(w + W.tau);
    int32_t* death_v = (int32_t*)(w + W.death);
    uint4* k_v = (uint4*)(w + W.k);
    uint4* v_v = (uint4*)(w + W.v);
    const sparsek_cfg cv = virtual_cfg(c, nv);
    hipLaunchKernelGGL(chunk_assemble_scores_kernel, dim3(rows), dim3(1024), 0, st, count, (const float*)(s + L.ret_u),
                       (const float*)nullptr, L.rcap, 0, u_v, (int32_t*)(w + W.first));
    const int gx = (int)std::min<size_t>(((size_t)nv * row16 + 255) / 256, 2048);
    hipLaunchKernelGGL(chunk_assemble_rows_kernel, dim3(gx, BH), dim3(256), 0, st, count, (const uint4*)(s + L.ret_k),
                       (const uint4*)(s + L.ret_v), (const uint4*)nullptr, (const uint4*)nullptr, c.H, c.Gu, L.rcap, 0,
                       row16, k_v, v_v);
    int rc = launch_mask(cv, u_v, tau_v, death_v, w + W.mask, st, std::max(0, L.rcap - c.w - 1));
    if (rc) return rc;
    hipLaunchKernelGGL(chunk_clear_padding_kernel, dim3((L.rcap + 255) / 256, rows), dim3(256), 0, st, count,
                       (const int32_t*)(s + L.ret_sel), L.rcap, nv, death_v);
    return launch_decode_load(dc, dstate, nv, k_v, v_v, u_v, tau_v, death_v, st);
}

int chunk_status(const sparsek_chunk_cfg& c, const void* state, int32_t* host_counts, int32_t* host_flags,
                 hipStream_t st)
{
    const ChunkLayout L = chunk_layout(c);
    const size_t rows = (size_t)c.B * c.Gu;
    const char* s = (const char*)state;
    if (host_counts && hipMemcpyAsync(host_counts, s + L.count, rows * 4, hipMemcpyDeviceToHost, st) != hipSuccess)
        return SPARSEK_ERR_LAUNCH;
    if (host_flags && hipMemcpyAsync(host_flags, s + L.flags, rows * 4, hipMemcpyDeviceToHost, st) != hipSuccess)
        return SPARSEK_ERR_LAUNCH;
    return hipStreamSynchronize(st) == hipSuccess ? SPARSEK_OK : SPARSEK_ERR_LAUNCH;
}

}  // namespace spk

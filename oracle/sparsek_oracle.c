/*
 * Plain CPU oracle for the SparseK attention hot path (arXiv 2406.16747).
 *
 * THIS IS TEST INFRASTRUCTURE, not the product: it is slow on purpose, follows the
 * paper's definitions step by step, computes in fp64, and shares no code, header,
 * table or helper with the HIP library.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.
 *
 * Conventions (0-indexed): n sequence length, d head dim, k selected pairs,
 * w sliding window; prefix t means scores u[0..t] (t+1 entries); query i attends the
 * window keys [max(0,i-w+1), i] with gate 1 and, when T=i-w >= 0, the hard top-k
 * keys of prefix T, each carrying its soft SPARSEK gate clip(u_j - tau_T, 0, 1)
 * (Sec. 3.2 selection equations, Sec. 3.4 sliding-window combination).
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *  - ties in the top-k use the total order "larger score first, then older first";
 *  - a prefix with at most k entries selects everything with gate 1 and stores
 *    tau = min(prefix) - 1; in general tau = sup{tau : sum clip(z - tau,0,1) >= min(k,m)},
 *    which also fixes tau on a flat segment (w* == u*) to z_(k) - 1;
 *  - k == 0: mask identically zero, tau = max(prefix);
 *  - gate_mode 0 gates keys and values (Eq. for selected attention with the soft
 *    selection matrix), 1 gates values only (Sec. 3.5 hard-K/soft-V), 2 gates nothing
 *    (hard selection, no gradient to the scores), 3 is the straight-through estimator
 *    of Sec. 3.4 applied to mode 0: the forward uses the hard selection (all gates 1,
 *    identical to mode 2) and the gradient flows through the soft selection matrix,
 *    dL/dm_ij being taken at m_ij = 1;
 *  - the softmax denominator is never re-weighted by the gate.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* SPARSEK operator: one shot, Sec. 3.3 solution + App. A.2 sweep             */
/* ------------------------------------------------------------------------- */

static int cmp_desc(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x < y) - (x > y);
}

static double clip01(double x) { return x < 0.0 ? 0.0 : (x > 1.0 ? 1.0 : x); }

/* tau for sorted coordinates zs[0..m-1] (descending) with cumulative sums
 * cs (cs[i] = zs[0]+..+zs[i-1]).  Sweeps the 2m breakpoints {z_j} U {z_j - 1} in
 * descending order (App. A.2); at each breakpoint beta the step functions
 * u(beta) = #{z >= beta+1}, w(beta) = #{z > beta} only grow, so two pointers follow
 * them, and f(beta) = sum_j clip(z_j - beta, 0, 1) = u + sum_{u<j<=w} z_(j) - (w-u) beta.
 * The sweep stops at the first breakpoint with f(beta) >= keff; the closed form
 * (Eq. for tau with u*, w*) is then applied on the segment to its right.
 * Returns u* and w* as well. */
static double tau_sorted(const double *zs, const double *cs, int m, int k, int *ustar, int *wstar)
{
    int keff = k < m ? k : m;
    if (k == 0) { /* degenerate: empty mask */
        *ustar = 0;
        *wstar = 0;
        return zs[0];
    }
    int a = 0, b = 0;   /* next breakpoint candidates: zs[a] and zs[b]-1 */
    int uu = 0, ww = 0; /* u(beta), w(beta) */
    double beta = 0.0, f = 0.0;
    while (a < m || b < m) {
        double ba = a < m ? zs[a] : -INFINITY;
        double bb = b < m ? zs[b] - 1.0 : -INFINITY;
        if (ba >= bb) { beta = ba; a++; } else { beta = bb; b++; }
        while (uu < m && zs[uu] >= beta + 1.0) uu++;
        if (ww < uu) ww = uu;
        while (ww < m && zs[ww] > beta) ww++;
        f = (double)uu + (cs[ww] - cs[uu]) - (double)(ww - uu) * beta;
        if (f >= (double)keff) break; /* reached at the latest at beta = z_(m)-1, f = m */
    }
    /* counts just to the right of beta: u' = #{z > beta+1}, w' = #{z > beta} */
    int u1 = 0, w1 = 0;
    while (u1 < m && zs[u1] > beta + 1.0) u1++;
    w1 = u1;
    while (w1 < m && zs[w1] > beta) w1++;
    double tau;
    if (w1 == u1 || f == (double)keff) {
        tau = beta; /* flat segment or exact hit: the sup of the level set is beta */
    } else {
        tau = ((cs[w1] - cs[u1]) + (double)u1 - (double)keff) / (double)(w1 - u1);
        if (tau < beta) tau = beta; /* rounding guard; the root lies in [beta, next) */
    }
    int us = 0, ws = 0;
    while (us < m && zs[us] >= tau + 1.0) us++;
    ws = us;
    while (ws < m && zs[ws] > tau) ws++;
    *ustar = us;
    *wstar = ws;
    return tau;
}

/* SPARSEK(z, k) for one vector: tau, mask p = clip(z - tau, 0, 1), u*, w*.
 * p may be NULL.  Returns 0, or -1 on bad arguments / allocation failure. */
int orc_sparsek(const float *z, int m, int k, double *tau_out, double *p, int *ustar, int *wstar)
{
    if (m < 1 || k < 0) return -1;
    double *zs = (double *)malloc(sizeof(double) * (size_t)m);
    double *cs = (double *)malloc(sizeof(double) * (size_t)(m + 1));
    if (!zs || !cs) { free(zs); free(cs); return -1; }
    for (int j = 0; j < m; j++) zs[j] = (double)z[j];
    qsort(zs, (size_t)m, sizeof(double), cmp_desc);
    cs[0] = 0.0;
    for (int j = 0; j < m; j++) cs[j + 1] = cs[j] + zs[j];
    int us, ws;
    double tau = tau_sorted(zs, cs, m, k, &us, &ws);
    *tau_out = tau;
    if (ustar) *ustar = us;
    if (wstar) *wstar = ws;
    if (p) for (int j = 0; j < m; j++) p[j] = (k == 0) ? 0.0 : clip01((double)z[j] - tau);
    free(zs);
    free(cs);
    return 0;
}

/* tau_t, u*_t, w*_t for every causal prefix t of one score row.  The sorted
 * coordinates of prefix t are those of prefix t-1 with u[t] inserted; everything
 * else is the one-shot evaluation above, redone for each prefix. */
int orc_tau_prefixes(const float *u, int n, int k, double *tau, int *ustar, int *wstar)
{
    if (n < 1 || k < 0) return -1;
    double *zs = (double *)malloc(sizeof(double) * (size_t)n);
    double *cs = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    if (!zs || !cs) { free(zs); free(cs); return -1; }
    for (int t = 0; t < n; t++) {
        double z = (double)u[t];
        int pos = t;
        while (pos > 0 && zs[pos - 1] < z) { zs[pos] = zs[pos - 1]; pos--; }
        zs[pos] = z;
        int m = t + 1;
        cs[0] = 0.0;
        for (int j = 0; j < m; j++) cs[j + 1] = cs[j] + zs[j];
        int us, ws;
        tau[t] = tau_sorted(zs, cs, m, k, &us, &ws);
        if (ustar) ustar[t] = us;
        if (wstar) wstar[t] = ws;
    }
    free(zs);
    free(cs);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Hard top-k selection (Sec. 3.2), total order: larger score, then older     */
/* ------------------------------------------------------------------------- */

/* 1 if entry a precedes entry b in the selection order */
static int precedes(const float *u, int a, int b)
{
    return (u[a] > u[b]) || (u[a] == u[b] && a < b);
}

/* sel(t): the min(k,t+1) first entries of prefix t in the selection order, written
 * in ascending position; returns their number. */
int orc_select_prefix(const float *u, int t, int k, int32_t *idx)
{
    int cnt = 0;
    for (int j = 0; j <= t; j++) {
        int before = 0;
        for (int i = 0; i <= t; i++) if (i != j && precedes(u, i, j)) before++;
        if (before < k) idx[cnt++] = j;
    }
    return cnt;
}

/* death[j]: first prefix t >= j whose top-k does not contain j (n if none).
 * j is in sel(t) iff fewer than k entries of prefix t precede it; that count only
 * grows with t, which is the irreversibility of Sec. 3.2. */
int orc_death(const float *u, int n, int k, int32_t *death)
{
    if (n < 1 || k < 0) return -1;
    for (int j = 0; j < n; j++) {
        int before = 0;
        for (int i = 0; i < j; i++) if (precedes(u, i, j)) before++;
        int dj = n;
        if (before >= k) dj = j;
        else {
            for (int t = j + 1; t < n; t++) {
                if (precedes(u, t, j)) before++;
                if (before >= k) { dj = t; break; }
            }
        }
        death[j] = dj;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Gated attention, one query, straight from the definition                   */
/* ------------------------------------------------------------------------- */

typedef struct {
    int n, d, k, w, gate_mode;
    double scale;
} orc_cfg;

/* Attention of query i over explicit key/gate lists (selected-attention equations of
 * Sec. 3.2 with the gating variants).  keys[0..nk), gates[0..nk).  o has d entries. */
static void attend_list(const float *qi, const float *K, const float *V, int d, const int *keys,
                        const double *gates, int nk, int gate_mode, double scale, double *o,
                        double *lse, double *p_out, double *qk_out)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)(nk > 0 ? nk : 1));
    double smax = -INFINITY;
    for (int a = 0; a < nk; a++) {
        const float *kj = K + (size_t)keys[a] * d;
        double dot = 0.0;
        for (int c = 0; c < d; c++) dot += (double)qi[c] * (double)kj[c];
        if (qk_out) qk_out[a] = dot;
        double gk = (gate_mode == 0) ? gates[a] : 1.0; /* modes 1, 2, 3: keys not gated */
        s[a] = scale * gk * dot;
        if (s[a] > smax) smax = s[a];
    }
    double den = 0.0;
    for (int a = 0; a < nk; a++) den += exp(s[a] - smax);
    for (int c = 0; c < d; c++) o[c] = 0.0;
    for (int a = 0; a < nk; a++) {
        double p = exp(s[a] - smax) / den;
        if (p_out) p_out[a] = p;
        double gv = (gate_mode == 2 || gate_mode == 3) ? 1.0 : gates[a];
        const float *vj = V + (size_t)keys[a] * d;
        for (int c = 0; c < d; c++) o[c] += p * gv * (double)vj[c];
    }
    if (lse) *lse = smax + log(den);
    free(s);
}

/* Key list of query i from per-prefix thresholds and lifetimes: selected part first
 * (ascending position), then the window.  Returns the list length. */
static int build_keys(const float *u, const double *tau, const int32_t *death, int i, int k, int w,
                      int *keys, double *gates)
{
    int nk = 0;
    int T = i - w;
    if (T >= 0 && k > 0) {
        for (int j = 0; j <= T; j++)
            if (death[j] > T) {
                keys[nk] = j;
                gates[nk] = clip01((double)u[j] - tau[T]);
                nk++;
            }
    }
    int lo = i - w + 1;
    if (lo < 0) lo = 0;
    for (int j = lo; j <= i; j++) {
        keys[nk] = j;
        gates[nk] = 1.0;
        nk++;
    }
    return nk;
}

/* One query, everything recomputed from scratch by definition: sort-based tau of
 * prefix T, counting-based top-k of prefix T, then the attention.  O(n^2) per call;
 * exists so that the faster whole-sequence routine below can be checked against it. */
int orc_attn_query_bydef(const float *q, const float *K, const float *V, const float *u, int n,
                         int d, int k, int w, int gate_mode, double scale, int i, double *o,
                         double *lse)
{
    if (i < 0 || i >= n || k < 0 || w < 0 || k + w < 1) return -1;
    int *keys = (int *)malloc(sizeof(int) * (size_t)(n + 1));
    double *gates = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int nk = 0;
    int T = i - w;
    if (T >= 0 && k > 0) {
        double tauT;
        orc_sparsek(u, T + 1, k, &tauT, NULL, NULL, NULL);
        int ns = orc_select_prefix(u, T, k, idx);
        for (int a = 0; a < ns; a++) {
            keys[nk] = idx[a];
            gates[nk] = clip01((double)u[idx[a]] - tauT);
            nk++;
        }
    }
    int lo = i - w + 1;
    if (lo < 0) lo = 0;
    for (int j = lo; j <= i; j++) { keys[nk] = j; gates[nk] = 1.0; nk++; }
    attend_list(q + (size_t)i * d, K, V, d, keys, gates, nk, gate_mode, scale, o, lse, NULL, NULL);
    free(keys);
    free(gates);
    free(idx);
    return 0;
}

/* Rows [i_begin, i_end) of one head, given that head's score row with its
 * thresholds and lifetimes.  o: [(i_end-i_begin), d], lse: [(i_end-i_begin)] or NULL. */
int orc_attn_rows(const float *q, const float *K, const float *V, const float *u, const double *tau,
                  const int32_t *death, int n, int d, int k, int w, int gate_mode, double scale,
                  int i_begin, int i_end, double *o, double *lse)
{
    if (i_begin < 0 || i_end > n || k < 0 || w < 0 || k + w < 1) return -1;
    int *keys = (int *)malloc(sizeof(int) * (size_t)(n + 1));
    double *gates = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    for (int i = i_begin; i < i_end; i++) {
        int nk = build_keys(u, tau, death, i, k, w, keys, gates);
        attend_list(q + (size_t)i * d, K, V, d, keys, gates, nk, gate_mode, scale,
                    o + (size_t)(i - i_begin) * d, lse ? lse + (i - i_begin) : NULL, NULL, NULL);
    }
    free(keys);
    free(gates);
    return 0;
}

/* All B*H heads; q,k,v [B,H,n,d] fp32 (bf16 inputs are widened by the caller),
 * u [B,Gu,n], tau [B,Gu,n] fp64, death [B,Gu,n].  o [B,H,n,d] fp64, lse [B,H,n].
 * Heads are independent; they are spread over nthreads OpenMP threads.
 * Returns the number of threads used, or -1. */
int orc_attn_fwd(const float *q, const float *K, const float *V, const float *u, const double *tau,
                 const int32_t *death, int B, int H, int Gu, int n, int d, int k, int w,
                 int gate_mode, double scale, double *o, double *lse, int nthreads)
{
    if (B < 1 || H < 1 || (Gu != 1 && Gu != H)) return -1;
    int used = 1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
    used = nthreads > 0 ? nthreads : omp_get_max_threads();
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; bh++) {
        int b = bh / H, h = bh % H;
        int g = (Gu == 1) ? 0 : h;
        size_t row = ((size_t)b * Gu + g) * (size_t)n;
        size_t off = (size_t)bh * n * d;
        int rc = orc_attn_rows(q + off, K + off, V + off, u + row, tau + row, death + row, n, d, k,
                               w, gate_mode, scale, 0, n, o + off, lse ? lse + (size_t)bh * n : NULL);
        if (rc) bad = 1;
    }
    return bad ? -1 : used;
}

/* ------------------------------------------------------------------------- */
/* Gradient of L = sum(dO * O) with respect to the scores u (App. A.3)        */
/* ------------------------------------------------------------------------- */

/* One head.  For every query i with T=i-w >= 0: g_j = dL/dm_ij for the selected keys
 * of prefix T (0 for everything else), then the SPARSEK Jacobian-vector product
 * s * (g - mean_{S*} g) over S*_T = {j <= T : tau_T < u_j < tau_T + 1} is added into
 * du.  The hard top-k set is treated as a constant.  du [n] is accumulated into. */
int orc_mask_bwd_head(const float *q, const float *K, const float *V, const float *u,
                      const double *tau, const int32_t *death, const float *dO, int n, int d, int k,
                      int w, int gate_mode, double scale, double *du)
{
    if (k < 0 || w < 0 || k + w < 1) return -1;
    int *keys = (int *)malloc(sizeof(int) * (size_t)(n + 1));
    double *gates = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *p = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *qk = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *g = (double *)malloc(sizeof(double) * (size_t)n);
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    for (int i = w; i < n && k > 0 && gate_mode != 2; i++) {
        int T = i - w;
        if (T + 1 <= k) continue; /* prefix with at most k entries: every gate is 1 by definition, S* is empty */
        int nk = build_keys(u, tau, death, i, k, w, keys, gates);
        attend_list(q + (size_t)i * d, K, V, d, keys, gates, nk, gate_mode, scale, o, NULL, p, qk);
        const float *dOi = dO + (size_t)i * d;
        double D = 0.0;
        for (int c = 0; c < d; c++) D += (double)dOi[c] * o[c];
        for (int j = 0; j <= T; j++) g[j] = 0.0;
        for (int a = 0; a < nk; a++) {
            int j = keys[a];
            if (j > T) continue; /* window keys carry the constant gate 1 */
            const float *vj = V + (size_t)j * d;
            double dov = 0.0;
            for (int c = 0; c < d; c++) dov += (double)dOi[c] * (double)vj[c];
            double gj = p[a] * dov; /* through the value gate */
            if (gate_mode == 0)     /* through the key gate: ds = p (m dO.v - D) */
                gj += scale * qk[a] * p[a] * (gates[a] * dov - D);
            if (gate_mode == 3)     /* straight-through: the same derivative taken at m = 1 */
                gj += scale * qk[a] * p[a] * (dov - D);
            g[j] = gj;
        }
        int cntS = 0;
        double sumg = 0.0;
        for (int j = 0; j <= T; j++) {
            double uj = (double)u[j];
            if (uj > tau[T] && uj < tau[T] + 1.0) { cntS++; sumg += g[j]; }
        }
        if (cntS == 0) continue;
        double ghat = sumg / (double)cntS;
        for (int j = 0; j <= T; j++) {
            double uj = (double)u[j];
            if (uj > tau[T] && uj < tau[T] + 1.0) du[j] += g[j] - ghat;
        }
    }
    free(keys); free(gates); free(p); free(qk); free(g); free(o);
    return 0;
}

/* All heads; du [B,Gu,n] fp64 is zeroed, then every head adds into its group's row. */
int orc_mask_bwd(const float *q, const float *K, const float *V, const float *u, const double *tau,
                 const int32_t *death, const float *dO, int B, int H, int Gu, int n, int d, int k,
                 int w, int gate_mode, double scale, double *du, int nthreads)
{
    if (B < 1 || H < 1 || (Gu != 1 && Gu != H)) return -1;
    memset(du, 0, sizeof(double) * (size_t)B * Gu * n);
    int used = 1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
    used = nthreads > 0 ? nthreads : omp_get_max_threads();
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; bh++) {
        int b = bh / H, h = bh % H;
        int g = (Gu == 1) ? 0 : h;
        size_t row = ((size_t)b * Gu + g) * (size_t)n;
        size_t off = (size_t)bh * n * d;
        double *tmp = (double *)calloc((size_t)n, sizeof(double));
        int rc = orc_mask_bwd_head(q + off, K + off, V + off, u + row, tau + row, death + row,
                                   dO + off, n, d, k, w, gate_mode, scale, tmp);
        if (rc) bad = 1;
#pragma omp critical
        for (int j = 0; j < n; j++) du[row + j] += tmp[j];
        free(tmp);
    }
    return bad ? -1 : used;
}

/* ------------------------------------------------------------------------- */
/* Gradient of L = sum(dO * O) with respect to q, k, v (the gates held fixed)   */
/* ------------------------------------------------------------------------- */

/* One head: plain backward of the selected-attention equations of Sec. 3.2 with the gating
 * variants.  With s_j = scale gk_j (q.k_j), p = softmax(s), o = sum_j p_j gv_j v_j and D = dO.o:
 *   dV_j += p_j gv_j dO,   dp_j = gv_j (dO.v_j),   ds_j = p_j (dp_j - D),
 *   dq   += ds_j scale gk_j k_j,   dK_j += ds_j scale gk_j q.
 * The scores enter only through the gates, whose gradient is orc_mask_bwd's business.
 * dQ, dK, dV [n,d] are accumulated into. */
int orc_attn_bwd_head(const float *q, const float *K, const float *V, const float *u, const double *tau,
                      const int32_t *death, const float *dO, int n, int d, int k, int w, int gate_mode,
                      double scale, double *dQ, double *dK, double *dV)
{
    if (k < 0 || w < 0 || k + w < 1) return -1;
    int *keys = (int *)malloc(sizeof(int) * (size_t)(n + 1));
    double *gates = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *p = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *qk = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    for (int i = 0; i < n; i++) {
        int nk = build_keys(u, tau, death, i, k, w, keys, gates);
        const float *qi = q + (size_t)i * d;
        const float *dOi = dO + (size_t)i * d;
        attend_list(qi, K, V, d, keys, gates, nk, gate_mode, scale, o, NULL, p, qk);
        double D = 0.0;
        for (int c = 0; c < d; c++) D += (double)dOi[c] * o[c];
        for (int a = 0; a < nk; a++) {
            int j = keys[a];
            double gk = (gate_mode == 0) ? gates[a] : 1.0;
            double gv = (gate_mode == 2 || gate_mode == 3) ? 1.0 : gates[a];
            const float *kj = K + (size_t)j * d;
            const float *vj = V + (size_t)j * d;
            double dov = 0.0;
            for (int c = 0; c < d; c++) dov += (double)dOi[c] * (double)vj[c];
            double ds = p[a] * (gv * dov - D);
            double coef = ds * scale * gk;
            for (int c = 0; c < d; c++) {
                dV[(size_t)j * d + c] += p[a] * gv * (double)dOi[c];
                dQ[(size_t)i * d + c] += coef * (double)kj[c];
                dK[(size_t)j * d + c] += coef * (double)qi[c];
            }
        }
    }
    free(keys); free(gates); free(p); free(qk); free(o);
    return 0;
}

/* All heads; dQ, dK, dV [B,H,n,d] fp64 are zeroed first. */
int orc_attn_bwd(const float *q, const float *K, const float *V, const float *u, const double *tau,
                 const int32_t *death, const float *dO, int B, int H, int Gu, int n, int d, int k,
                 int w, int gate_mode, double scale, double *dQ, double *dK, double *dV, int nthreads)
{
    if (B < 1 || H < 1 || (Gu != 1 && Gu != H)) return -1;
    size_t tot = (size_t)B * H * n * d;
    memset(dQ, 0, sizeof(double) * tot);
    memset(dK, 0, sizeof(double) * tot);
    memset(dV, 0, sizeof(double) * tot);
    int used = 1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
    used = nthreads > 0 ? nthreads : omp_get_max_threads();
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; bh++) {
        int b = bh / H, h = bh % H;
        int g = (Gu == 1) ? 0 : h;
        size_t row = ((size_t)b * Gu + g) * (size_t)n;
        size_t off = (size_t)bh * n * d;
        int rc = orc_attn_bwd_head(q + off, K + off, V + off, u + row, tau + row, death + row, dO + off, n, d,
                                   k, w, gate_mode, scale, dQ + off, dK + off, dV + off);
        if (rc) bad = 1;
    }
    return bad ? -1 : used;
}

/* ------------------------------------------------------------------------- */
/* Importance scores: scoring network + position slope (Sec. 3.2, Eq. for u),  */
/* optional timestep normalisation (Sec. 3.5, "score normalization")           */
/* ------------------------------------------------------------------------- */

/* One sequence.  X [n, D] row-major, w [D].  raw_t = X_t . w + t * slope (t counted from 0).
 * norm == 0: u_t = raw_t.
 * norm != 0: u_t = (raw_t - mean_t) / sqrt(var_t + norm_eps) with the cumulative statistics of
 * the timesteps seen so far, mean_t = (1/(t+1)) sum_{i<=t} raw_i and var_t = (1/(t+1))
 * sum_{i<=t} (raw_i - mean_t)^2, each recomputed from scratch for every t (two passes).
 * Readings (the paper only says "cumulative mean and variance for each timestep"): population
 * variance, no learnable gain or bias, norm_eps added under the root. */
int orc_scores_row(const float *X, const float *w, int n, int D, double slope, int norm,
                   double norm_eps, double *u)
{
    if (n < 1 || D < 1) return -1;
    double *raw = (double *)malloc(sizeof(double) * (size_t)n);
    for (int t = 0; t < n; t++) {
        double acc = 0.0;
        for (int c = 0; c < D; c++) acc += (double)X[(size_t)t * D + c] * (double)w[c];
        raw[t] = acc + (double)t * slope;
    }
    for (int t = 0; t < n; t++) {
        if (!norm) { u[t] = raw[t]; continue; }
        double mean = 0.0, var = 0.0;
        for (int i = 0; i <= t; i++) mean += raw[i];
        mean /= (double)(t + 1);
        for (int i = 0; i <= t; i++) var += (raw[i] - mean) * (raw[i] - mean);
        var /= (double)(t + 1);
        u[t] = (raw[t] - mean) / sqrt(var + norm_eps);
    }
    free(raw);
    return 0;
}

/* X [B, n, D], u [B, n]: every sequence on its own. */
int orc_scores(const float *X, const float *w, int B, int n, int D, double slope, int norm,
               double norm_eps, double *u)
{
    if (B < 1) return -1;
    int rc = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int b = 0; b < B; b++) {
        int r = orc_scores_row(X + (size_t)b * n * D, w, n, D, slope, norm, norm_eps, u + (size_t)b * n);
        if (r) rc = r;
    }
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Incremental evaluation (Sec. 3.3, the step-by-step algorithm with two      */
/* min-heaps) and a decode loop built on it                                   */
/* ------------------------------------------------------------------------- */

/* a binary min-heap of doubles that also keeps the sum of its entries */
typedef struct {
    double *a;
    int n, cap;
    double sum;
} orc_heap;

static int heap_init(orc_heap *h, int cap)
{
    h->a = (double *)malloc(sizeof(double) * (size_t)(cap > 0 ? cap : 1));
    h->n = 0;
    h->cap = cap;
    h->sum = 0.0;
    return h->a ? 0 : -1;
}

static void heap_push(orc_heap *h, double x)
{
    int i = h->n++;
    h->a[i] = x;
    h->sum += x;
    while (i > 0) {
        int p = (i - 1) / 2;
        if (h->a[p] <= h->a[i]) break;
        double t = h->a[p]; h->a[p] = h->a[i]; h->a[i] = t;
        i = p;
    }
}

static double heap_pop(orc_heap *h)
{
    double top = h->a[0];
    h->sum -= top;
    h->a[0] = h->a[--h->n];
    int i = 0;
    for (;;) {
        int l = 2 * i + 1, r = l + 1, m = i;
        if (l < h->n && h->a[l] < h->a[m]) m = l;
        if (r < h->n && h->a[r] < h->a[m]) m = r;
        if (m == i) break;
        double t = h->a[m]; h->a[m] = h->a[i]; h->a[i] = t;
        i = m;
    }
    return top;
}

/* State of the incremental evaluation: S holds every score above the threshold, F every score at least one above
 * it (F is a subset of S, as in the algorithm's input line); m counts the prefix. */
typedef struct {
    orc_heap S, F;
    int m, k;
    double tau, zmin, zmax;
} orc_incr;

/* One step of the algorithm: score z joins the prefix.  The threshold never decreases when a score is added, so
 * scores that left S or F never come back.  z enters the heaps it belongs to under the old threshold; then the pair
 * (u, w) = (|F|, |S|) walks downwards one breakpoint at a time: on the current linear piece the threshold is the
 * solution equation of Sec. 3.3; it is the answer if it satisfies the order conditions z_(w) > tau and
 * z_(u) >= tau + 1, i.e. lies below the nearest breakpoint (min(S), where a score drops out of the support, or
 * min(F) - 1, where a score turns fractional); otherwise that score leaves its heap and the next pair is tried.
 * A prefix of at most k scores selects everything (tau = min - 1); on a flat piece (w == u == k) the threshold is
 * the upper end of the level set, min(F) - 1. */
static double incr_step(orc_incr *st, double z)
{
    st->m++;
    if (st->m == 1 || z < st->zmin) st->zmin = z;
    if (st->m == 1 || z > st->zmax) st->zmax = z;
    if (st->k == 0) { st->tau = st->zmax; return st->tau; }
    if (st->m <= st->k) {           /* everything selected, every gate 1: all scores sit in both heaps */
        heap_push(&st->S, z);
        heap_push(&st->F, z);
        st->tau = st->zmin - 1.0;
        return st->tau;
    }
    if (z >= st->tau + 1.0) heap_push(&st->F, z);
    if (z > st->tau) heap_push(&st->S, z);
    for (;;) {
        const int u = st->F.n, w = st->S.n;
        if (w == u) {               /* no fractional score: f = u on this piece */
            if (u > st->k) { heap_pop(&st->F); continue; }   /* the threshold lies higher: min(F) turns fractional */
            st->tau = st->F.a[0] - 1.0;                       /* u == k: upper end of the level set */
            break;
        }
        double tau = ((st->S.sum - st->F.sum) + (double)u - (double)st->k) / (double)(w - u);
        if (tau < st->tau) tau = st->tau;                     /* rounding only: the threshold is monotone */
        if (tau < st->S.a[0] && (u == 0 || tau + 1.0 <= st->F.a[0])) { st->tau = tau; break; }
        if (u > 0 && st->F.a[0] - 1.0 <= st->S.a[0]) heap_pop(&st->F);
        else heap_pop(&st->S);
    }
    return st->tau;
}

/* tau of every prefix of a score row by the incremental algorithm (compare orc_tau_prefixes, which re-sorts). */
int orc_tau_incremental(const float *u, int n, int k, double *tau)
{
    if (n < 1 || k < 0) return -1;
    orc_incr st;
    memset(&st, 0, sizeof st);
    st.k = k;
    if (heap_init(&st.S, n) || heap_init(&st.F, n)) return -1;
    for (int t = 0; t < n; t++) tau[t] = incr_step(&st, (double)u[t]);
    free(st.S.a);
    free(st.F.a);
    return 0;
}

/* Decode of one head with constant work per token: positions 0..n_ctx-1 are consumed first (only their scores
 * matter), then every step t = n_ctx .. n_ctx+steps-1 appends one position: the key leaving the window (position
 * T = t - w) joins the SPARSEK prefix -- incremental threshold as above; the hard top-k as a min-heap of the k
 * selected keys in the selection order, where a newcomer replaces the weakest only with a strictly larger score --
 * and the new query attends the selected keys (gates from the current threshold) and the window.
 * q_steps [steps,d]; K, V [n_ctx+steps,d]; u [n_ctx+steps]; o [steps,d].  seconds (may be NULL) receives the time
 * spent in the steps alone, without the context. */
typedef struct {
    double z;
    int j;
} orc_selkey;

static int sel_weaker(const orc_selkey *a, const orc_selkey *b)   /* a comes after b in the selection order */
{
    return a->z < b->z || (a->z == b->z && a->j > b->j);
}

static double now_seconds(void)
{
#ifdef _OPENMP
    return omp_get_wtime();
#else
    return 0.0;
#endif
}

int orc_decode_incremental(const float *q_steps, const float *K, const float *V, const float *u, int n_ctx,
                           int steps, int d, int k, int w, int gate_mode, double scale, double *o,
                           double *seconds)
{
    if (n_ctx < 0 || steps < 1 || k < 0 || w < 0 || k + w < 1) return -1;
    const int n = n_ctx + steps;
    orc_incr st;
    memset(&st, 0, sizeof st);
    st.k = k;
    orc_selkey *sel = (orc_selkey *)malloc(sizeof(orc_selkey) * (size_t)(k > 0 ? k : 1));   /* min-heap: weakest on top */
    int nsel = 0;
    int *keys = (int *)malloc(sizeof(int) * (size_t)(k + w + 1));
    double *gates = (double *)malloc(sizeof(double) * (size_t)(k + w + 1));
    if (heap_init(&st.S, n) || heap_init(&st.F, n) || !sel || !keys || !gates) return -1;
    double t0 = 0.0;
    for (int t = 0; t < n; t++) {
        if (t == n_ctx) t0 = now_seconds();
        const int T = t - w;            /* the position that joins the prefix at this step */
        if (T >= 0) {
            incr_step(&st, (double)u[T]);
            if (k > 0) {
                orc_selkey nk = {(double)u[T], T};
                if (nsel < k) {
                    int i = nsel++;
                    sel[i] = nk;
                    while (i > 0 && sel_weaker(&sel[i], &sel[(i - 1) / 2])) {
                        orc_selkey x = sel[i]; sel[i] = sel[(i - 1) / 2]; sel[(i - 1) / 2] = x;
                        i = (i - 1) / 2;
                    }
                } else if (sel_weaker(&sel[0], &nk)) {   /* strictly larger score: equal scores keep the older key */
                    sel[0] = nk;
                    int i = 0;
                    for (;;) {
                        int l = 2 * i + 1, r = l + 1, m = i;
                        if (l < nsel && sel_weaker(&sel[l], &sel[m])) m = l;
                        if (r < nsel && sel_weaker(&sel[r], &sel[m])) m = r;
                        if (m == i) break;
                        orc_selkey x = sel[i]; sel[i] = sel[m]; sel[m] = x;
                        i = m;
                    }
                }
            }
        }
        if (t < n_ctx) continue;
        int nk = 0;
        if (T >= 0)
            for (int a = 0; a < nsel; a++) {
                keys[nk] = sel[a].j;
                gates[nk] = clip01(sel[a].z - st.tau);
                nk++;
            }
        int lo = t - w + 1;
        if (lo < 0) lo = 0;
        for (int j = lo; j <= t; j++) { keys[nk] = j; gates[nk] = 1.0; nk++; }
        attend_list(q_steps + (size_t)(t - n_ctx) * d, K, V, d, keys, gates, nk, gate_mode, scale,
                    o + (size_t)(t - n_ctx) * d, NULL, NULL, NULL);
    }
    if (seconds) *seconds = now_seconds() - t0;
    free(st.S.a);
    free(st.F.a);
    free(sel);
    free(keys);
    free(gates);
    return 0;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

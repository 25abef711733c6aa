/*
 * libsparsek -- SparseK attention hot path for AMD MI355X (gfx950), C ABI.
 *
 * Method: "Sparser is Faster and Less is More: Efficient Sparse Attention for
 * Long-Range Transformers" (arXiv 2406.16747).  Three stages, all on the GPU:
 *   (1) SPARSEK mask operator for every causal prefix of the KV importance scores
 *       (Sec. 3.3: projection onto {0<=m<=1, sum m = k}, m = clip(u - tau, 0, 1));
 *   (2) hard top-k selection per prefix (Sec. 3.2), stored compactly as one lifetime
 *       per key, which the irreversibility of the selection makes possible;
 *   (3) causal attention over the gated top-k pairs plus a sliding window (Sec. 3.2
 *       selected-attention equations, Sec. 3.4 window combination, Sec. 3.5 hard-K /
 *       soft-V variant), and the same as a constant-memory one-token decode step.
 *
 * Conventions.  0-indexed positions.  n sequence length, d head dim (64 or 128 for
 * bf16, any multiple of 4 up to 128 for fp32), k selected pairs, w window size.
 * "prefix t" = scores u[0..t].  Query i attends the window keys max(0,i-w+1)..i with
 * gate 1 and, if T = i-w >= 0, the top-k keys of prefix T with gates
 * clip(u_j - tau_T, 0, 1).  Heads h of batch b use score row (b, g) with g = 0 when
 * Gu == 1 and g = h when Gu == H.
 *
 * All tensor pointers are DEVICE pointers to caller-owned, contiguous memory; the
 * library never allocates, frees or synchronises (except sparsek_decode_status).
 * Every call validates its arguments on the host, enqueues its kernels on `stream`
 * (a hipStream_t passed as void*, NULL = the default stream) and returns at once.
 * Return value: 0 on success; a negative SPARSEK_ERR_* code when nothing was enqueued.
 * Scores must not be NaN (undefined result); -0.0 and +0.0 compare equal.
 */
#ifndef SPARSEK_H
#define SPARSEK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPARSEK_OK 0
#define SPARSEK_ERR_INVALID_ARG (-1)    /* null pointer, n<1, k<0, w<0, k+w<1, Gu not in {1,H}, bad range */
#define SPARSEK_ERR_UNSUPPORTED (-2)    /* head dim / dtype / size outside what the kernels handle (n, k, w > 2^28; decode k, w > 2^24) */
#define SPARSEK_ERR_WORKSPACE (-3)      /* workspace or state buffer smaller than the *_bytes query says */
#define SPARSEK_ERR_LAUNCH (-5)         /* the HIP runtime refused a launch */
#define SPARSEK_ERR_TOO_LARGE (-6)      /* sparsek_mask_static: the problem needs more scratch than the built-in array holds */

#define SPARSEK_F32 0
#define SPARSEK_BF16 1

/* gate_mode: where the soft gate m_ij multiplies.
 *   0  keys and values: s_ij = scale * m_ij * q_i.k_j, o_i = sum_j p_ij m_ij v_j  (soft selection matrix on K and V)
 *   1  values only:     s_ij = scale * q_i.k_j,        o_i = sum_j p_ij m_ij v_j  (Sec. 3.5)
 *   2  nowhere:         plain attention over the selected + window keys (hard selection; no gradient to the scores)
 *   3  straight-through estimator of Sec. 3.4 for mode 0: the forward is that of mode 2 (the
 *      multiplication by the gates is skipped), and sparsek_mask_bwd sends dL/dm_ij, taken at m_ij = 1,
 *      through the soft selection matrix.
 * p_i = softmax_j(s_ij) over the attended keys; the denominator is never gated. */
typedef struct {
    int32_t B, H, Gu, n, d, k, w;
    int32_t dtype;     /* SPARSEK_F32 or SPARSEK_BF16: storage type of q, k, v, o, dO */
    int32_t gate_mode; /* 0, 1, 2 or 3 */
    float softmax_scale; /* finite and > 0 */
} sparsek_cfg;

const char *sparsek_strerror(int code);

/* ---- stages 1+2: thresholds and lifetimes (Sec. 3.3 solution equations; Sec. 3.2) ----
 * u     in  [B,Gu,n] fp32 scores.
 * tau   out [B,Gu,n] fp32: tau[t] = sup{ x : sum_{j<=t} clip(u_j - x, 0, 1) >= min(k, t+1) };
 *           for t+1 <= k this is min(u[0..t]) - 1 (all gates 1); on a flat segment
 *           (w* == u*) it is z_(k) - 1; for k == 0 it is max(u[0..t]) (all gates 0).
 * death out [B,Gu,n] int32: key j belongs to the top-k of prefix t exactly for
 *           j <= t < death[j]  (death[j] == j: never selected; == n: still selected at the end).
 *           Order of the top-k: larger score first, among equal scores the older key.
 * ws    scratch of at least sparsek_mask_workspace_bytes(cfg) bytes (uses cfg->B, Gu, n, k). */
size_t sparsek_mask_workspace_bytes(const sparsek_cfg *cfg);
int sparsek_mask(const sparsek_cfg *cfg, const float *u, float *tau, int32_t *death, void *ws,
                 size_t ws_bytes, void *stream);
/* Copies the status word that the last sparsek_mask call on `ws` (same cfg) left there to *host_flag (host memory)
 * and synchronises the stream.  0: every threshold is the exact root.  bit 0: a threshold solve stopped at its
 * iteration cap (the bracket-and-bisect safeguard ran out; not observed on finite scores -- that threshold is then
 * the last iterate and may miss the 1e-5 bar).  The word is cleared at the start of every sparsek_mask call. */
int sparsek_mask_status(const sparsek_cfg *cfg, const void *ws, size_t ws_bytes, int32_t *host_flag, void *stream);

/* ---- stages 1+2 without a workspace, for callers that cannot allocate ----
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: same inputs, outputs,
 * kernels and results as sparsek_mask, but the scratch (one fp32 lower bound per 2048 positions of every score row,
 * the status word and one bit per 128 positions) lives in a 64 KiB device array built into the library, which each GPU holds until the process
 * ends.  The call allocates and frees nothing.  The current device must be the one that owns u, tau and death.
 * Limit: sparsek_mask_workspace_bytes(cfg) -- B*Gu*ceil(n/2048)*4 bytes of lower bounds, one bit per 128 positions
 * of every score row, each rounded up to 256 bytes, plus 256 -- must not exceed SPARSEK_MASK_STATIC_MAX_BYTES, e.g. 32
 * rows of 512 K scores;
 * beyond it nothing is enqueued and SPARSEK_ERR_TOO_LARGE is returned.  All calls on one GPU share the array: calls
 * that may overlap (different streams, or threads) race and must be ordered by the caller.  The status word of this
 * variant is not readable. */
#define SPARSEK_MASK_STATIC_MAX_BYTES 65536
int sparsek_mask_static(const sparsek_cfg *cfg, const float *u, float *tau, int32_t *death, void *stream);

/* ---- stage 2, explicit form (verification aid; O((t_end-t_begin)*k) memory) ----
 * For every prefix t in [t_begin, t_end): idx [B,Gu,t_end-t_begin,k] int32 = positions of the
 * top-k of prefix t in ascending order, padded with -1; gate (same shape, fp32, may be NULL)
 * = clip(u_j - tau_t, 0, 1) of those positions, 0 in the padding. */
int sparsek_materialize(const sparsek_cfg *cfg, const float *u, const float *tau,
                        const int32_t *death, int32_t t_begin, int32_t t_end, int32_t *idx,
                        float *gate, void *stream);

/* ---- stage 3: gated attention forward (Sec. 3.2, 3.4, 3.5) ----
 * q,k,v in  [B,H,n,d] of cfg->dtype;  u,tau,death as produced by sparsek_mask.
 * o     out [B,H,n,d] of cfg->dtype;  lse out [B,H,n] fp32 (natural log of the softmax
 *           denominator, including the running maximum), may be NULL.
 * ws    scratch of at least sparsek_attn_fwd_workspace_bytes(cfg) bytes. */
size_t sparsek_attn_fwd_workspace_bytes(const sparsek_cfg *cfg);
int sparsek_attn_fwd(const sparsek_cfg *cfg, const void *q, const void *k, const void *v,
                     const float *u, const float *tau, const int32_t *death, void *o, float *lse,
                     void *ws, size_t ws_bytes, void *stream);

/* ---- SPARSEK mask backward (App. A.3 Jacobian) ----
 * du out [B,Gu,n] fp32 = gradient of L = sum(dO * O) with respect to the scores through the
 * soft gates (the hard top-k set is a constant): for every prefix T, with g_j = dL/dm_{T+w,j},
 * du += s * (g - mean_{S*} g), S* = { j <= T : tau_T < u_j < tau_T + 1 }.  Heads of one score
 * group add into the same row.  o and lse are the outputs of sparsek_attn_fwd on the same inputs.
 * gate_mode 2 has no gate in the forward, so du = 0; gate_mode 3 takes g_j at gate 1 (o, lse from the
 * mode 3 forward) and applies the same Jacobian. */
size_t sparsek_mask_bwd_workspace_bytes(const sparsek_cfg *cfg);
int sparsek_mask_bwd(const sparsek_cfg *cfg, const void *q, const void *k, const void *v,
                     const float *u, const float *tau, const int32_t *death, const void *o,
                     const float *lse, const void *dO, float *du, void *ws, size_t ws_bytes,
                     void *stream);

/* ---- attention backward: gradients with respect to q, k, v (selected-attention equations of Sec. 3.2) ----
 * dq, dk, dv out [B,H,n,d] of cfg->dtype: gradient of L = sum(dO * O) with the gates held fixed; the gradient that
 * flows through the gates to the scores is sparsek_mask_bwd.  With s_ij = scale gk_ij (q_i.k_j), p = softmax_j(s),
 * o_i = sum_j p_ij gv_ij v_j and D_i = dO_i.o_i:
 *     dv_j = sum_i p_ij gv_ij dO_i,   ds_ij = p_ij (gv_ij dO_i.v_j - D_i),
 *     dq_i = sum_j ds_ij scale gk_ij k_j,   dk_j = sum_i ds_ij scale gk_ij q_i
 * (gk / gv: the gate where gate_mode puts it, else 1; gate_mode 3 differentiates its hard forward, like mode 2).
 * o, lse in: outputs of sparsek_attn_fwd on the same inputs and gate_mode; dO in [B,H,n,d] of cfg->dtype.
 * ws: scratch of at least sparsek_attn_bwd_workspace_bytes(cfg) bytes (block lists, D_i, fp32 accumulators of dk, dv). */
size_t sparsek_attn_bwd_workspace_bytes(const sparsek_cfg *cfg);
int sparsek_attn_bwd(const sparsek_cfg *cfg, const void *q, const void *k, const void *v, const float *u,
                     const float *tau, const int32_t *death, const void *o, const float *lse, const void *dO,
                     void *dq, void *dk, void *dv, void *ws, size_t ws_bytes, void *stream);

/* The whole backward of the operator in one call: dq, dk, dv as sparsek_attn_bwd and du as sparsek_mask_bwd
 * (same arguments, same results; the two parts are enqueued back to back on the stream).
 * ws: scratch of at least sparsek_bwd_workspace_bytes(cfg) bytes. */
size_t sparsek_bwd_workspace_bytes(const sparsek_cfg *cfg);
int sparsek_bwd(const sparsek_cfg *cfg, const void *q, const void *k, const void *v, const float *u,
                const float *tau, const int32_t *death, const void *o, const float *lse, const void *dO,
                void *dq, void *dk, void *dv, float *du, void *ws, size_t ws_bytes, void *stream);

/* ---- importance scores (Sec. 3.2 scoring network with position slope; Sec. 3.5 score normalisation) ----
 * u out [B,n] fp32, one row per sequence (the single score group of the paper; feed it to sparsek_mask with Gu = 1):
 *     raw_t = x_t . w + t * slope        (t counted from 0),
 *     norm == 0:  u_t = raw_t
 *     norm == 1:  u_t = (raw_t - mean_t) / sqrt(var_t + norm_eps),  mean_t / var_t = mean and population variance
 *                 of raw_0 .. raw_t (timestep normalisation: cumulative statistics, no gain or bias).
 * x  in [B,n,D] hidden states of `dtype` (SPARSEK_BF16 or SPARSEK_F32), contiguous; D a multiple of 8, D <= 8192.
 * w  in [D] fp32 scorer.  Products and sums are accumulated in fp64; u is rounded once to fp32.
 * ws scratch of at least sparsek_scores_workspace_bytes(cfg) bytes (raw scores in fp64 and block sums; unused when norm == 0).
 * Errors: INVALID_ARG for null pointers, B, n, D < 1, norm not 0/1, norm_eps <= 0 with norm == 1, non-finite slope;
 * UNSUPPORTED for D % 8 != 0, D > 8192 or another dtype. */
typedef struct {
    int32_t B, n, D;
    int32_t dtype;   /* storage type of x */
    int32_t norm;    /* 0 or 1 */
    float slope;     /* epsilon of the position slope, >= 0 in the paper */
    float norm_eps;  /* > 0 when norm == 1 */
} sparsek_scores_cfg;
size_t sparsek_scores_workspace_bytes(const sparsek_scores_cfg *cfg);
int sparsek_scores(const sparsek_scores_cfg *cfg, const void *x, const float *w, float *u, void *ws,
                   size_t ws_bytes, void *stream);

/* ---- constant-memory decode (Sec. 3.2 irreversibility; Sec. 3.3 incremental evaluation) ----
 * The state holds, per (b,h), k+w key/value slots and, per (b,g), the scores of the window,
 * of the selected keys and of every other key still above the threshold (at most cand_cap of
 * them: the bounded-heap variant of Sec. 3.3; when more would be needed the smallest are
 * dropped and bit 0 of that row's status word is set -- tau is then approximate).
 * One step appends position t: the key leaving the window (position t-w) joins the SPARSEK
 * prefix, tau and the top-k are updated incrementally, an evicted key frees its slot, and the
 * new query attends the k selected + w window slots exactly as query t of the prefill would. */
typedef struct {
    int32_t B, H, Gu, d, k, w;
    int32_t cand_cap;  /* capacity for scores above tau outside the top-k; 0 = default 4*max(k,16) */
    int32_t dtype;     /* SPARSEK_BF16 (fp32 also accepted) */
    int32_t gate_mode;
    float softmax_scale;
} sparsek_decode_cfg;

size_t sparsek_decode_state_bytes(const sparsek_decode_cfg *cfg);
/* empty context (next position 0) */
int sparsek_decode_init(const sparsek_decode_cfg *cfg, void *state, size_t state_bytes, void *stream);
/* state after consuming positions 0..n_ctx-1: k,v [B,H,n_ctx,d]; u,tau,death [B,Gu,n_ctx] from
 * sparsek_mask with the same k (tau, death may come from a longer sequence's first n_ctx entries
 * only if death was computed on exactly n_ctx entries). */
int sparsek_decode_load(const sparsek_decode_cfg *cfg, void *state, size_t state_bytes, int32_t n_ctx,
                        const void *k, const void *v, const float *u, const float *tau,
                        const int32_t *death, void *stream);
/* q_new,k_new,v_new [B,H,d]; u_new [B,Gu]; o out [B,H,d].  state is updated in place. */
int sparsek_decode_step(const sparsek_decode_cfg *cfg, void *state, const void *q_new,
                        const void *k_new, const void *v_new, const float *u_new, void *o,
                        void *stream);
/* copies the per-row status words [B*Gu] to host memory; synchronises the stream.  bit 0: candidate overflow */
int sparsek_decode_status(const sparsek_decode_cfg *cfg, const void *state, int32_t *host_flags,
                          void *stream);

/* ---- chunk-wise recurrent prefill with a fixed-size scored cache (Sec. 3.4, the chunk recurrence) ----
 * A sequence is consumed chunk by chunk; every call returns the attention output of its chunk's queries, equal to
 * rows of sparsek_attn_fwd on the whole sequence.  Between calls the state keeps, per score row and in position
 * order, the scores and (per head) the K/V rows of the last w keys, of the keys still selected and of every other
 * key whose score is still above the SPARSEK threshold: at most R_cap = k + w + cand_cap entries (rounded up to a
 * multiple of 128) whatever the sequence length.  A key outside that set can never be selected again nor move a
 * later threshold, because the threshold does not decrease.  If more than cand_cap unselected keys stay above the
 * threshold, the oldest of them are dropped and bit 0 of the row's flag word is set (thresholds are then approximate,
 * as with the bounded heap of Sec. 3.3).
 * q,k,v in [B,H,c,d], u in [B,Gu,c], o out [B,H,c,d]; 1 <= c <= chunk_max; d*sizeof(dtype) a multiple of 16.
 * state: caller-owned device buffer of sparsek_chunk_state_bytes(cfg) bytes, set up by sparsek_chunk_init;
 * ws: scratch of sparsek_chunk_workspace_bytes(cfg) bytes (sized for chunk_max).  Calls on one state must be
 * ordered on one stream.  gate_mode as in sparsek_cfg (3 runs as 2). */
typedef struct {
    int32_t B, H, Gu, d, k, w;
    int32_t cand_cap;   /* 0 = default 4*max(k,16) */
    int32_t chunk_max;  /* longest chunk of a call */
    int32_t dtype;      /* SPARSEK_BF16 or SPARSEK_F32 */
    int32_t gate_mode;
    float softmax_scale;
} sparsek_chunk_cfg;
size_t sparsek_chunk_state_bytes(const sparsek_chunk_cfg *cfg);
size_t sparsek_chunk_workspace_bytes(const sparsek_chunk_cfg *cfg);
int sparsek_chunk_init(const sparsek_chunk_cfg *cfg, void *state, size_t state_bytes, void *stream);
int sparsek_chunk_prefill(const sparsek_chunk_cfg *cfg, void *state, size_t state_bytes, int32_t c,
                          const void *q, const void *k, const void *v, const float *u, void *o, void *ws,
                          size_t ws_bytes, void *stream);
/* Backward of the chunk that the last sparsek_chunk_prefill call on `fwd_ws` processed, with the gradient of the
 * cache stopped (training with chunk-wise recurrence, Algorithm 3): for L = sum(dO * o) over the chunk's outputs,
 *     dq, dk, dv out [B,H,c,d]  gradients with respect to the chunk's own q, k, v (gates held fixed),
 *     du out [B,Gu,c] fp32      gradient with respect to the chunk's own scores through the soft gates and thresholds
 * (the retained keys of earlier chunks and their scores are constants).  Equal to the gradients of the unchunked
 * operator for an upstream gradient that vanishes outside the chunk's rows, restricted to the chunk's positions.
 * q, o, dO in [B,H,c,d]: the chunk's queries, the outputs the forward call returned, their upstream gradient; c as
 * in that call.  fwd_ws: that call's workspace, untouched since (it holds the chunk's virtual sequence; read only).
 * ws: scratch of sparsek_chunk_bwd_workspace_bytes(cfg) bytes.  bf16 with d = 64 or 128 only (UNSUPPORTED otherwise;
 * the size query then returns 0). */
size_t sparsek_chunk_bwd_workspace_bytes(const sparsek_chunk_cfg *cfg);
int sparsek_chunk_bwd(const sparsek_chunk_cfg *cfg, int32_t c, const void *q, const void *o, const void *dO,
                      const void *fwd_ws, size_t fwd_ws_bytes, void *dq, void *dk, void *dv, float *du, void *ws,
                      size_t ws_bytes, void *stream);
/* Hands the sequence over to the single-token decode: fills decode_state (of sparsek_decode_state_bytes(dcfg)
 * bytes) with the state after the n_consumed tokens passed so far, so that sparsek_decode_step continues exactly
 * where the chunks ended.  dcfg must agree with cfg in B, H, Gu, d, k, w and dtype.  n_consumed (the caller's count
 * of tokens passed to sparsek_chunk_prefill) must be at least k + w (UNSUPPORTED otherwise).  Uses ws; the chunk
 * state is left unchanged. */
int sparsek_chunk_to_decode(const sparsek_chunk_cfg *cfg, void *state, size_t state_bytes, int64_t n_consumed,
                            void *ws, size_t ws_bytes, const sparsek_decode_cfg *dcfg, void *decode_state,
                            size_t decode_state_bytes, void *stream);
/* Copies the number of retained entries and the flag word of every score row ([B*Gu] int32 each, either may be
 * null) to host memory and synchronises the stream. */
int sparsek_chunk_status(const sparsek_chunk_cfg *cfg, const void *state, int32_t *host_counts,
                         int32_t *host_flags, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARSEK_H */

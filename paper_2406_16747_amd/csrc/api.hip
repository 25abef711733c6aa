// C-ABI entry points of libsparsek: argument validation, then the launch wrappers.
#include "common.hpp"

using namespace spk;

namespace {

int check_common(const sparsek_cfg* c)
{
    if (!c) return SPARSEK_ERR_INVALID_ARG;
    if (c->B < 1 || c->H < 1 || c->n < 1 || c->k < 0 || c->w < 0 || (long long)c->k + c->w < 1)
        return SPARSEK_ERR_INVALID_ARG;
    if (c->Gu != 1 && c->Gu != c->H) return SPARSEK_ERR_INVALID_ARG;
    if ((long long)c->B * c->H > 65535) return SPARSEK_ERR_UNSUPPORTED;
    if ((long long)c->n > (1 << 28)) return SPARSEK_ERR_UNSUPPORTED;
    // k and w beyond n mean the same as n; larger values are refused rather than clamped so that sums such as
    // k + w and w - 1 + death[j] stay far from the int32 range everywhere
    if (c->k > (1 << 28) || c->w > (1 << 28)) return SPARSEK_ERR_UNSUPPORTED;
    return SPARSEK_OK;
}

int check_attn(const sparsek_cfg* c)
{
    int rc = check_common(c);
    if (rc) return rc;
    if (c->gate_mode < 0 || c->gate_mode > 3) return SPARSEK_ERR_INVALID_ARG;
    if (c->dtype != SPARSEK_F32 && c->dtype != SPARSEK_BF16) return SPARSEK_ERR_UNSUPPORTED;
    if (c->d < 4 || c->d > 128 || (c->d % 4) != 0) return SPARSEK_ERR_UNSUPPORTED;
    if (!(c->softmax_scale > 0.0f) || !(c->softmax_scale < INFINITY)) return SPARSEK_ERR_INVALID_ARG;
    return SPARSEK_OK;
}

}  // namespace

extern "C" {

const char* sparsek_strerror(int code)
{
    switch (code) {
        case SPARSEK_OK: return "ok";
        case SPARSEK_ERR_INVALID_ARG: return "invalid argument";
        case SPARSEK_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case SPARSEK_ERR_WORKSPACE: return "workspace or state buffer too small";
        case SPARSEK_ERR_LAUNCH: return "HIP launch failed";
        case SPARSEK_ERR_TOO_LARGE: return "problem larger than the built-in scratch array of sparsek_mask_static";
        default: return "unknown error";
    }
}

size_t sparsek_mask_workspace_bytes(const sparsek_cfg* cfg)
{
    if (check_common(cfg)) return 0;
    return mask_ws_bytes(*cfg);
}

int sparsek_mask(const sparsek_cfg* cfg, const float* u, float* tau, int32_t* death, void* ws,
                 size_t ws_bytes, void* stream)
{
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!u || !tau || !death || !ws) return SPARSEK_ERR_INVALID_ARG;
    if (ws_bytes < mask_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return launch_mask(*cfg, u, tau, death, ws, (hipStream_t)stream);
}

int sparsek_mask_status(const sparsek_cfg* cfg, const void* ws, size_t ws_bytes, int32_t* host_flag, void* stream)
{
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!ws || !host_flag) return SPARSEK_ERR_INVALID_ARG;
    if (ws_bytes < mask_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return mask_status(*cfg, ws, host_flag, (hipStream_t)stream);
}

int sparsek_materialize(const sparsek_cfg* cfg, const float* u, const float* tau, const int32_t* death,
                        int32_t t_begin, int32_t t_end, int32_t* idx, float* gate, void* stream)
{
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!u || !tau || !death || !idx) return SPARSEK_ERR_INVALID_ARG;
    if (t_begin < 0 || t_end < t_begin || t_end > cfg->n) return SPARSEK_ERR_INVALID_ARG;
    if (t_end - t_begin > 65535 * 16) return SPARSEK_ERR_UNSUPPORTED;
    return launch_materialize(*cfg, u, tau, death, t_begin, t_end, idx, gate, (hipStream_t)stream);
}

size_t sparsek_attn_fwd_workspace_bytes(const sparsek_cfg* cfg)
{
    if (check_attn(cfg)) return 0;
    return attn_fwd_ws_bytes(*cfg);
}

int sparsek_attn_fwd(const sparsek_cfg* cfg, const void* q, const void* k, const void* v, const float* u,
                     const float* tau, const int32_t* death, void* o, float* lse, void* ws,
                     size_t ws_bytes, void* stream)
{
    int rc = check_attn(cfg);
    if (rc) return rc;
    if (!q || !k || !v || !u || !tau || !death || !o || !ws) return SPARSEK_ERR_INVALID_ARG;
    if (ws_bytes < attn_fwd_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    sparsek_cfg c = *cfg;
    if (c.gate_mode == 3) c.gate_mode = 2;  // the straight-through forward is the hard-selection forward
    return launch_attn_fwd(c, q, k, v, u, tau, death, o, lse, ws, (hipStream_t)stream);
}

}  // extern "C"


extern "C" {

size_t sparsek_attn_bwd_workspace_bytes(const sparsek_cfg* cfg)
{
    if (check_attn(cfg)) return 0;
    return spk::attn_bwd_ws_bytes(*cfg);
}

int sparsek_attn_bwd(const sparsek_cfg* cfg, const void* q, const void* k, const void* v, const float* u,
                     const float* tau, const int32_t* death, const void* o, const float* lse, const void* dO, void* dq,
                     void* dk, void* dv, void* ws, size_t ws_bytes, void* stream)
{
    int rc = check_attn(cfg);
    if (rc) return rc;
    if (!q || !k || !v || !u || !tau || !death || !o || !lse || !dO || !dq || !dk || !dv || !ws)
        return SPARSEK_ERR_INVALID_ARG;
    if (ws_bytes < spk::attn_bwd_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    sparsek_cfg c = *cfg;
    if (c.gate_mode == 3) c.gate_mode = 2;  // the straight-through forward has no gates on q, k, v
    return spk::launch_attn_bwd(c, q, k, v, u, tau, death, o, lse, dO, dq, dk, dv, ws, (hipStream_t)stream);
}

}  // extern "C"

// ---- importance scores (scores.hip) ----
namespace spk {
size_t scores_ws_bytes(int B, int n);
int launch_scores(int B, int n, int D, int dtype, int norm, double slope, double norm_eps, const void* x,
                  const float* w, float* u, void* ws, hipStream_t st);
}  // namespace spk

namespace {
int check_scores(const sparsek_scores_cfg* c)
{
    if (!c) return SPARSEK_ERR_INVALID_ARG;
    if (c->B < 1 || c->n < 1 || c->D < 1) return SPARSEK_ERR_INVALID_ARG;
    if (c->norm != 0 && c->norm != 1) return SPARSEK_ERR_INVALID_ARG;
    if (!(c->slope > -INFINITY) || !(c->slope < INFINITY)) return SPARSEK_ERR_INVALID_ARG;
    if (c->norm == 1 && (!(c->norm_eps > 0.0f) || !(c->norm_eps < INFINITY))) return SPARSEK_ERR_INVALID_ARG;
    if (c->dtype != SPARSEK_F32 && c->dtype != SPARSEK_BF16) return SPARSEK_ERR_UNSUPPORTED;
    if ((c->D % 8) != 0 || c->D > 8192) return SPARSEK_ERR_UNSUPPORTED;
    if ((long long)c->n > (1 << 28) || c->B > 65535) return SPARSEK_ERR_UNSUPPORTED;
    return SPARSEK_OK;
}
}  // namespace

extern "C" {

size_t sparsek_scores_workspace_bytes(const sparsek_scores_cfg* cfg)
{
    if (check_scores(cfg)) return 0;
    return spk::scores_ws_bytes(cfg->B, cfg->n);
}

int sparsek_scores(const sparsek_scores_cfg* cfg, const void* x, const float* w, float* u, void* ws,
                   size_t ws_bytes, void* stream)
{
    int rc = check_scores(cfg);
    if (rc) return rc;
    if (!x || !w || !u) return SPARSEK_ERR_INVALID_ARG;
    if (cfg->norm == 1 && (!ws || ws_bytes < spk::scores_ws_bytes(cfg->B, cfg->n))) return SPARSEK_ERR_WORKSPACE;
    return spk::launch_scores(cfg->B, cfg->n, cfg->D, cfg->dtype, cfg->norm, (double)cfg->slope,
                              (double)cfg->norm_eps, x, w, u, ws, (hipStream_t)stream);
}

}  // extern "C"

// ---- entry points whose kernels live in mask_bwd.hip and decode.hip ----
namespace spk {
size_t decode_state_bytes(const sparsek_decode_cfg& c);
int launch_decode_init(const sparsek_decode_cfg& c, void* state, hipStream_t st);
int launch_decode_load(const sparsek_decode_cfg& c, void* state, int n_ctx, const void* k, const void* v,
                       const float* u, const float* tau, const int32_t* death, hipStream_t st);
int launch_decode_step(const sparsek_decode_cfg& c, void* state, const void* q, const void* k, const void* v,
                       const float* u_new, void* o, hipStream_t st);
int decode_status(const sparsek_decode_cfg& c, const void* state, int32_t* host_flags, hipStream_t st);
}  // namespace spk

namespace {
int check_decode(const sparsek_decode_cfg* c)
{
    if (!c) return SPARSEK_ERR_INVALID_ARG;
    if (c->B < 1 || c->H < 1 || c->k < 0 || c->w < 0 || (long long)c->k + c->w < 1 || c->cand_cap < 0)
        return SPARSEK_ERR_INVALID_ARG;
    if (c->Gu != 1 && c->Gu != c->H) return SPARSEK_ERR_INVALID_ARG;
    if (c->gate_mode < 0 || c->gate_mode > 3) return SPARSEK_ERR_INVALID_ARG;
    if (c->dtype != SPARSEK_F32 && c->dtype != SPARSEK_BF16) return SPARSEK_ERR_UNSUPPORTED;
    // the state holds k + w slots per head and cand_cap (default 4k) scores per row: sizes are computed in int
    if (c->k > (1 << 24) || c->w > (1 << 24) || c->cand_cap > (1 << 26)) return SPARSEK_ERR_UNSUPPORTED;
    if (c->d < 8 || c->d > 128 || (c->d % 8) != 0) return SPARSEK_ERR_UNSUPPORTED;
    if ((long long)c->B * c->H > (1 << 24)) return SPARSEK_ERR_UNSUPPORTED;
    if (!(c->softmax_scale > 0.0f) || !(c->softmax_scale < INFINITY)) return SPARSEK_ERR_INVALID_ARG;
    return SPARSEK_OK;
}
}  // namespace

extern "C" {

size_t sparsek_mask_bwd_workspace_bytes(const sparsek_cfg* cfg)
{
    if (check_attn(cfg)) return 0;
    return mask_bwd_ws_bytes(*cfg);
}

int sparsek_mask_bwd(const sparsek_cfg* cfg, const void* q, const void* k, const void* v, const float* u,
                     const float* tau, const int32_t* death, const void* o, const float* lse, const void* dO,
                     float* du, void* ws, size_t ws_bytes, void* stream)
{
    int rc = check_attn(cfg);
    if (rc) return rc;
    if (!q || !k || !v || !u || !tau || !death || !o || !lse || !dO || !du || !ws)
        return SPARSEK_ERR_INVALID_ARG;
    if (ws_bytes < mask_bwd_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return launch_mask_bwd(*cfg, q, k, v, u, tau, death, o, lse, dO, du, ws, (hipStream_t)stream);
}

size_t sparsek_bwd_workspace_bytes(const sparsek_cfg* cfg)
{
    if (check_attn(cfg)) return 0;
    return align_up(spk::attn_bwd_ws_bytes(*cfg), 256) + mask_bwd_ws_bytes(*cfg);
}

int sparsek_bwd(const sparsek_cfg* cfg, const void* q, const void* k, const void* v, const float* u, const float* tau,
                const int32_t* death, const void* o, const float* lse, const void* dO, void* dq, void* dk, void* dv,
                float* du, void* ws, size_t ws_bytes, void* stream)
{
    int rc = check_attn(cfg);
    if (rc) return rc;
    if (!q || !k || !v || !u || !tau || !death || !o || !lse || !dO || !dq || !dk || !dv || !du || !ws)
        return SPARSEK_ERR_INVALID_ARG;
    if (ws_bytes < sparsek_bwd_workspace_bytes(cfg)) return SPARSEK_ERR_WORKSPACE;
    sparsek_cfg c = *cfg;
    if (c.gate_mode == 3) c.gate_mode = 2;  // the straight-through forward has no gates on q, k, v
    rc = spk::launch_attn_bwd(c, q, k, v, u, tau, death, o, lse, dO, dq, dk, dv, ws, (hipStream_t)stream);
    if (rc) return rc;
    return launch_mask_bwd(*cfg, q, k, v, u, tau, death, o, lse, dO, du,
                           (char*)ws + align_up(spk::attn_bwd_ws_bytes(*cfg), 256), (hipStream_t)stream);
}

size_t sparsek_decode_state_bytes(const sparsek_decode_cfg* cfg)
{
    if (check_decode(cfg)) return 0;
    return decode_state_bytes(*cfg);
}

int sparsek_decode_init(const sparsek_decode_cfg* cfg, void* state, size_t state_bytes, void* stream)
{
    int rc = check_decode(cfg);
    if (rc) return rc;
    if (!state) return SPARSEK_ERR_INVALID_ARG;
    if (state_bytes < decode_state_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return launch_decode_init(*cfg, state, (hipStream_t)stream);
}

int sparsek_decode_load(const sparsek_decode_cfg* cfg, void* state, size_t state_bytes, int32_t n_ctx,
                        const void* k, const void* v, const float* u, const float* tau, const int32_t* death,
                        void* stream)
{
    int rc = check_decode(cfg);
    if (rc) return rc;
    if (!state || n_ctx < 0) return SPARSEK_ERR_INVALID_ARG;
    if (n_ctx > 0 && (!k || !v || !u || !tau || !death)) return SPARSEK_ERR_INVALID_ARG;
    if (state_bytes < decode_state_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    if (n_ctx == 0) return launch_decode_init(*cfg, state, (hipStream_t)stream);
    return launch_decode_load(*cfg, state, n_ctx, k, v, u, tau, death, (hipStream_t)stream);
}

int sparsek_decode_step(const sparsek_decode_cfg* cfg, void* state, const void* q_new, const void* k_new,
                        const void* v_new, const float* u_new, void* o, void* stream)
{
    int rc = check_decode(cfg);
    if (rc) return rc;
    if (!state || !q_new || !k_new || !v_new || !u_new || !o) return SPARSEK_ERR_INVALID_ARG;
    sparsek_decode_cfg c = *cfg;
    if (c.gate_mode == 3) c.gate_mode = 2;  // straight-through: the forward skips the gates
    return launch_decode_step(c, state, q_new, k_new, v_new, u_new, o, (hipStream_t)stream);
}

int sparsek_decode_status(const sparsek_decode_cfg* cfg, const void* state, int32_t* host_flags, void* stream)
{
    int rc = check_decode(cfg);
    if (rc) return rc;
    if (!state || !host_flags) return SPARSEK_ERR_INVALID_ARG;
    return decode_status(*cfg, state, host_flags, (hipStream_t)stream);
}

}  // extern "C"

// ---- chunk-wise recurrent prefill (chunk.hip) ----
namespace spk {
size_t chunk_state_bytes(const sparsek_chunk_cfg& c);
size_t chunk_ws_bytes(const sparsek_chunk_cfg& c);
int launch_chunk_init(const sparsek_chunk_cfg& c, void* state, hipStream_t st);
int launch_chunk_prefill(const sparsek_chunk_cfg& c, void* state, int clen, const void* q, const void* k,
                         const void* v, const float* u, void* o, void* ws, hipStream_t st);
int chunk_status(const sparsek_chunk_cfg& c, const void* state, int32_t* host_counts, int32_t* host_flags,
                 hipStream_t st);
int launch_chunk_to_decode(const sparsek_chunk_cfg& c, void* state, void* ws, const sparsek_decode_cfg& dc,
                           void* dstate, hipStream_t st);
size_t chunk_bwd_ws_bytes(const sparsek_chunk_cfg& c);
int launch_chunk_bwd(const sparsek_chunk_cfg& c, int clen, const void* q, const void* o, const void* dO,
                     const void* fwd_ws, void* dq, void* dk, void* dv, float* du, void* ws, hipStream_t st);
}  // namespace spk

namespace {
int check_chunk(const sparsek_chunk_cfg* c)
{
    if (!c) return SPARSEK_ERR_INVALID_ARG;
    if (c->B < 1 || c->H < 1 || c->k < 0 || c->w < 0 || (long long)c->k + c->w < 1 || c->cand_cap < 0 || c->chunk_max < 1)
        return SPARSEK_ERR_INVALID_ARG;
    if (c->Gu != 1 && c->Gu != c->H) return SPARSEK_ERR_INVALID_ARG;
    if (c->gate_mode < 0 || c->gate_mode > 3) return SPARSEK_ERR_INVALID_ARG;
    if (!(c->softmax_scale > 0.0f) || !(c->softmax_scale < INFINITY)) return SPARSEK_ERR_INVALID_ARG;
    if (c->dtype != SPARSEK_F32 && c->dtype != SPARSEK_BF16) return SPARSEK_ERR_UNSUPPORTED;
    if (c->d < 4 || c->d > 128 || (c->d % 4) != 0) return SPARSEK_ERR_UNSUPPORTED;
    if ((c->d * (c->dtype == SPARSEK_BF16 ? 2 : 4)) % 16 != 0) return SPARSEK_ERR_UNSUPPORTED;
    if ((long long)c->B * c->H > 65535) return SPARSEK_ERR_UNSUPPORTED;
    if ((long long)c->k + c->w + c->cand_cap + c->chunk_max > (1 << 26)) return SPARSEK_ERR_UNSUPPORTED;
    return SPARSEK_OK;
}
}  // namespace

extern "C" {

size_t sparsek_chunk_state_bytes(const sparsek_chunk_cfg* cfg)
{
    if (check_chunk(cfg)) return 0;
    return spk::chunk_state_bytes(*cfg);
}

size_t sparsek_chunk_workspace_bytes(const sparsek_chunk_cfg* cfg)
{
    if (check_chunk(cfg)) return 0;
    return spk::chunk_ws_bytes(*cfg);
}

int sparsek_chunk_init(const sparsek_chunk_cfg* cfg, void* state, size_t state_bytes, void* stream)
{
    int rc = check_chunk(cfg);
    if (rc) return rc;
    if (!state) return SPARSEK_ERR_INVALID_ARG;
    if (state_bytes < spk::chunk_state_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return spk::launch_chunk_init(*cfg, state, (hipStream_t)stream);
}

int sparsek_chunk_prefill(const sparsek_chunk_cfg* cfg, void* state, size_t state_bytes, int32_t c, const void* q,
                          const void* k, const void* v, const float* u, void* o, void* ws, size_t ws_bytes,
                          void* stream)
{
    int rc = check_chunk(cfg);
    if (rc) return rc;
    if (!state || !q || !k || !v || !u || !o || !ws) return SPARSEK_ERR_INVALID_ARG;
    if (c < 1 || c > cfg->chunk_max) return SPARSEK_ERR_INVALID_ARG;
    if (state_bytes < spk::chunk_state_bytes(*cfg) || ws_bytes < spk::chunk_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return spk::launch_chunk_prefill(*cfg, state, c, q, k, v, u, o, ws, (hipStream_t)stream);
}

size_t sparsek_chunk_bwd_workspace_bytes(const sparsek_chunk_cfg* cfg)
{
    if (check_chunk(cfg)) return 0;
    if (cfg->dtype != SPARSEK_BF16 || (cfg->d != 64 && cfg->d != 128)) return 0;
    return spk::chunk_bwd_ws_bytes(*cfg);
}

int sparsek_chunk_bwd(const sparsek_chunk_cfg* cfg, int32_t c, const void* q, const void* o, const void* dO,
                      const void* fwd_ws, size_t fwd_ws_bytes, void* dq, void* dk, void* dv, float* du, void* ws,
                      size_t ws_bytes, void* stream)
{
    int rc = check_chunk(cfg);
    if (rc) return rc;
    if (!q || !o || !dO || !fwd_ws || !dq || !dk || !dv || !du || !ws) return SPARSEK_ERR_INVALID_ARG;
    if (c < 1 || c > cfg->chunk_max) return SPARSEK_ERR_INVALID_ARG;
    if (cfg->dtype != SPARSEK_BF16 || (cfg->d != 64 && cfg->d != 128)) return SPARSEK_ERR_UNSUPPORTED;
    if (fwd_ws_bytes < spk::chunk_ws_bytes(*cfg) || ws_bytes < spk::chunk_bwd_ws_bytes(*cfg)) return SPARSEK_ERR_WORKSPACE;
    return spk::launch_chunk_bwd(*cfg, c, q, o, dO, fwd_ws, dq, dk, dv, du, ws, (hipStream_t)stream);
}

int sparsek_chunk_to_decode(const sparsek_chunk_cfg* cfg, void* state, size_t state_bytes, int64_t n_consumed,
                            void* ws, size_t ws_bytes, const sparsek_decode_cfg* dcfg, void* decode_state,
                            size_t decode_state_bytes, void* stream)
{
    int rc = check_chunk(cfg);
    if (rc) return rc;
    rc = check_decode(dcfg);
    if (rc) return rc;
    if (!state || !ws || !decode_state) return SPARSEK_ERR_INVALID_ARG;
    if (dcfg->B != cfg->B || dcfg->H != cfg->H || dcfg->Gu != cfg->Gu || dcfg->d != cfg->d || dcfg->k != cfg->k ||
        dcfg->w != cfg->w || dcfg->dtype != cfg->dtype)
        return SPARSEK_ERR_INVALID_ARG;
    if (n_consumed < (int64_t)cfg->k + cfg->w) return SPARSEK_ERR_UNSUPPORTED;
    if (state_bytes < spk::chunk_state_bytes(*cfg) || ws_bytes < spk::chunk_ws_bytes(*cfg) ||
        decode_state_bytes < spk::decode_state_bytes(*dcfg))
        return SPARSEK_ERR_WORKSPACE;
    return spk::launch_chunk_to_decode(*cfg, state, ws, *dcfg, decode_state, (hipStream_t)stream);
}

int sparsek_chunk_status(const sparsek_chunk_cfg* cfg, const void* state, int32_t* host_counts, int32_t* host_flags,
                         void* stream)
{
    int rc = check_chunk(cfg);
    if (rc) return rc;
    if (!state) return SPARSEK_ERR_INVALID_ARG;
    return spk::chunk_status(*cfg, state, host_counts, host_flags, (hipStream_t)stream);
}

}  // extern "C"


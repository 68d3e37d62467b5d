// C-ABI entry points of libphoton: argument validation, context life cycle and dispatch.
// The operations are those of the paper's execution pipeline (Alg. 1) and of the cross-silo
// FL algorithm (Alg. 3): TrainClient, pseudo-gradient, weighted mean, ServerOpt.

#include <cmath>
#include <new>

#include "common.h"

namespace {

bool cfg_valid(const photon_model_cfg *c) {
    if (!c) return false;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ff < 1 || c->vocab < 2 || c->seq_len < 1)
        return false;
    if (c->d_model % c->n_heads != 0) return false;
    if (c->d_model % 8 != 0 || c->d_ff % 8 != 0) return false;  // 128-bit row accesses
    if (!(c->ln_eps > 0.f)) return false;
    if (c->compute_dtype != PHOTON_FP32 && c->compute_dtype != PHOTON_BF16) return false;
    if (c->recompute < 0 || c->recompute > 2) return false;
    if (c->micro_fuse < 0 || c->micro_fuse > 64) return false;
    return true;
}

// [a, a + an) and [b, b + bn) share a byte
bool overlaps(const void *a, int64_t an, const void *b, int64_t bn) {
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return a && b && pa < pb + (uintptr_t)bn && pb < pa + (uintptr_t)an;
}

bool hp_valid(const photon_adamw_hp *hp) {
    return hp && hp->beta1 >= 0.f && hp->beta1 < 1.f && hp->beta2 >= 0.f && hp->beta2 < 1.f && hp->eps > 0.f &&
           hp->weight_decay >= 0.f;
}

}  // namespace

extern "C" {

int64_t photon_param_count(const photon_model_cfg *c) {
    if (!cfg_valid(c)) return PHOTON_EINVAL;
    const int64_t d = c->d_model, f = c->d_ff;
    return (int64_t)c->vocab * d + (int64_t)c->n_layers * (2 * d + 4 * d * d + 2 * d * f) + d;
}

static int create_common(int64_t n, void *stream, photon_ctx **out) {
    photon_ctx *ctx = new (std::nothrow) photon_ctx();
    if (!ctx) return PHOTON_ENOMEM;
    ctx->stream = (hipStream_t)stream;
    ctx->n = n;
    const int rc = flat_init(ctx);
    if (rc != PHOTON_OK) {
        flat_free(ctx);
        delete ctx;
        return rc;
    }
    *out = ctx;
    return PHOTON_OK;
}

int photon_create_flat(int64_t n, void *hip_stream, photon_ctx **out) {
    if (!out || n < 1) return PHOTON_EINVAL;
    *out = nullptr;
    return create_common(n, hip_stream, out);
}

int photon_create(const photon_model_cfg *cfg, int32_t micro_batch, void *hip_stream, photon_ctx **out) {
    if (!out) return PHOTON_EINVAL;
    *out = nullptr;
    if (!cfg_valid(cfg) || micro_batch < 1) return PHOTON_EINVAL;
    if (cfg->recompute == 2) return PHOTON_ENOTIMPL;  // reserved: a policy coarser than per block
    photon_ctx *ctx = nullptr;
    int rc = create_common(photon_param_count(cfg), hip_stream, &ctx);
    if (rc != PHOTON_OK) return rc;
    ctx->has_model = true;
    ctx->cfg = *cfg;
    ctx->micro_batch = micro_batch;
    rc = model_create(ctx);
    if (rc != PHOTON_OK) {
        photon_destroy(ctx);
        return rc;
    }
    *out = ctx;
    return PHOTON_OK;
}

void photon_destroy(photon_ctx *ctx) {
    if (!ctx) return;
    if (ctx->has_model) model_destroy(ctx);
    flat_free(ctx);
    for (hipEvent_t e : ctx->timer.pool) (void)hipEventDestroy(e);
    ctx->timer.pool.clear();
    delete ctx;
}

const char *photon_strerror(int status) {
    switch (status) {
        case PHOTON_OK: return "ok";
        case PHOTON_EINVAL: return "invalid argument";
        case PHOTON_ENOMEM: return "out of memory";
        case PHOTON_EHIP: return "HIP runtime error";
        case PHOTON_ENONFINITE: return "non-finite loss";
        case PHOTON_ENOTIMPL: return "not implemented";
        case PHOTON_ELIMIT: return "size beyond the limit of the allocation-free entry point";
        default: return "unknown status";
    }
}

int photon_last_hip_error(const photon_ctx *ctx) { return ctx ? ctx->last_hip_error : 0; }

int64_t photon_workspace_bytes(const photon_ctx *ctx) { return ctx ? ctx->workspace_bytes : 0; }

int photon_client_local_steps(photon_ctx *ctx, float *params, photon_opt_state *st, const int32_t *tokens,
                              int32_t n_steps, int32_t n_micro, const float *lrs, const photon_adamw_hp *hp,
                              float *loss_out) {
    if (!ctx || !ctx->has_model || !params || !st || !st->m || !st->v || !tokens || !lrs || !loss_out) return PHOTON_EINVAL;
    if (n_steps < 0 || n_micro < 1 || st->step < 0 || !hp_valid(hp)) return PHOTON_EINVAL;
    if (!aligned16(params) || !aligned16(st->m) || !aligned16(st->v) || !aligned16(tokens)) return PHOTON_EINVAL;
    for (int s = 0; s < n_steps; ++s)
        if (!std::isfinite(lrs[s]) || lrs[s] < 0.f) return PHOTON_EINVAL;
    if (n_steps == 0) return PHOTON_OK;
    TimerScope ts(ctx);
    return model_local_steps(ctx, params, st, tokens, n_steps, n_micro, lrs, hp, loss_out);
}

int photon_client_loss_grad(photon_ctx *ctx, const float *params, const int32_t *tokens, float *grads_out,
                            float *loss_out) {
    if (!ctx || !ctx->has_model || !params || !tokens || !grads_out || !loss_out) return PHOTON_EINVAL;
    if (!aligned16(params) || !aligned16(grads_out) || !aligned16(tokens)) return PHOTON_EINVAL;
    TimerScope ts(ctx);
    return model_loss_grad(ctx, params, tokens, grads_out, loss_out);
}

int photon_adamw_step(photon_ctx *ctx, float *params, photon_opt_state *st, const float *grads, float lr,
                      const photon_adamw_hp *hp, void *bf16_out) {
    if (!ctx || !params || !st || !st->m || !st->v || !grads || !hp_valid(hp)) return PHOTON_EINVAL;
    if (st->step < 0 || !std::isfinite(lr) || lr < 0.f) return PHOTON_EINVAL;
    if (!aligned16(params) || !aligned16(st->m) || !aligned16(st->v) || !aligned16(grads) || !aligned16(bf16_out))
        return PHOTON_EINVAL;
    TimerScope ts(ctx);
    const int rc = flat_adamw(ctx, params, st->m, st->v, grads, ctx->n, st->step + 1, lr, hp, (bf16 *)bf16_out);
    if (rc == PHOTON_OK) st->step += 1;
    return rc;
}

int photon_export_delta(photon_ctx *ctx, const float *global_params, const float *client_params, void *delta_out,
                        int32_t dtype) {
    if (!ctx || !global_params || !client_params || !delta_out) return PHOTON_EINVAL;
    if (dtype != PHOTON_FP32 && dtype != PHOTON_BF16) return PHOTON_EINVAL;
    if (!aligned16(global_params) || !aligned16(client_params) || !aligned16(delta_out)) return PHOTON_EINVAL;
    TimerScope ts(ctx);
    return flat_export_delta(ctx, global_params, client_params, delta_out, dtype, ctx->n);
}

// Argument checks shared by the two aggregation entry points; fills the normalised weights.
static int aggregate_args_ok(int64_t n, const float *global_params, const void *const *client_bufs, int32_t K,
                             int32_t max_clients, int32_t kind, int32_t dtype, const double *client_weights,
                             const photon_outer_opt *oo, float *wnorm) {
    if (!global_params || !client_bufs || !client_weights || !oo || n < 1) return PHOTON_EINVAL;
    if (K < 1 || K > max_clients) return PHOTON_EINVAL;
    if (kind != PHOTON_CLIENT_PARAMS && kind != PHOTON_CLIENT_DELTAS) return PHOTON_EINVAL;
    if (dtype != PHOTON_FP32 && dtype != PHOTON_BF16) return PHOTON_EINVAL;
    if (kind == PHOTON_CLIENT_PARAMS && dtype != PHOTON_FP32) return PHOTON_EINVAL;
    if (!std::isfinite(oo->eta_s) || !std::isfinite(oo->mu)) return PHOTON_EINVAL;
    if (oo->mu != 0.f && !oo->momentum) return PHOTON_EINVAL;
    if (!aligned16(global_params) || !aligned16(oo->momentum)) return PHOTON_EINVAL;
    // the kernel reads the client buffers while it rewrites the model and the momentum in place:
    // none of them may share memory with either, nor those two with each other
    const int64_t nb = n * 4, cb = n * (dtype == PHOTON_BF16 ? 2 : 4);
    if (overlaps(global_params, nb, oo->momentum, nb)) return PHOTON_EINVAL;
    double sum = 0.0;
    for (int k = 0; k < K; ++k) {
        if (!client_bufs[k] || !aligned16(client_bufs[k])) return PHOTON_EINVAL;
        if (overlaps(client_bufs[k], cb, global_params, nb) || overlaps(client_bufs[k], cb, oo->momentum, nb))
            return PHOTON_EINVAL;
        if (!std::isfinite(client_weights[k]) || client_weights[k] < 0.0) return PHOTON_EINVAL;
        sum += client_weights[k];
    }
    if (!(sum > 0.0) || !std::isfinite(sum)) return PHOTON_EINVAL;
    for (int k = 0; k < K; ++k) wnorm[k] = (float)(client_weights[k] / sum);  // normalised in float64
    return PHOTON_OK;
}

int photon_aggregate(photon_ctx *ctx, float *global_params, const void *const *client_bufs, int32_t K, int32_t kind,
                     int32_t dtype, const double *client_weights, photon_outer_opt *oo, photon_agg_metrics *metrics) {
    if (!ctx) return PHOTON_EINVAL;
    float wnorm[PHOTON_MAX_CLIENTS];
    const int rc = aggregate_args_ok(ctx->n, global_params, client_bufs, K, PHOTON_MAX_CLIENTS, kind, dtype,
                                     client_weights, oo, wnorm);
    if (rc != PHOTON_OK) return rc;
    TimerScope ts(ctx);
    return flat_aggregate(ctx, global_params, client_bufs, K, kind, dtype, wnorm, oo, metrics, ctx->n);
}

int photon_aggregate_static(void *hip_stream, int64_t n, float *global_params, const void *const *client_bufs,
                            int32_t K, int32_t kind, int32_t dtype, const double *client_weights,
                            photon_outer_opt *oo, double *norms_out, int32_t *hip_error_out) {
    if (hip_error_out) *hip_error_out = 0;
    if (K > PHOTON_STATIC_MAX_CLIENTS && K <= PHOTON_MAX_CLIENTS) return PHOTON_ELIMIT;
    if (norms_out && (reinterpret_cast<uintptr_t>(norms_out) & 7u)) return PHOTON_EINVAL;
    float wnorm[PHOTON_MAX_CLIENTS];
    const int rc = aggregate_args_ok(n, global_params, client_bufs, K, PHOTON_STATIC_MAX_CLIENTS, kind, dtype,
                                     client_weights, oo, wnorm);
    if (rc != PHOTON_OK) return rc;
    int hip_error = 0;
    const int rc2 = flat_aggregate_static((hipStream_t)hip_stream, global_params, client_bufs, K, kind, dtype, wnorm,
                                          oo, norms_out, n, &hip_error);
    if (hip_error_out) *hip_error_out = hip_error;
    return rc2;
}

int photon_client_init(photon_ctx *ctx, const float *global_params, float *client_params, photon_opt_state *st) {
    if (!ctx || !global_params || !client_params || !st || !st->m || !st->v) return PHOTON_EINVAL;
    if (!aligned16(global_params) || !aligned16(client_params) || !aligned16(st->m) || !aligned16(st->v))
        return PHOTON_EINVAL;
    if (global_params == client_params) return PHOTON_EINVAL;
    const int rc = flat_client_init(ctx, global_params, client_params, st->m, st->v, ctx->n);
    if (rc == PHOTON_OK) st->step = 0;
    return rc;
}

int photon_clip_delta(photon_ctx *ctx, void *delta, int32_t dtype, double max_norm, double *norm_out) {
    if (!ctx || !delta || !aligned16(delta) || !(max_norm > 0.0)) return PHOTON_EINVAL;
    if (dtype != PHOTON_FP32 && dtype != PHOTON_BF16) return PHOTON_EINVAL;
    return flat_clip(ctx, delta, dtype, max_norm, norm_out, ctx->n);
}

}  // extern "C"

// C ABI of the multi-layer float workloads (MLP stack, decoder) and of their unperturbed glue: argument
// validation only; the sequencing lives in k_models.hip, the kernels in k_decoder.hip and k_forward.hip.
#include "common.hpp"

using namespace egg;

static egg_status common_checks(eggroll_ctx* c, egg_key key, const egg_shape* shape, uint32_t noise_layers, bool need_rows)
{
    egg_status s = validate_shape(c, shape, need_rows, false);
    if (s != EGG_OK) return s;
    if ((uint64_t)key.layer + noise_layers > 0x80000000ull) return fail(c, EGG_EINVAL, "noise layers must stay below 2^31");
    return EGG_OK;
}

static bool ok_ptr(const void* p) { return p && aligned16(p); }

extern "C" {

egg_status eggroll_embed_rows_bf16(eggroll_ctx* c, int64_t rows, int d, int vocab, const void* emb, const int32_t* tokens, void* X)
{
    if (!c) return EGG_EINVAL;
    if (rows < 0 || rows > 0x7FFFFFFFLL || d <= 0 || vocab <= 0) return fail(c, EGG_EINVAL, "rows, d or vocab out of range");
    if (d % 8) return fail(c, EGG_EUNSUPPORTED, "d must be a multiple of 8");
    if (!ok_ptr(emb) || !ok_ptr(X) || !tokens) return fail(c, EGG_EINVAL, "pointers must be non-NULL and 16-byte aligned");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_embed_rows(c, rows, d, vocab, emb, tokens, X);
}

egg_status eggroll_rmsnorm_bf16(eggroll_ctx* c, int64_t rows, int d, float eps, const void* gain, const void* X, void* Y)
{
    if (!c) return EGG_EINVAL;
    if (rows < 0 || rows > 0x7FFFFFFFLL || d <= 0) return fail(c, EGG_EINVAL, "rows or d out of range");
    if (d % 8) return fail(c, EGG_EUNSUPPORTED, "d must be a multiple of 8");
    if (!(eps >= 0.0f)) return fail(c, EGG_EINVAL, "eps must be >= 0");
    if (!ok_ptr(gain) || !ok_ptr(X) || !ok_ptr(Y)) return fail(c, EGG_EINVAL, "pointers must be non-NULL and 16-byte aligned");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_rmsnorm(c, rows, d, eps, gain, X, Y);
}

egg_status eggroll_causal_attention_bf16(eggroll_ctx* c, int64_t members, int rows_per_member, int heads, int head_dim,
                                         const void* Q, const void* K, const void* V, void* O)
{
    if (!c) return EGG_EINVAL;
    if (members < 0 || rows_per_member <= 0 || heads <= 0) return fail(c, EGG_EINVAL, "members, rows_per_member or heads out of range");
    if (!ok_ptr(Q) || !ok_ptr(K) || !ok_ptr(V) || !ok_ptr(O)) return fail(c, EGG_EINVAL, "pointers must be non-NULL and 16-byte aligned");
    if (O == Q || O == K || O == V) return fail(c, EGG_EINVAL, "O must not overlap Q, K or V");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_attention(c, members, rows_per_member, heads, head_dim, Q, K, V, O);
}

egg_status eggroll_causal_attention_project_bf16(eggroll_ctx* c, egg_key key, int64_t member_begin, int64_t members, int rows_per_member,
                                                 int heads, int head_dim, const void* Q, const void* K, const void* V, void* O,
                                                 float* t_next)
{
    if (!c) return EGG_EINVAL;
    if (members < 0 || rows_per_member <= 0 || heads <= 0 || head_dim <= 0) return fail(c, EGG_EINVAL, "members, rows_per_member, heads or head_dim out of range");
    if (member_begin < 0 || member_begin + members > (int64_t(1) << 32)) return fail(c, EGG_EINVAL, "member ids must stay below 2^32");
    if (key.layer >> 31) return fail(c, EGG_EINVAL, "layer must be < 2^31");
    if (!ok_ptr(Q) || !ok_ptr(K) || !ok_ptr(V) || !ok_ptr(O) || !t_next) return fail(c, EGG_EINVAL, "pointers must be non-NULL (tensors 16-byte aligned)");
    if (O == Q || O == K || O == V) return fail(c, EGG_EINVAL, "O must not overlap Q, K or V");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    if (members == 0) return EGG_OK;
    // the consuming layer's rank-1 factors B over the model width, exactly what eggroll_noise_gen writes for that layer
    const int64_t d = (int64_t)heads * head_dim;
    egg_status s = reserve(c, c->next_b, (size_t)members * d * 2);
    if (s != EGG_OK) return s;
    s = launch_noise(c, make_stream_key(key.seed, key.step, key.layer, 1), (uint32_t)member_begin, members, d, EGG_BF16, EGG_NORMAL, 0, c->next_b.p);
    if (s != EGG_OK) return s;
    return launch_attention(c, members, rows_per_member, heads, head_dim, Q, K, V, O, c->next_b.p, t_next);
}

egg_status eggroll_token_loglik_bf16(eggroll_ctx* c, int64_t members, int rows_per_member, int vocab, const void* logits,
                                     const int32_t* tokens, float* out)
{
    if (!c) return EGG_EINVAL;
    if (members < 0 || rows_per_member <= 0 || vocab <= 0) return fail(c, EGG_EINVAL, "members, rows_per_member or vocab out of range");
    if (vocab % 8) return fail(c, EGG_EUNSUPPORTED, "vocab must be a multiple of 8");
    if (!ok_ptr(logits) || !tokens || !out) return fail(c, EGG_EINVAL, "pointers must be non-NULL (logits 16-byte aligned)");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_token_loglik(c, members, rows_per_member, vocab, logits, tokens, out);
}

static egg_status mlp_checks(eggroll_ctx* c, egg_key key, const egg_shape* shape, int layers, int d_ff, bool fwd)
{
    if (layers < 1 || layers > 4096) return fail(c, EGG_EINVAL, "layers outside [1, 4096]");
    egg_status s = common_checks(c, key, shape, 2u * (uint32_t)layers, fwd);
    if (s != EGG_OK) return s;
    if (shape->d_out != shape->d_in) return fail(c, EGG_EINVAL, "d_out and d_in must both be the width d");
    if (d_ff <= 0 || d_ff % 8 || shape->d_in % 8) return fail(c, EGG_EUNSUPPORTED, "d and d_ff must be positive multiples of 8");
    return EGG_OK;
}

egg_status eggroll_mlp_stack_forward(eggroll_ctx* c, egg_key key, const egg_shape* shape, int layers, int d_ff, float sigma,
                                     const void* W1, const void* W2, const void* X, void* Y, int64_t chunk_members)
{
    if (!c) return EGG_EINVAL;
    egg_status s = mlp_checks(c, key, shape, layers, d_ff, true);
    if (s != EGG_OK) return s;
    if (!(sigma >= 0.0f)) return fail(c, EGG_EINVAL, "sigma must be >= 0");
    if (!ok_ptr(W1) || !ok_ptr(W2) || !ok_ptr(X) || !ok_ptr(Y) || X == Y) return fail(c, EGG_EINVAL, "pointers must be non-NULL, 16-byte aligned, X != Y");
    if (chunk_members < 0) return fail(c, EGG_EINVAL, "chunk_members must be >= 0");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_mlp_stack_forward(c, key, *shape, layers, d_ff, sigma, W1, W2, X, Y, chunk_members);
}

egg_status eggroll_mlp_stack_update(eggroll_ctx* c, egg_key key, const egg_shape* shape, int layers, int d_ff,
                                    const float* fitness, float scale, float lr, void* W1, void* W2)
{
    if (!c) return EGG_EINVAL;
    egg_status s = mlp_checks(c, key, shape, layers, d_ff, false);
    if (s != EGG_OK) return s;
    if (!fitness || !ok_ptr(W1) || !ok_ptr(W2)) return fail(c, EGG_EINVAL, "pointers must be non-NULL (weights 16-byte aligned)");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_mlp_stack_update(c, key, *shape, layers, d_ff, fitness, scale, lr, W1, W2);
}

static egg_status decoder_checks(eggroll_ctx* c, egg_key key, const egg_shape* shape, const egg_decoder_cfg* cfg,
                                 const egg_decoder_weights* w, bool fwd)
{
    if (!cfg || !w) return fail(c, EGG_EINVAL, "cfg and weights must be non-NULL");
    if (cfg->layers < 0 || cfg->layers > 4096) return fail(c, EGG_EINVAL, "layers outside [0, 4096]");
    egg_status s = common_checks(c, key, shape, 6u * (uint32_t)cfg->layers + 1u, fwd);
    if (s != EGG_OK) return s;
    if (cfg->d_model <= 0 || cfg->heads <= 0 || cfg->d_ff <= 0 || cfg->vocab <= 0) return fail(c, EGG_EINVAL, "non-positive model size");
    if (cfg->d_model % cfg->heads) return fail(c, EGG_EINVAL, "d_model must be heads * head_dim");
    const int hd = cfg->d_model / cfg->heads;
    if (hd != 32 && hd != 64 && hd != 128) return fail(c, EGG_EUNSUPPORTED, "head dimension %d not in {32, 64, 128}", hd);
    if (cfg->d_ff % 8 || cfg->vocab % 8) return fail(c, EGG_EUNSUPPORTED, "d_ff and vocab must be multiples of 8");
    if (!(cfg->rms_eps >= 0.0f)) return fail(c, EGG_EINVAL, "rms_eps must be >= 0");
    if (fwd && shape->rows_per_member > 256) return fail(c, EGG_EUNSUPPORTED, "rows_per_member above 256");
    const void* always[] = {w->emb, w->norm_f, w->head};
    for (const void* p : always)
        if (!ok_ptr(p)) return fail(c, EGG_EINVAL, "weight pointers must be non-NULL and 16-byte aligned");
    if (cfg->layers > 0) {
        const void* per_layer[] = {w->norm1, w->wq, w->wk, w->wv, w->wo, w->norm2, w->w_up, w->w_down};
        for (const void* p : per_layer)
            if (!ok_ptr(p)) return fail(c, EGG_EINVAL, "weight pointers must be non-NULL and 16-byte aligned");
    }
    return EGG_OK;
}

egg_status eggroll_decoder_forward(eggroll_ctx* c, egg_key key, const egg_shape* shape, const egg_decoder_cfg* cfg,
                                   const egg_decoder_weights* weights, float sigma, const int32_t* tokens, void* logits,
                                   float* loglik, int64_t chunk_members)
{
    if (!c) return EGG_EINVAL;
    egg_status s = decoder_checks(c, key, shape, cfg, weights, true);
    if (s != EGG_OK) return s;
    if (!(sigma >= 0.0f)) return fail(c, EGG_EINVAL, "sigma must be >= 0");
    if (!tokens) return fail(c, EGG_EINVAL, "tokens must be non-NULL");
    if (!logits && !loglik) return fail(c, EGG_EINVAL, "pass logits, loglik or both");
    if (logits && !aligned16(logits)) return fail(c, EGG_EINVAL, "logits must be 16-byte aligned");
    if (chunk_members < 0) return fail(c, EGG_EINVAL, "chunk_members must be >= 0");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_decoder_forward(c, key, *shape, *cfg, *weights, sigma, tokens, logits, loglik, chunk_members);
}

egg_status eggroll_decoder_update(eggroll_ctx* c, egg_key key, const egg_shape* shape, const egg_decoder_cfg* cfg,
                                  const float* fitness, float scale, float lr, const egg_decoder_weights* weights)
{
    if (!c) return EGG_EINVAL;
    egg_status s = decoder_checks(c, key, shape, cfg, weights, false);
    if (s != EGG_OK) return s;
    if (!fitness) return fail(c, EGG_EINVAL, "fitness must be non-NULL");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_decoder_update(c, key, *shape, *cfg, fitness, scale, lr, *weights);
}

}  // extern "C"

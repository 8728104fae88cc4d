// Whole-model drivers over the perturbed linear layer (Sec. 4.2) for the two multi-layer float workloads:
// a GELU MLP stack and a pre-norm decoder.  A population is walked in chunks of members (a member's rows
// depend on no other member, so chunking is exact and the noise, addressed by global member id, is the
// same for any chunk size); every matrix of the model is perturbed independently under its own noise
// layer id (Alg. 1: one E_i per parameter matrix), and the update applies the EGGROLL UPDATE box to each
// matrix in turn.  Host code here only sequences kernels and sizes the activation scratch.
#include "common.hpp"

namespace egg {

// activations of one chunk, carved out of one scratch allocation
struct Carver {
    char* p;
    size_t off = 0;
    void* take(size_t bytes)
    {
        void* r = p + off;
        off += (bytes + 255) & ~size_t(255);
        return r;
    }
};

static int64_t pick_chunk(int64_t members, int S, int64_t chunk_members, int64_t max_rows)
{
    int64_t cm = chunk_members > 0 ? chunk_members : std::max<int64_t>(1, max_rows / S);
    return std::min(cm, members);
}

egg_status launch_mlp_stack_forward(eggroll_ctx* c, egg_key key, const egg_shape& s, int L, int d_ff, float sigma,
                                    const void* W1, const void* W2, const void* X, void* Y, int64_t chunk_members)
{
    const int d = s.d_in, S = s.rows_per_member;
    const int64_t cm = pick_chunk(s.member_count, S, chunk_members, int64_t(1) << 18);
    const size_t rows_max = (size_t)cm * S;
    auto pad = [](size_t b) { return (b + 255) & ~size_t(255); };
    // Rank 1: the up-projection's epilogue also projects what it stores onto the down-projection's factors, where it can, so
    // that the widest activation is not read a second time by a projection pass.  (At rank 2 and 4 the form exists too, but
    // measured on 2^18 rows of 2048 -> 8192 -> 2048 it only breaks even -- rank 4, 64 rows per member: 15.5 against 15.4 ms
    // for the pair of layers; rank 2: 15.0 against 15.1 -- because the factors it reads have to be materialised first,
    // 4096 x 8192 x 4 normals per chunk, where the projection pass draws them on the fly.)
    egg_shape probe = s;
    probe.member_count = cm;
    probe.d_out = d_ff;
    const bool fuse_dn = s.rank == 1 && forward_fuses_next_projection(probe, EGG_BF16, EGG_BF16, sigma, EGG_ACT_GELU, false);
    size_t need = pad(rows_max * d_ff * 2) + pad(rows_max * d * 2);
    if (fuse_dn) need += pad((size_t)cm * d_ff * s.rank * 2) + pad(rows_max * s.rank * sizeof(float));
    egg_status st = reserve(c, c->model, need);
    if (st != EGG_OK) return st;
    for (int64_t m0 = 0; m0 < s.member_count; m0 += cm) {
        const int64_t n = std::min(cm, s.member_count - m0);
        const size_t r0 = (size_t)m0 * S;
        Carver cv{(char*)c->model.p};
        void* u = cv.take(rows_max * d_ff * 2);
        void* h = cv.take(rows_max * d * 2);
        void* Bdn = fuse_dn ? cv.take((size_t)cm * d_ff * s.rank * 2) : nullptr;
        float* tdn = fuse_dn ? (float*)cv.take(rows_max * s.rank * sizeof(float)) : nullptr;
        egg_shape up = s, dn = s;
        up.member_begin = dn.member_begin = s.member_begin + m0;
        up.member_count = dn.member_count = n;
        up.d_out = d_ff; up.d_in = d;
        dn.d_out = d; dn.d_in = d_ff;
        // (a last chunk with fewer members may fall below the tile count the fused form needs)
        const bool fuse = fuse_dn && forward_fuses_next_projection(up, EGG_BF16, EGG_BF16, sigma, EGG_ACT_GELU, false);
        const char* in = (const char*)X + r0 * d * 2;
        for (int l = 0; l < L; ++l) {
            const egg_key k1{key.seed, key.step, key.layer + 2u * (uint32_t)l}, k2{key.seed, key.step, key.layer + 2u * (uint32_t)l + 1u};
            NextProjection np{Bdn, tdn};
            if (fuse) {
                // the down-projection's factors B_i over d_ff for this chunk's members, as its projection pass would draw them
                st = launch_noise(c, make_stream_key(key.seed, key.step, k2.layer, 1), (uint32_t)up.member_begin, n, (int64_t)d_ff * s.rank,
                                  EGG_BF16, EGG_NORMAL, 0, Bdn);
                if (st != EGG_OK) return st;
            }
            st = forward_linear(c, k1, up, EGG_BF16, EGG_BF16, sigma, EGG_ACT_GELU, (const char*)W1 + (size_t)l * d_ff * d * 2, in, u,
                                nullptr, nullptr, nullptr, nullptr, nullptr, fuse ? &np : nullptr);
            if (st != EGG_OK) return st;
            void* out = l == L - 1 ? (void*)((char*)Y + r0 * d * 2) : h;
            st = forward_linear(c, k2, dn, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, (const char*)W2 + (size_t)l * d * d_ff * 2, u, out,
                                nullptr, nullptr, nullptr, nullptr, fuse ? tdn : nullptr);
            if (st != EGG_OK) return st;
            in = (const char*)h;
        }
    }
    return EGG_OK;
}

// G = scale * sum_i f_i A_i B_i^T into scratch, then W += lr * G rounded to bf16, for one matrix
static egg_status update_matrix(eggroll_ctx* c, egg_key key, uint32_t layer, const egg_shape& s, int d_out, int d_in,
                                const float* fitness, float scale, float lr, void* W)
{
    egg_shape sh = s;
    sh.d_out = d_out;
    sh.d_in = d_in;
    egg_status st = reserve(c, c->model_g, (size_t)d_out * d_in * sizeof(float));
    if (st != EGG_OK) return st;
    return launch_update(c, make_stream_key(key.seed, key.step, layer, 0), make_stream_key(key.seed, key.step, layer, 1), sh, EGG_BF16,
                         fitness, scale, 0, (float*)c->model_g.p, W, EGG_BF16, lr, nullptr, nullptr, false);
}

egg_status launch_mlp_stack_update(eggroll_ctx* c, egg_key key, const egg_shape& s, int L, int d_ff, const float* fitness,
                                   float scale, float lr, void* W1, void* W2)
{
    const int d = s.d_in;
    for (int l = 0; l < L; ++l) {
        egg_status st = update_matrix(c, key, key.layer + 2u * (uint32_t)l, s, d_ff, d, fitness, scale, lr, (char*)W1 + (size_t)l * d_ff * d * 2);
        if (st != EGG_OK) return st;
        st = update_matrix(c, key, key.layer + 2u * (uint32_t)l + 1u, s, d, d_ff, fitness, scale, lr, (char*)W2 + (size_t)l * d * d_ff * 2);
        if (st != EGG_OK) return st;
    }
    return EGG_OK;
}

egg_status launch_decoder_forward(eggroll_ctx* c, egg_key key, const egg_shape& s, const egg_decoder_cfg& cfg,
                                  const egg_decoder_weights& w, float sigma, const int32_t* tokens, void* logits, float* loglik,
                                  int64_t chunk_members)
{
    const int d = cfg.d_model, ff = cfg.d_ff, V = cfg.vocab, L = cfg.layers, S = s.rows_per_member;
    const int hd = d / cfg.heads;
    const int64_t cm = pick_chunk(s.member_count, S, chunk_members, int64_t(1) << 18);
    const size_t rows_max = (size_t)cm * S;
    auto pad = [](size_t b) { return (b + 255) & ~size_t(255); };
    size_t need = 5 * pad(rows_max * d * 2) + pad(rows_max * ff * 2);
    if (!logits) need += pad(rows_max * V * 2);
    // rank 1: the normalisation passes form the projections of the layers that read their output (q, k, v; up; head),
    // so those layers' inputs are not read a second time by a projection pass
    const bool fuse_proj = sigma != 0.0f && s.rank == 1;
    if (fuse_proj) need += 3 * (pad((size_t)cm * d * 2) + pad(rows_max * sizeof(float))) + pad((size_t)cm * ff * 2) + pad(rows_max * sizeof(float));
    egg_status st = reserve(c, c->model, need);
    if (st != EGG_OK) return st;
    const size_t dd = (size_t)d * d * 2, dff = (size_t)d * ff * 2;
    for (int64_t m0 = 0; m0 < s.member_count; m0 += cm) {
        const int64_t n = std::min(cm, s.member_count - m0);
        const int64_t rows = n * S;
        const size_t r0 = (size_t)m0 * S;
        Carver cv{(char*)c->model.p};
        void* x = cv.take(rows_max * d * 2);
        void* h = cv.take(rows_max * d * 2);
        void* q = cv.take(rows_max * d * 2);
        void* k = cv.take(rows_max * d * 2);
        void* v = cv.take(rows_max * d * 2);
        void* u = cv.take(rows_max * ff * 2);
        void* lg = logits ? (void*)((char*)logits + r0 * V * 2) : cv.take(rows_max * V * 2);
        void* Bf[3] = {nullptr, nullptr, nullptr};
        float* tf[3] = {nullptr, nullptr, nullptr};
        if (fuse_proj)
            for (int j = 0; j < 3; ++j) {
                Bf[j] = cv.take((size_t)cm * d * 2);
                tf[j] = (float*)cv.take(rows_max * sizeof(float));
            }
        void* Bdn = nullptr;   // the down-projection's factors over d_ff and its projections, formed by the up-projection's epilogue
        float* tdn = nullptr;
        if (fuse_proj) {
            Bdn = cv.take((size_t)cm * ff * 2);
            tdn = (float*)cv.take(rows_max * sizeof(float));
        }
        // factors B_i of the layer with noise id `layer` for this chunk's members, as the projection pass would draw them
        auto gen_b = [&](uint32_t layer, void* out, int len) {
            return launch_noise(c, make_stream_key(key.seed, key.step, layer, 1), (uint32_t)(s.member_begin + m0), n, len, EGG_BF16, EGG_NORMAL, 0, out);
        };
        egg_shape sq = s;
        sq.member_begin = s.member_begin + m0;
        sq.member_count = n;
        sq.d_out = d; sq.d_in = d;
        egg_shape sup = sq, sdn = sq, shd = sq;
        sup.d_out = ff;
        sdn.d_in = ff;
        shd.d_out = V;
        const int32_t* tok = tokens + r0;
        if ((st = launch_embed_rows(c, rows, d, V, w.emb, tok, x)) != EGG_OK) return st;
        for (int l = 0; l < L; ++l) {
            const uint32_t lid = key.layer + 6u * (uint32_t)l;
            auto kk = [&](uint32_t j) { return egg_key{key.seed, key.step, lid + j}; };
            if (fuse_proj) {
                for (uint32_t j = 0; j < 3; ++j)
                    if ((st = gen_b(lid + j, Bf[j], d)) != EGG_OK) return st;
                if ((st = launch_rmsnorm_proj(c, rows, S, d, cfg.rms_eps, (const char*)w.norm1 + (size_t)l * d * 2, x, h, 3, Bf, tf)) != EGG_OK) return st;
            } else if ((st = launch_rmsnorm(c, rows, d, cfg.rms_eps, (const char*)w.norm1 + (size_t)l * d * 2, x, h)) != EGG_OK) return st;
            if ((st = forward_linear(c, kk(0), sq, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, (const char*)w.wq + l * dd, h, q, nullptr, nullptr, nullptr, nullptr, tf[0])) != EGG_OK) return st;
            if ((st = forward_linear(c, kk(1), sq, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, (const char*)w.wk + l * dd, h, k, nullptr, nullptr, nullptr, nullptr, tf[1])) != EGG_OK) return st;
            if ((st = forward_linear(c, kk(2), sq, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, (const char*)w.wv + l * dd, h, v, nullptr, nullptr, nullptr, nullptr, tf[2])) != EGG_OK) return st;
            // the attention kernel forms the o-projection's projections of the rows it writes
            if (fuse_proj && (st = gen_b(lid + 3, Bf[0], d)) != EGG_OK) return st;
            if ((st = launch_attention(c, n, S, cfg.heads, hd, q, k, v, h, fuse_proj ? Bf[0] : nullptr, fuse_proj ? tf[0] : nullptr)) != EGG_OK) return st;
            if ((st = forward_linear(c, kk(3), sq, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, (const char*)w.wo + l * dd, h, x, nullptr, nullptr, x, nullptr, fuse_proj ? tf[0] : nullptr)) != EGG_OK) return st;
            if (fuse_proj) {
                if ((st = gen_b(lid + 4, Bf[0], d)) != EGG_OK) return st;
                if ((st = launch_rmsnorm_proj(c, rows, S, d, cfg.rms_eps, (const char*)w.norm2 + (size_t)l * d * 2, x, h, 1, Bf, tf)) != EGG_OK) return st;
            } else if ((st = launch_rmsnorm(c, rows, d, cfg.rms_eps, (const char*)w.norm2 + (size_t)l * d * 2, x, h)) != EGG_OK) return st;
            // the up-projection's epilogue also projects what it stores onto the down-projection's factors, where it can
            const bool fuse_dn = fuse_proj && forward_fuses_next_projection(sup, EGG_BF16, EGG_BF16, sigma, EGG_ACT_GELU, false);
            NextProjection np{Bdn, tdn};
            if (fuse_dn && (st = gen_b(lid + 5, Bdn, ff)) != EGG_OK) return st;
            if ((st = forward_linear(c, kk(4), sup, EGG_BF16, EGG_BF16, sigma, EGG_ACT_GELU, (const char*)w.w_up + l * dff, h, u, nullptr, nullptr, nullptr, nullptr, tf[0], fuse_dn ? &np : nullptr)) != EGG_OK) return st;
            if ((st = forward_linear(c, kk(5), sdn, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, (const char*)w.w_down + l * dff, u, x, nullptr, nullptr, x, nullptr, fuse_dn ? tdn : nullptr)) != EGG_OK) return st;
        }
        const egg_key kh{key.seed, key.step, key.layer + 6u * (uint32_t)L};
        if (fuse_proj) {
            if ((st = gen_b(kh.layer, Bf[0], d)) != EGG_OK) return st;
            if ((st = launch_rmsnorm_proj(c, rows, S, d, cfg.rms_eps, w.norm_f, x, h, 1, Bf, tf)) != EGG_OK) return st;
        } else if ((st = launch_rmsnorm(c, rows, d, cfg.rms_eps, w.norm_f, x, h)) != EGG_OK) return st;
        if ((st = forward_linear(c, kh, shd, EGG_BF16, EGG_BF16, sigma, EGG_ACT_NONE, w.head, h, lg, nullptr, nullptr, nullptr, nullptr, tf[0])) != EGG_OK) return st;
        if (loglik && (st = launch_token_loglik(c, n, S, V, lg, tok, loglik + r0)) != EGG_OK) return st;
    }
    return EGG_OK;
}

egg_status launch_decoder_update(eggroll_ctx* c, egg_key key, const egg_shape& s, const egg_decoder_cfg& cfg, const float* fitness,
                                 float scale, float lr, const egg_decoder_weights& w)
{
    const int d = cfg.d_model, ff = cfg.d_ff, V = cfg.vocab, L = cfg.layers;
    const size_t dd = (size_t)d * d * 2, dff = (size_t)d * ff * 2;
    egg_status st;
    for (int l = 0; l < L; ++l) {
        const uint32_t lid = key.layer + 6u * (uint32_t)l;
        char* sq[4] = {(char*)w.wq, (char*)w.wk, (char*)w.wv, (char*)w.wo};
        for (uint32_t j = 0; j < 4; ++j)
            if ((st = update_matrix(c, key, lid + j, s, d, d, fitness, scale, lr, sq[j] + l * dd)) != EGG_OK) return st;
        if ((st = update_matrix(c, key, lid + 4, s, ff, d, fitness, scale, lr, (char*)w.w_up + l * dff)) != EGG_OK) return st;
        if ((st = update_matrix(c, key, lid + 5, s, d, ff, fitness, scale, lr, (char*)w.w_down + l * dff)) != EGG_OK) return st;
    }
    return update_matrix(c, key, key.layer + 6u * (uint32_t)L, s, V, d, fitness, scale, lr, w.head);
}

}  // namespace egg

// Host-side plumbing shared by the translation units of libeggroll: the context (stream, scratch,
// error text, optional per-kernel event timing) and launch helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <map>
#include <string>
#include <vector>

#include "../../include/eggroll.h"
#include "rng.hpp"

struct eggroll_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    int compute_units = 256;  // of the device (grid size of persistent kernels)
    int cache_layout = 0;  // egg_cache_layout of the forward/update caches
    bool conservative_waits = false;  // diagnostic: kernels with counted s_waitcnt wait for everything instead

    // scratch, grown on demand and kept for the life of the context
    struct Buf {
        void* p = nullptr;
        size_t bytes = 0;
    };
    Buf t_buf;        // projections t[R][r] fp32 (forward) / int32 dots (int8 path)
    Buf a_buf, b_buf; // materialised [member][d][r] factors when the caller keeps no cache
    Buf fnorm;        // update: power-of-two normaliser of the fitness vector
    Buf pack_a;       // update: K-packed diag(f)A panel
    Buf pack_b;       // update: K-packed B panel
    Buf i8_a, i8_b;   // int8 path: factors, generated once per episode
    Buf i8_h;         // int8 path: ping-pong state
    Buf gru;          // integer GRU cell: factors of its four matrices, gate and matmul intermediates
    Buf zero_page;    // 256 zero bytes (K-tail loads of the GEMM core)
    Buf lut;          // integer log-likelihood: EXP2 table and the thresholds that invert LOG2
    Buf norm_tab;     // integer normal noise: the 65536-entry table round(16 z) (uploaded on first use)
    Buf model;        // multi-layer drivers: activations of one chunk of members
    Buf model_g;      // multi-layer updates: fp32 G of the matrix being updated
    Buf proj_part;    // fused next-layer projection: per (128-row slab of d_out, row) partial sums
    Buf next_b;       // fused next-layer projection through the C ABI: the next layer's factors B'[member][d_out]
    // buffers that a later, larger call outgrew: kept until eggroll_trim / eggroll_destroy, because work already
    // enqueued -- or a HIP graph captured earlier -- may still hold their addresses
    std::vector<Buf> retired;
    uint64_t scratch_generation = 0;  // bumped whenever a scratch buffer is replaced

    // profiling
    bool prof = false;
    struct Rec {
        const char* name;
        hipEvent_t a, b;
    };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> free_events;
    std::map<std::string, int> shaped_names;  // interned "kernel[d_out x d_in]" labels (node addresses are stable)
};

namespace egg {

egg_status fail(eggroll_ctx* c, egg_status s, const char* fmt, ...);
egg_status check_hip(eggroll_ctx* c, hipError_t e, const char* what);
egg_status reserve(eggroll_ctx* c, eggroll_ctx::Buf& b, size_t bytes);

// RAII bracket: records events around one kernel launch when profiling is on
struct KernelScope {
    eggroll_ctx* c;
    const char* name;
    hipEvent_t a = nullptr, b = nullptr;
    KernelScope(eggroll_ctx* ctx, const char* n);
    ~KernelScope();
};

// A kernel that needs more than the default dynamic LDS must have its limit raised; this does it on first use (and again
// only if a later launch needs more), instead of on every launch.  The limit belongs to the function, not to a context:
// the bookkeeping is process-wide (per device).
egg_status ensure_dynamic_lds(eggroll_ctx* c, const void* kern, size_t bytes, const char* what);

// label of a per-shape timing row, e.g. forward_gemm_bf16[8192x2048]; only built when profiling is on
inline const char* shaped_name(eggroll_ctx* c, const char* base, int d_out, int d_in)
{
    if (!c->prof) return base;
    char buf[96];
    snprintf(buf, sizeof buf, "%s[%dx%d]", base, d_out, d_in);
    return c->shaped_names.emplace(buf, 0).first->first.c_str();
}

// int_bound arguments: a bound in [0, 127] (uniform integers) or EGG_INT_NOISE_NORMAL16 (the table of round(16 z))
inline bool valid_int_bound(int b) { return (b >= 0 && b <= 127) || b == EGG_INT_NOISE_NORMAL16; }
// largest |value| the selected integer noise can take: 16 * Phi^-1(1 - 2^-17) rounds to 69 for the table
inline int noise_max(int b) { return b == EGG_INT_NOISE_NORMAL16 ? 69 : b; }
void normal_int_table(int8_t* out);  // host: fills the 65536 entries

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

egg_status validate_shape(eggroll_ctx* c, const egg_shape* s, bool need_rows, bool forward_pass);

// entry points implemented per translation unit (kernel launchers)
egg_status launch_noise(eggroll_ctx* c, const StreamKey& k, uint32_t member_begin, int64_t members, int64_t n,
                        egg_dtype dtype, egg_dist dist, int int_bound, void* out);
egg_status launch_project(eggroll_ctx* c, const StreamKey& kb, const egg_shape& s, egg_dtype io, const void* X,
                          float* t, void* B_cache, bool panel);
// A layer whose output feeds the next perturbed layer directly (up-projection -> down-projection) can form that
// layer's projections (same rank, 1, 2 or 4) in its own epilogue, from the bf16 values it stores: B = the next layer's
// factors [member][d_out][rank] bf16, t = where the projections [rows][rank] go.  Supported where
// forward_fuses_next_projection says so.
struct NextProjection {
    const void* B;
    float* t;
};
bool forward_fuses_next_projection(const egg_shape& s, egg_dtype io, egg_dtype yd, float sigma, egg_act act, bool resid);
egg_status launch_forward_gemm(eggroll_ctx* c, const StreamKey& ka, const egg_shape& s, egg_dtype io, egg_dtype yd,
                               float sigma, egg_act act, const void* W, const void* X, void* Y, const float* t,
                               void* A_cache, const void* resid = nullptr, const NextProjection* next = nullptr);
egg_status launch_update(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                         egg_dtype noise_dtype, const float* fitness, float scale, int accumulate, float* G, void* W,
                         egg_dtype w_dtype, float lr, const void* A_cache, const void* B_cache, bool b_panel);
egg_status forward_linear(eggroll_ctx* c, egg_key key, const egg_shape& shape, egg_dtype io_dtype, egg_dtype y_dtype, float sigma,
                          egg_act act, const void* W, const void* X, void* Y, void* A_cache, void* B_cache, const void* resid,
                          float* t_fixed = nullptr, const float* t_ready = nullptr, const NextProjection* next = nullptr);
egg_status checked_forward(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype io_dtype, egg_dtype y_dtype,
                           float sigma, egg_act act, const void* W, const void* X, const void* R_in, bool need_r, void* Y,
                           void* A_cache, void* B_cache, float* t_fixed, size_t t_capacity, const float* t_in = nullptr,
                           bool want_next = false, uint32_t next_layer = 0, float* t_next = nullptr);
// unperturbed glue of the decoder workload
egg_status launch_embed_rows(eggroll_ctx* c, int64_t rows, int d, int vocab, const void* emb, const int32_t* tokens, void* X);
egg_status launch_rmsnorm(eggroll_ctx* c, int64_t rows, int d, float eps, const void* gain, const void* X, void* Y);
egg_status launch_rmsnorm_proj(eggroll_ctx* c, int64_t rows, int S, int d, float eps, const void* gain, const void* X, void* Y, int nc,
                               const void* const* B, float* const* t);
// Bo != NULL: also t_next[row] = sum_j O[row][j] * Bo[member][j] (Bo: [members][heads * head_dim] bf16, rank-1 factors of the
// layer that reads O)
egg_status launch_attention(eggroll_ctx* c, int64_t members, int S, int heads, int head_dim, const void* Q, const void* K,
                            const void* V, void* O, const void* Bo = nullptr, float* t_next = nullptr);
// t[n] = sum over slabs p of part[p][n], in slab order
egg_status launch_sum_slabs(eggroll_ctx* c, const float* part, int slabs, int64_t R, float* t);
egg_status launch_token_loglik(eggroll_ctx* c, int64_t members, int S, int vocab, const void* logits, const int32_t* tokens, float* out);
// multi-layer drivers
egg_status launch_mlp_stack_forward(eggroll_ctx* c, egg_key key, const egg_shape& s, int L, int d_ff, float sigma,
                                    const void* W1, const void* W2, const void* X, void* Y, int64_t chunk_members);
egg_status launch_mlp_stack_update(eggroll_ctx* c, egg_key key, const egg_shape& s, int L, int d_ff, const float* fitness,
                                   float scale, float lr, void* W1, void* W2);
egg_status launch_decoder_forward(eggroll_ctx* c, egg_key key, const egg_shape& s, const egg_decoder_cfg& cfg,
                                  const egg_decoder_weights& w, float sigma, const int32_t* tokens, void* logits, float* loglik,
                                  int64_t chunk_members);
egg_status launch_decoder_update(eggroll_ctx* c, egg_key key, const egg_shape& s, const egg_decoder_cfg& cfg, const float* fitness,
                                 float scale, float lr, const egg_decoder_weights& w);
egg_status launch_forward_i8(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                             int int_bound, int corr_shift, int out_shift, int steps, const int8_t* W,
                             const int8_t* H_in, int8_t* H_out);

// GRU gating fused into the epilogue of an integer matmul (see I8Args in k_int8.hip)
struct I8Gate {
    int mode;  // 1: f and f^,  2: h
    const int8_t *other, *state, *f, *bias;
    int8_t* out2;
};
egg_status launch_i8_matmul(eggroll_ctx* c, const int8_t* A, const int8_t* B, int anti, int64_t rows, int d_out, int d_in,
                            int int_bound, int corr_shift, int out_shift, const int8_t* W, const int8_t* src, int8_t* dst,
                            int* dots, bool dots_ready, const I8Gate* gate, const int8_t* B_next = nullptr, int* dots_next = nullptr);
egg_status launch_zero_i32(eggroll_ctx* c, int* p0, int* p1, int64_t n);  // clears one or two int32 vectors (p1 may be NULL)
egg_status launch_dots_i8(eggroll_ctx* c, const int8_t* X0, const int8_t* B0, const int8_t* B1, const int8_t* X1, const int8_t* B2,
                          int64_t rows, int d, int anti, int* d0, int* d1, int* d2);
// factors, weights and intermediates of one GRU cell (matrix order: Wf, Uf, Wh, Uh)
struct GruStep {
    const int8_t *A[4], *B[4], *W[4];
    const int8_t *bf, *bh;
    int8_t *a1, *a3, *f, *fh;  // [rows][D] each
    int* dot[4];               // [rows] each: u.B_Wf, s.B_Uf, u.B_Wh, f^.B_Uh
    bool u_dots_ready = false; // dot[0] and dot[2] were filled by whoever produced u
    bool s_dot_ready = false;  // dot[1] was filled by the previous step's last epilogue
    bool fh_dot_zeroed = false;// dot[3] is zero: the first gate's epilogue accumulates f^.B_Uh there
    int* dot_s_next = nullptr; // zeroed [rows]: the last epilogue accumulates h.B_Uf for the next step there
};
egg_status launch_gru_step(eggroll_ctx* c, const GruStep& g, int anti, int64_t rows, int D, int int_bound, int corr_shift,
                           int out_shift, const int8_t* u, const int8_t* state, int8_t* next);
egg_status launch_gru_i8(eggroll_ctx* c, egg_key key, const egg_shape& s, int int_bound, int corr_shift, int out_shift,
                         int steps, const int8_t* const W[4], const int8_t* bf, const int8_t* bh, const int8_t* U,
                         const int8_t* S_in, int8_t* S_out);
// optional by-products of the normalisation pass: dot products of the normalised rows with up to two factor
// arrays (what the matmuls that consume u need), and up to two int32 vectors cleared for later accumulation
struct LnExtras {
    const int8_t* B[2] = {nullptr, nullptr};  // [ids][D]
    int* dot[2] = {nullptr, nullptr};         // [rows]
    int* zero[2] = {nullptr, nullptr};        // [rows]
    int anti = 0;
};
egg_status launch_layernorm_i8(eggroll_ctx* c, const int8_t* add, int8_t* y, const int8_t* ln, int8_t* u, int64_t rows, int D,
                               const LnExtras* extras = nullptr);
egg_status launch_embed_i8(eggroll_ctx* c, egg_key key, const egg_shape& s, int int_bound, int corr_shift, const int8_t* emb,
                           const uint8_t* tokens, int8_t* Y);
egg_status launch_egg_forward_i8(eggroll_ctx* c, egg_key key, const egg_shape& s, int L, int int_bound, int corr_shift, int T,
                                 const egg_model_i8& P, const uint8_t* tokens, const int8_t* S_in, int8_t* S_out,
                                 int8_t* logits);
egg_status launch_loglik_i8(eggroll_ctx* c, int64_t rows, const int8_t* logits, const uint8_t* targets, int accumulate, int32_t* out);
egg_status launch_update_i8(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                            int int_bound, const int8_t* F, int32_t threshold, int8_t* theta, int32_t* E_out);

}  // namespace egg

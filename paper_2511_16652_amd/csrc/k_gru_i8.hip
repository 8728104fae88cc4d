// Integer GRU cell of the int8 model (App. "GRU" of the EGG architecture), a population of states advanced
// over a sequence of inputs, bit-exact:
//   f  = I8(u @ Wf^T + s @ Uf^T + bf)              f^ = I8(((f + 127) s) >> 8)
//   h^ = I8(u @ Wh^T + f^ @ Uh^T + bh)             h  = I8(s + I8(((f + 127)(h^ - s)) >> 8))
// "@" is the perturbed scaled matmul (App. "Matrix Multiplication", "Adding EGGROLL Perturbations"); the
// four matrices carry independent rank-1 perturbations (noise layers layer .. layer+3), generated once
// per call -- a member's perturbation is fixed while it is evaluated (Alg. 1).  Per time step: four int8
// MFMA matmuls; the gates are fused into the epilogues of the second and fourth (a lane finishes 16 consecutive
// entries of a row there, so the gate operands are 16-byte loads), three of the four u.B / s.B dot products
// share one pass over u and s.
#include "common.hpp"

namespace egg {

// One time step of the cell for all rows: u and the old state in, the new state out.
egg_status launch_gru_step(eggroll_ctx* c, const GruStep& g, int anti, int64_t rows, int D, int int_bound, int corr_shift,
                           int out_shift, const int8_t* u, const int8_t* state, int8_t* next)
{
    egg_status st;
    // dot products nobody has delivered yet: u . B_Wf, u . B_Wh and s . B_Uf share one pass over u and s
    if (!g.u_dots_ready) {
        if ((st = launch_dots_i8(c, u, g.B[0], g.B[2], g.s_dot_ready ? nullptr : state, g.s_dot_ready ? nullptr : g.B[1], rows, D, anti,
                                 g.dot[0], g.dot[2], g.dot[1])) != EGG_OK) return st;
    } else if (!g.s_dot_ready) {
        if ((st = launch_dots_i8(c, state, g.B[1], nullptr, nullptr, nullptr, rows, D, anti, g.dot[1], nullptr, nullptr)) != EGG_OK) return st;
    }
    // the gates ride in the epilogues of the second matmul of each pair: a2 and a4 never reach memory
    const I8Gate g1{1, g.a1, state, nullptr, g.bf, g.fh}, g2{2, g.a3, state, g.f, g.bh, nullptr};
#define EGG_MM(M, SRC, DST, READY, GATE, BN, DN) \
    if ((st = launch_i8_matmul(c, g.A[M], g.B[M], anti, rows, D, D, int_bound, corr_shift, out_shift, g.W[M], SRC, DST, g.dot[M], READY, GATE, BN, DN)) != EGG_OK) return st;
    EGG_MM(0, u, g.a1, true, nullptr, nullptr, nullptr)
    EGG_MM(2, u, g.a3, true, nullptr, nullptr, nullptr)
    // writes f and f^; f^ . B_Uh is accumulated on the way when dot[3] was cleared for it
    EGG_MM(1, state, g.f, true, &g1, g.fh_dot_zeroed ? g.B[3] : nullptr, g.fh_dot_zeroed ? g.dot[3] : nullptr)
    // writes h; h . B_Uf for the next time step on request
    EGG_MM(3, g.fh, next, g.fh_dot_zeroed, &g2, g.dot_s_next ? g.B[1] : nullptr, g.dot_s_next)
#undef EGG_MM
    return EGG_OK;
}

egg_status launch_gru_i8(eggroll_ctx* c, egg_key key, const egg_shape& s, int int_bound, int corr_shift, int out_shift,
                         int steps, const int8_t* const W[4], const int8_t* bf, const int8_t* bh, const int8_t* U,
                         const int8_t* S_in, int8_t* S_out)
{
    const int D = s.d_in;
    const int64_t rows = s.member_count;
    const int anti = s.antithetic ? 1 : 0;
    const int64_t ids = anti ? rows / 2 : rows;
    const uint32_t first_id = (uint32_t)(anti ? s.member_begin / 2 : s.member_begin);
    const size_t fac = ((size_t)ids * D + 255) & ~size_t(255);   // one factor buffer
    const size_t act = ((size_t)rows * D + 255) & ~size_t(255);  // one activation buffer
    const size_t dots = ((size_t)rows * sizeof(int) + 255) & ~size_t(255);  // one vector of dot products
    egg_status st;
    // 8 factor buffers; a1, a3, f, f^ and two ping-pong states; five vectors of dot products (s . B_Uf twice:
    // the one this step reads and the one its last epilogue accumulates for the next step)
    if ((st = reserve(c, c->gru, 8 * fac + 6 * act + 5 * dots)) != EGG_OK) return st;
    char* base = (char*)c->gru.p;
    int8_t *A[4], *B[4];
    for (int m = 0; m < 4; ++m) {
        A[m] = (int8_t*)(base + (2 * m) * fac);
        B[m] = (int8_t*)(base + (2 * m + 1) * fac);
        if ((st = launch_noise(c, make_stream_key(key.seed, key.step, key.layer + m, 0), first_id, ids, D, EGG_I8, EGG_UNIFORM_INT, int_bound, A[m])) != EGG_OK) return st;
        if ((st = launch_noise(c, make_stream_key(key.seed, key.step, key.layer + m, 1), first_id, ids, D, EGG_I8, EGG_UNIFORM_INT, int_bound, B[m])) != EGG_OK) return st;
    }
    int8_t* buf[6];
    for (int b = 0; b < 6; ++b) buf[b] = (int8_t*)(base + 8 * fac + b * act);
    int* dot[5];
    for (int m = 0; m < 5; ++m) dot[m] = (int*)(base + 8 * fac + 6 * act + m * dots);
    int* dot_s[2] = {dot[1], dot[4]};

    GruStep g;
    for (int m = 0; m < 4; ++m) { g.A[m] = A[m]; g.B[m] = B[m]; g.W[m] = W[m]; g.dot[m] = dot[m]; }
    g.a1 = buf[0]; g.a3 = buf[1]; g.f = buf[2]; g.fh = buf[3]; g.bf = bf; g.bh = bh;
    g.fh_dot_zeroed = true;
    const int8_t* state = S_in;
    for (int t = 0; t < steps; ++t) {
        int8_t* next = (t == steps - 1) ? S_out : buf[4 + (t & 1)];
        g.dot[1] = dot_s[t & 1];
        g.s_dot_ready = t > 0;
        g.dot_s_next = t + 1 < steps ? dot_s[(t + 1) & 1] : nullptr;
        if ((st = launch_zero_i32(c, g.dot[3], g.dot_s_next, rows)) != EGG_OK) return st;
        if ((st = launch_gru_step(c, g, anti, rows, D, int_bound, corr_shift, out_shift, U + (size_t)t * rows * D, state, next)) != EGG_OK) return st;
        state = next;
    }
    return EGG_OK;
}

}  // namespace egg

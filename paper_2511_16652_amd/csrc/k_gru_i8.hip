// Integer GRU cell of the int8 model (App. "GRU" of the EGG architecture), a population of states advanced
// over a sequence of inputs, bit-exact:
//   f  = I8(u @ Wf^T + s @ Uf^T + bf)              f^ = I8(((f + 127) s) >> 8)
//   h^ = I8(u @ Wh^T + f^ @ Uh^T + bh)             h  = I8(s + I8(((f + 127)(h^ - s)) >> 8))
// "@" is the perturbed scaled matmul (App. "Matrix Multiplication", "Adding EGGROLL Perturbations"); the
// four matrices carry independent rank-1 perturbations (noise layers layer .. layer+3), generated once
// per call -- a member's perturbation is fixed while it is evaluated (Alg. 1).  Per time step: four int8
// MFMA matmuls and two elementwise gate kernels (16 entries per thread, HBM-bound).
#include "common.hpp"

namespace egg {

typedef uint32_t gu32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int sx8(uint32_t w, int b) { return (int)(int8_t)(w >> (8 * b)); }
__device__ __forceinline__ int clip127(int v) { return min(127, max(-127, v)); }

// f = I8(a1 + a2 + bf), f^ = I8(((f + 127) s) >> 8)
__global__ __launch_bounds__(256) void gru_gate1_kernel(const gu32x4* __restrict__ a1, const gu32x4* __restrict__ a2,
                                                        const gu32x4* __restrict__ s, const gu32x4* __restrict__ bf, int d16,
                                                        int64_t n16, gu32x4* __restrict__ f, gu32x4* __restrict__ fh)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const gu32x4 x1 = a1[i], x2 = a2[i], sv = s[i], b = bf[i % d16];
    gu32x4 of, oh;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t pf = 0, ph = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int fv = clip127(sx8(x1[w], e) + sx8(x2[w], e) + sx8(b[w], e));
            const int hv = clip127(((fv + 127) * sx8(sv[w], e)) >> 8);  // arithmetic shift: floor
            pf |= ((uint32_t)fv & 0xFFu) << (8 * e);
            ph |= ((uint32_t)hv & 0xFFu) << (8 * e);
        }
        of[w] = pf;
        oh[w] = ph;
    }
    f[i] = of;
    fh[i] = oh;
}

// h^ = I8(a3 + a4 + bh), h = I8(s + I8(((f + 127)(h^ - s)) >> 8))
__global__ __launch_bounds__(256) void gru_gate2_kernel(const gu32x4* __restrict__ a3, const gu32x4* __restrict__ a4,
                                                        const gu32x4* __restrict__ f, const gu32x4* __restrict__ s,
                                                        const gu32x4* __restrict__ bh, int d16, int64_t n16, gu32x4* __restrict__ h)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const gu32x4 x3 = a3[i], x4 = a4[i], fv4 = f[i], sv = s[i], b = bh[i % d16];
    gu32x4 o;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t p = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int hh = clip127(sx8(x3[w], e) + sx8(x4[w], e) + sx8(b[w], e));
            const int sj = sx8(sv[w], e);
            const int delta = clip127(((sx8(fv4[w], e) + 127) * (hh - sj)) >> 8);
            p |= ((uint32_t)clip127(sj + delta) & 0xFFu) << (8 * e);
        }
        o[w] = p;
    }
    h[i] = o;
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
    const size_t dots = ((size_t)rows * sizeof(int) + 255) & ~size_t(255);
    egg_status st;
    // 8 factor buffers, a1..a4, f, f^, two ping-pong states, the dot products
    if ((st = reserve(c, c->gru, 8 * fac + 8 * act + dots)) != EGG_OK) return st;
    char* base = (char*)c->gru.p;
    int8_t *A[4], *B[4];
    for (int m = 0; m < 4; ++m) {
        A[m] = (int8_t*)(base + (2 * m) * fac);
        B[m] = (int8_t*)(base + (2 * m + 1) * fac);
        if ((st = launch_noise(c, make_stream_key(key.seed, key.step, key.layer + m, 0), first_id, ids, D, EGG_I8, EGG_UNIFORM_INT, int_bound, A[m])) != EGG_OK) return st;
        if ((st = launch_noise(c, make_stream_key(key.seed, key.step, key.layer + m, 1), first_id, ids, D, EGG_I8, EGG_UNIFORM_INT, int_bound, B[m])) != EGG_OK) return st;
    }
    int8_t* buf[8];
    for (int b = 0; b < 8; ++b) buf[b] = (int8_t*)(base + 8 * fac + b * act);
    int8_t *a1 = buf[0], *a2 = buf[1], *a3 = buf[2], *a4 = buf[3], *f = buf[4], *fh = buf[5];
    int* dot = (int*)(base + 8 * fac + 8 * act);
    const int64_t n16 = rows * D / 16;
    const dim3 eg((unsigned)((n16 + 255) / 256)), eb(256);

    const int8_t* state = S_in;
    for (int t = 0; t < steps; ++t) {
        const int8_t* u = U + (size_t)t * rows * D;
        int8_t* next = (t == steps - 1) ? S_out : buf[6 + (t & 1)];
#define EGG_MM(M, SRC, DST) \
        if ((st = launch_i8_matmul(c, A[M], B[M], anti, rows, D, D, int_bound, corr_shift, out_shift, W[M], SRC, DST, dot)) != EGG_OK) return st;
        EGG_MM(0, u, a1)
        EGG_MM(1, state, a2)
        EGG_MM(2, u, a3)
        {
            KernelScope ks(c, "gru_gate1");
            hipLaunchKernelGGL(gru_gate1_kernel, eg, eb, 0, c->stream, (const gu32x4*)a1, (const gu32x4*)a2, (const gu32x4*)state,
                               (const gu32x4*)bf, D / 16, n16, (gu32x4*)f, (gu32x4*)fh);
        }
        EGG_MM(3, fh, a4)
#undef EGG_MM
        {
            KernelScope ks(c, "gru_gate2");
            hipLaunchKernelGGL(gru_gate2_kernel, eg, eb, 0, c->stream, (const gu32x4*)a3, (const gu32x4*)a4, (const gu32x4*)f,
                               (const gu32x4*)state, (const gu32x4*)bh, D / 16, n16, (gu32x4*)next);
        }
        if ((st = check_hip(c, hipGetLastError(), "gru gates")) != EGG_OK) return st;
        state = next;
    }
    return EGG_OK;
}

}  // namespace egg

// Unperturbed glue of the decoder workload: token embedding gather, RMS normalisation, causal softmax
// attention over a member's own tokens, and the per-token log-likelihood of the next token.  The paper
// perturbs the matrix parameters of a model (Sec. 4.1; Alg. 1); everything here is identical in the
// perturbed and the unperturbed pass and exists so that the perturbed linear layers can be driven as a
// whole model.  All tensors are bf16 row-major [rows][d], rows member-major.
#include "common.hpp"
#include "gemm_core.hpp"

namespace egg {

// ---- embedding gather: X[row] = emb[token[row]] ----------------------------------------------------
__global__ __launch_bounds__(256) void embed_rows_kernel(const int32_t* __restrict__ tokens, const uint4* __restrict__ emb,
                                                         uint4* __restrict__ X, int64_t rows, int chunks, int vocab)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int tok = min(max(tokens[row], 0), vocab - 1);  // ids are validated by the caller; never read outside the table
    const uint4* src = emb + (int64_t)tok * chunks;
    uint4* dst = X + row * chunks;
    for (int c = lane; c < chunks; c += 64) dst[c] = src[c];
}

// ---- RMS normalisation: Y[row][k] = X[row][k] * gain[k] / sqrt(mean_k X[row][k]^2 + eps) -------------
// One wave per row.  Rows of up to 4096 values stay in the wave's registers between the sum of squares and the scaling
// (CPL = 16-byte chunks per lane, known at compile time); longer rows are read a second time.  (Counters showed the
// second read coming back from beyond the L2 for 0.6-0.9 of the row.)  HBM-bound: 2 d bytes in, 2 d out.
__device__ __forceinline__ void unpack8(const uint4& v, float (&x)[8])
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = bf16_lo(w[e]);
        x[2 * e + 1] = bf16_hi(w[e]);
    }
}

// NC > 0: the pass also forms the rank-1 projections t_c[row] = sum_k Y[row][k] B_c[member(row)][k] of up to three linear
// layers that consume Y (Sec. 4.2: the "batch of vector-vector dot products"), from the bf16 values it stores, in exactly the
// order of the stand-alone projection pass (lane = 16-byte chunk modulo 64, ascending; then the xor-shuffle tree): the same
// bits as that pass, without reading Y again.  B_c: materialised factors [member][d] (bf16).
struct NormProj {
    const uint16_t* B[3];
    float* t[3];
    int S;  // rows per member
};

template <int NC, int CPL>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint4* __restrict__ X, const uint4* __restrict__ gain,
                                                      uint4* __restrict__ Y, int64_t rows, int chunks, float inv_d, float eps,
                                                      NormProj np)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const uint4* xr = X + row * chunks;
    float ss = 0.f;
    uint4 keep[CPL > 0 ? CPL : 1];  // CPL > 0: chunks <= 64 CPL (the launcher's choice); same order of accumulation either way
    if constexpr (CPL > 0) {
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const int c = lane + 64 * i;
            keep[i] = c < chunks ? xr[c] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            float x[8];
            unpack8(keep[i], x);
            if (lane + 64 * i < chunks) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
            }
        }
    } else {
        for (int c = lane; c < chunks; c += 64) {
            float x[8];
            unpack8(xr[c], x);
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    const float r = 1.0f / sqrtf(ss * inv_d + eps);
    uint4* yr = Y + row * chunks;
    const int64_t member = NC > 0 ? row / np.S : 0;
    float acc[NC > 0 ? NC : 1];
#pragma unroll
    for (int q = 0; q < (NC > 0 ? NC : 1); ++q) acc[q] = 0.f;
    // one 16-byte chunk of the row: scale, store, and add its share of the fused projections
    auto chunk = [&](int c, const uint4& xv) __attribute__((always_inline)) {
        float x[8], g[8];
        unpack8(xv, x);
        unpack8(gain[c], g);
        uint4 o;
        o.x = pack_bf16x2(x[0] * r * g[0], x[1] * r * g[1]);
        o.y = pack_bf16x2(x[2] * r * g[2], x[3] * r * g[3]);
        o.z = pack_bf16x2(x[4] * r * g[4], x[5] * r * g[5]);
        o.w = pack_bf16x2(x[6] * r * g[6], x[7] * r * g[7]);
        yr[c] = o;
        if constexpr (NC > 0) {
            float y[8];
            unpack8(o, y);
#pragma unroll
            for (int q = 0; q < NC; ++q) {
                float b[8];
                unpack8(((const uint4*)(np.B[q] + member * (int64_t)chunks * 8))[c], b);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[q] = fmaf(y[e], b[e], acc[q]);
            }
        }
    };
    if constexpr (CPL > 0) {
#pragma unroll
        for (int i = 0; i < CPL; ++i)
            if (lane + 64 * i < chunks) chunk(lane + 64 * i, keep[i]);
    } else {
        for (int c = lane; c < chunks; c += 64) chunk(c, xr[c]);   // (not unrolled: the trip count is a run-time value)
    }
    if constexpr (NC > 0) {
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            float v = acc[q];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0) np.t[q][row] = v;
        }
    }
}

// ---- causal softmax attention ------------------------------------------------------------------------
// One workgroup (8 waves) per (member, head): K [S][HD] and V transposed [HD][S] of the head sit in LDS, wave w
// owns 32 query rows and walks the key blocks 0 .. its own (the causal triangle).  The two waves of a SIMD get
// query blocks b and 7 - b, so every SIMD does the same number of key blocks.
//   scores^T = K Q^T      as MFMA C[m = key][n = query]: a lane holds 16 scores of ONE query, so the row
//                         maximum and sum are in-lane reductions plus one exchange between the lane halves;
//   O^T     += V^T P^T    as MFMA C[m = hd][n = query]: the P operand is the lane's own 16 probabilities
//                         (bf16), the V^T operand reads the keys in the same order from LDS.
// Online softmax in base 2 (running maximum and sum per query, fp32).  S <= 256.
template <int HD>
struct AttnCfg {
    static constexpr int SMAX = 256;
    static constexpr int KP = HD * 2 + 16;    // K row pitch in bytes (68 dwords at HD = 128: 16 lanes cover all banks)
    static constexpr int VP = SMAX * 2 + 8;   // V^T row pitch in bytes (130 dwords: 32 lanes x 8 bytes cover all banks)
    static constexpr int LDS = SMAX * KP + HD * VP;
};

template <int HD>
__global__ __launch_bounds__(512) void attention_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                                                        const uint16_t* __restrict__ V, uint16_t* __restrict__ O, int S,
                                                        int heads, int64_t ld, float scale_log2,
                                                        const uint16_t* __restrict__ Bo, float* __restrict__ part, int64_t rows_total)
{
    // Bo != NULL: the rows written here feed a perturbed layer (the o-projection) whose rank-1 factors are Bo[member][heads * HD];
    // the head's share of that layer's projections, sum over its HD columns of O[row][col] * Bo[col] (from the bf16 values stored),
    // goes to part[head][row] and a small pass adds the heads in order -- so the attention output is not read a second time.
    typedef AttnCfg<HD> C;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sK = smem;
    char* sV = smem + C::SMAX * C::KP;
    char* sB = smem + C::LDS;  // HD bf16 of Bo for this (member, head)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t member = blockIdx.x / heads;
    const int head = (int)(blockIdx.x - member * heads);
    const int64_t base = member * S * ld + (int64_t)head * HD;
    const uint16_t *Qg = Q + base, *Kg = K + base, *Vg = V + base;
    const int SP = (S + 31) & ~31;
    constexpr int CPR = HD / 8;  // 16-byte chunks per row

    // The wave's query rows first (they are needed last): 32 rows, the lane's half of every 16 columns.
    const int nqb = SP / 32;
    const int qb = wave < 4 ? wave : 11 - wave;
    const int n = lane & 31, h = lane >> 5;
    const int qrow = qb * 32 + n;
    u32x4 qf[HD / 16];
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) {
        qf[ks] = u32x4{0u, 0u, 0u, 0u};
        if (qb < nqb && qrow < S) qf[ks] = *(const u32x4*)(Qg + (int64_t)qrow * ld + (2 * ks + h) * 8);
    }
    if (Bo && tid < CPR) *(uint4*)(sB + tid * 16) = *(const uint4*)(Bo + (member * heads + head) * (int64_t)HD + tid * 8);
    // K and V of the head pass through registers on their way to LDS.  Every load of a thread is issued before the first
    // LDS write (fixed trip counts for S = SMAX, predicated), so the workgroup pays the memory latency once, not per 16 bytes.
    constexpr int KIT = C::SMAX * CPR / 512, VIT = (C::SMAX / 64) * CPR / 8;
    static_assert(C::SMAX * CPR % 512 == 0 && (C::SMAX / 64) * CPR % 8 == 0, "whole passes of the workgroup");
    uint4 kreg[KIT], vreg[VIT];
#pragma unroll
    for (int i = 0; i < KIT; ++i) {
        const int idx = i * 512 + tid;
        const int row = idx / CPR, ch = idx - row * CPR;
        kreg[i] = make_uint4(0, 0, 0, 0);
        if (row < S) kreg[i] = *(const uint4*)(Kg + (int64_t)row * ld + ch * 8);
    }
    // V: a wave's 64 lanes take 64 consecutive keys of one 8-column chunk, so each 2-byte transposed store
    // instruction writes 128 contiguous bytes of one V^T row
#pragma unroll
    for (int i = 0; i < VIT; ++i) {
        const int it = i * 8 + wave;
        const int kg = it / CPR, ch = it - kg * CPR;
        const int key = kg * 64 + lane;
        vreg[i] = make_uint4(0, 0, 0, 0);
        if (key < S) vreg[i] = *(const uint4*)(Vg + (int64_t)key * ld + ch * 8);
    }
#pragma unroll
    for (int i = 0; i < KIT; ++i) {
        const int idx = i * 512 + tid;
        const int row = idx / CPR, ch = idx - row * CPR;
        if (row < SP) *(uint4*)(sK + row * C::KP + ch * 16) = kreg[i];
    }
#pragma unroll
    for (int i = 0; i < VIT; ++i) {
        const int it = i * 8 + wave;
        const int kg = it / CPR, ch = it - kg * CPR;
        const int key = kg * 64 + lane;
        if (key < SP) {
            const uint32_t w[4] = {vreg[i].x, vreg[i].y, vreg[i].z, vreg[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                *(uint16_t*)(sV + (ch * 8 + 2 * e) * C::VP + key * 2) = (uint16_t)(w[e] & 0xFFFFu);
                *(uint16_t*)(sV + (ch * 8 + 2 * e + 1) * C::VP + key * 2) = (uint16_t)(w[e] >> 16);
            }
        }
    }
    __syncthreads();
    if (qb >= nqb) return;  // no barrier follows
    f32x16 oacc[HD / 32];
#pragma unroll
    for (int mb = 0; mb < HD / 32; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[mb][e] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;

    for (int kb = 0; kb <= qb; ++kb) {
        f32x16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = 0.f;
        const char* kp = sK + (kb * 32 + n) * C::KP + h * 16;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) {
            const u32x4 a = *(const u32x4*)(kp + ks * 32);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, qf[ks]), s, 0, 0, 0);
        }
        float p[16];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = kb * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            p[i] = (kb == qb && key > qrow) ? -INFINITY : s[i] * scale_log2;
            mx = fmaxf(mx, p[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mnew = fmaxf(mrun, mx);  // finite: key 0 of the member is visible to every query
        const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            p[i] = __builtin_amdgcn_exp2f(p[i] - mnew);
            lsum += p[i];
        }
        lrun = lrun * alpha + lsum;
        mrun = mnew;
#pragma unroll
        for (int mb = 0; mb < HD / 32; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[mb][e] *= alpha;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4 pb = {pack_bf16x2(p[8 * t], p[8 * t + 1]), pack_bf16x2(p[8 * t + 2], p[8 * t + 3]),
                              pack_bf16x2(p[8 * t + 4], p[8 * t + 5]), pack_bf16x2(p[8 * t + 6], p[8 * t + 7])};
#pragma unroll
            for (int mb = 0; mb < HD / 32; ++mb) {
                // K-slots j < 4: keys kb*32 + 16t + 4h + j;  j >= 4: the same + 8 -- the order of the lane's p values
                const char* vp = sV + (mb * 32 + n) * C::VP + (kb * 32 + 16 * t + 4 * h) * 2;
                const uint2 lo = *(const uint2*)vp, hi = *(const uint2*)(vp + 16);
                const u32x4 a = {lo.x, lo.y, hi.x, hi.y};
                oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, pb), oacc[mb], 0, 0, 0);
            }
        }
    }
    const float inv = 1.0f / (lrun + __shfl_xor(lrun, 32, 64));
    uint16_t* orow = O + base + (int64_t)qrow * ld;
    float tp = 0.f;
#pragma unroll
    for (int mb = 0; mb < HD / 32; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint2 o = make_uint2(pack_bf16x2(oacc[mb][4 * q] * inv, oacc[mb][4 * q + 1] * inv),
                                       pack_bf16x2(oacc[mb][4 * q + 2] * inv, oacc[mb][4 * q + 3] * inv));
            if (qrow < S) *(uint2*)(orow + mb * 32 + 8 * q + 4 * h) = o;
            if (Bo) {
                const uint2 bv = *(const uint2*)(sB + (mb * 32 + 8 * q + 4 * h) * 2);
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                tp = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, o.x), __builtin_bit_cast(bf16x2_t, bv.x), tp, false);
                tp = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, o.y), __builtin_bit_cast(bf16x2_t, bv.y), tp, false);
            }
        }
    if (Bo) {
        tp += __shfl_xor(tp, 32, 64);  // the two lane halves hold the two halves of every 8 columns
        if (h == 0 && qrow < S) part[(int64_t)head * rows_total + member * S + qrow] = tp;
    }
}

// ---- next-token log-likelihood: out[row] = logits[row][token[row+1]] - log sum_j exp(logits[row][j]) -----
// One workgroup per row; online maximum / sum in base 2 per thread, combined through LDS.  The member's last
// token has no successor: 0.  HBM-bound: 2 V bytes per row.
__global__ __launch_bounds__(256) void token_loglik_kernel(const uint4* __restrict__ logits, const int32_t* __restrict__ tokens,
                                                           float* __restrict__ out, int S, int vocab)
{
    __shared__ float red_m[4], red_l[4];
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    if ((int)(row % S) == S - 1) {
        if (tid == 0) out[row] = 0.f;
        return;
    }
    const int chunks = vocab >> 3;
    const uint4* lr = logits + row * chunks;
    constexpr float LOG2E = 1.4426950408889634f;
    float m = -INFINITY, l = 0.f;
    for (int c = tid; c < chunks; c += 256) {
        float x[8];
        unpack8(lr[c], x);
        float mx = x[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, x[e]);
        const float mnew = fmaxf(m, mx * LOG2E);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += exp2f(x[e] * LOG2E - mnew);
        l = l * exp2f(m - mnew) + s;
        m = mnew;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float om = __shfl_xor(m, off, 64), ol = __shfl_xor(l, off, 64);
        const float mn = fmaxf(m, om);
        l = (m == -INFINITY ? 0.f : l * exp2f(m - mn)) + (om == -INFINITY ? 0.f : ol * exp2f(om - mn));
        m = mn;
    }
    if ((tid & 63) == 0) {
        red_m[tid >> 6] = m;
        red_l[tid >> 6] = l;
    }
    __syncthreads();
    if (tid == 0) {
        float mm = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
        float ll = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            if (red_m[w] != -INFINITY) ll += red_l[w] * exp2f(red_m[w] - mm);
        const int tgt = min(max(tokens[row + 1], 0), vocab - 1);
        const float xt = bf16_bits_to_f32(((const uint16_t*)lr)[tgt]);
        out[row] = xt - (mm + log2f(ll)) * 0.6931471805599453f;
    }
}

// ---- launchers -------------------------------------------------------------------------------------------
egg_status launch_embed_rows(eggroll_ctx* c, int64_t rows, int d, int vocab, const void* emb, const int32_t* tokens, void* X)
{
    if (rows == 0) return EGG_OK;
    KernelScope ks(c, "embed_rows");
    hipLaunchKernelGGL(embed_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->stream, tokens, (const uint4*)emb,
                       (uint4*)X, rows, d / 8, vocab);
    return check_hip(c, hipGetLastError(), "embed_rows launch");
}

// rows of up to 2048 / 4096 values are held in registers (4 / 8 chunks per lane), longer ones take the two-pass form
template <int NC>
static void launch_rmsnorm_nc(eggroll_ctx* c, int64_t rows, int d, float eps, const void* gain, const void* X, void* Y, const NormProj& np)
{
    const dim3 g((unsigned)((rows + 3) / 4)), b(256);
    const int chunks = d / 8;
#define EGG_NORM(CPL) \
    hipLaunchKernelGGL((rmsnorm_kernel<NC, CPL>), g, b, 0, c->stream, (const uint4*)X, (const uint4*)gain, (uint4*)Y, rows, chunks, 1.0f / (float)d, eps, np)
    if (chunks <= 256) EGG_NORM(4);
    else if (chunks <= 512) EGG_NORM(8);
    else EGG_NORM(0);
#undef EGG_NORM
}

egg_status launch_rmsnorm(eggroll_ctx* c, int64_t rows, int d, float eps, const void* gain, const void* X, void* Y)
{
    if (rows == 0) return EGG_OK;
    KernelScope ks(c, "rmsnorm");
    launch_rmsnorm_nc<0>(c, rows, d, eps, gain, X, Y, NormProj{});
    return check_hip(c, hipGetLastError(), "rmsnorm launch");
}

// the normalisation with the projections of nc (1 or 3) consuming layers fused in; B[q]: [members][d] bf16, t[q]: [rows]
egg_status launch_rmsnorm_proj(eggroll_ctx* c, int64_t rows, int S, int d, float eps, const void* gain, const void* X, void* Y, int nc,
                               const void* const* B, float* const* t)
{
    if (rows == 0) return EGG_OK;
    NormProj np{};
    for (int q = 0; q < nc; ++q) {
        np.B[q] = (const uint16_t*)B[q];
        np.t[q] = t[q];
    }
    np.S = S;
    KernelScope ks(c, "rmsnorm_project");
    if (nc == 1)
        launch_rmsnorm_nc<1>(c, rows, d, eps, gain, X, Y, np);
    else if (nc == 3)
        launch_rmsnorm_nc<3>(c, rows, d, eps, gain, X, Y, np);
    else
        return fail(c, EGG_EINVAL, "rmsnorm_proj: %d consumers", nc);
    return check_hip(c, hipGetLastError(), "rmsnorm_project launch");
}

template <int HD>
static egg_status launch_attention_t(eggroll_ctx* c, int64_t members, int S, int heads, const void* Q, const void* K,
                                     const void* V, void* O, const void* Bo, float* part)
{
    auto kern = attention_kernel<HD>;
    constexpr size_t LDS = (size_t)AttnCfg<HD>::LDS + HD * 2;
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, LDS, "attention smem attr");
    if (st != EGG_OK) return st;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
    KernelScope ks(c, "attention");
    hipLaunchKernelGGL(kern, dim3((unsigned)(members * heads)), dim3(512), LDS, c->stream, (const uint16_t*)Q,
                       (const uint16_t*)K, (const uint16_t*)V, (uint16_t*)O, S, heads, (int64_t)heads * HD, scale_log2,
                       (const uint16_t*)Bo, part, members * S);
    return check_hip(c, hipGetLastError(), "attention launch");
}

egg_status launch_attention(eggroll_ctx* c, int64_t members, int S, int heads, int head_dim, const void* Q, const void* K,
                            const void* V, void* O, const void* Bo, float* t_next)
{
    if (members == 0) return EGG_OK;
    float* part = nullptr;
    if (Bo) {
        egg_status st = reserve(c, c->proj_part, (size_t)heads * members * S * sizeof(float));
        if (st != EGG_OK) return st;
        part = (float*)c->proj_part.p;
    }
    egg_status st = EGG_EUNSUPPORTED;
    if (S < 1 || S > 256) return fail(c, EGG_EUNSUPPORTED, "attention: rows_per_member %d outside [1, 256]", S);
    if (members * heads > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "attention: too many (member, head) pairs in one call");
    switch (head_dim) {
        case 32: st = launch_attention_t<32>(c, members, S, heads, Q, K, V, O, Bo, part); break;
        case 64: st = launch_attention_t<64>(c, members, S, heads, Q, K, V, O, Bo, part); break;
        case 128: st = launch_attention_t<128>(c, members, S, heads, Q, K, V, O, Bo, part); break;
        default: return fail(c, EGG_EUNSUPPORTED, "attention: head dimension %d not in {32, 64, 128}", head_dim);
    }
    if (st != EGG_OK || !Bo) return st;
    return launch_sum_slabs(c, part, heads, members * S, t_next);
}

egg_status launch_token_loglik(eggroll_ctx* c, int64_t members, int S, int vocab, const void* logits, const int32_t* tokens, float* out)
{
    const int64_t rows = members * S;
    if (rows == 0) return EGG_OK;
    if (rows > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "token_loglik: too many rows in one call");
    KernelScope ks(c, "token_loglik");
    hipLaunchKernelGGL(token_loglik_kernel, dim3((unsigned)rows), dim3(256), 0, c->stream, (const uint4*)logits, tokens, out, S, vocab);
    return check_hip(c, hipGetLastError(), "token_loglik launch");
}

}  // namespace egg

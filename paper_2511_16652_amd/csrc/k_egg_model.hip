// The integer model around the GRU cell (App. "EGG architecture": Embedding, Layer Normalisation, MLP,
// Alg. "EGG forward pass"), for a population of members with one token each per time step, bit-exact:
//     y = EMBED(emb, t)
//     per layer:  y', s' = GRU(LN(ln1, y), s);  y = I8(y' + y);   y' = (LN(ln2, y) @ mlp1^T) @ mlp2^T;  y = I8(y' + y)
//     logits = LN(ln_out, y) @ head^T
// "@" is the perturbed scaled int8 matmul (MFMA kernels of the integer path); the row-wise pieces here
// are bandwidth work: a lane owns 16 consecutive bytes of a row, D/16 adjacent lanes own the row.
//   * the residual add is fused with the layer normalisation that follows it (one read of y and of the
//     block's output, one write each of y and of the normalised row);
//   * DIVIDE(x, mav): |x| <= 127^2 < 2^14 and mav < 2^7, so floor(|x| / mav) = (|x| * ceil(2^21 / mav)) >> 21
//     exactly (the multiplier's excess (mav - 1) * |x| stays below 2^21); one integer division per lane
//     for the multiplier, a multiply-high per element -- no table.
#include "common.hpp"
#include <math.h>

namespace egg {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int sat127(int v) { return min(127, max(-127, v)); }
__device__ __forceinline__ int sbyte(uint32_t w, int b) { return (int)(int8_t)(w >> (8 * b)); }

// y[row] = I8(y[row] + add[row]) when add != nullptr (written back), then u[row] = LN(ln, y[row]).
// By-products (LnExtras): dot products of the normalised row with the row of up to two factor arrays (the
// u . B of the matmuls that read u; the odd member of an antithetic pair uses -B), and two int32 vectors
// cleared for epilogues that accumulate into them later.
__global__ __launch_bounds__(256) void resid_ln_kernel(const int8_t* __restrict__ add, int8_t* __restrict__ y,
                                                       const int8_t* __restrict__ ln, int8_t* __restrict__ u,
                                                       int64_t rows, int lpr_log2, int d_log2, LnExtras ex)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = gid >> lpr_log2;
    const int part = (int)(gid & ((1 << lpr_log2) - 1));
    const bool live = row < rows;   // dead lanes run the shuffles with zeros
    const size_t off = ((size_t)row << d_log2) + (size_t)part * 16;
    u32x4 yv = {0, 0, 0, 0};
    if (live) {
        yv = *(const u32x4*)(y + off);
        if (add) {
            const u32x4 av = *(const u32x4*)(add + off);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t yw = yv[w], aw = av[w];
                uint32_t o = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) o |= (uint32_t)(sat127(sbyte(yw, b) + sbyte(aw, b)) & 0xFF) << (8 * b);
                yv[w] = o;
            }
            *(u32x4*)(y + off) = yv;
        }
    }
    int sum = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t yw = yv[w];
#pragma unroll
        for (int b = 0; b < 4; ++b) sum += abs(sbyte(yw, b));
    }
    for (int o = 1; o < (1 << lpr_log2); o <<= 1) sum += __shfl_xor(sum, o, 64);
    if (!live) return;
    const uint32_t mav = (uint32_t)max(sum >> d_log2, 1);
    const uint32_t magic = ((1u << 21) + mav - 1u) / mav;
    const u32x4 lv = *(const u32x4*)(ln + (size_t)part * 16);
    u32x4 ov;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t yw = yv[w], lw = lv[w];
        uint32_t o = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int prod = sbyte(yw, b) * sbyte(lw, b);
            const int q = (int)__umulhi((uint32_t)abs(prod) << 11, magic);
            o |= (uint32_t)((prod < 0 ? -min(q, 127) : min(q, 127)) & 0xFF) << (8 * b);
        }
        ov[w] = o;
    }
    *(u32x4*)(u + off) = ov;
    if (ex.dot[0]) {
        const size_t foff = ((size_t)(ex.anti ? row >> 1 : row) << d_log2) + (size_t)part * 16;
        const u32x4 b0 = *(const u32x4*)(ex.B[0] + foff);
        int d0 = 0, d1 = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) d0 = __builtin_amdgcn_sdot4((int)ov[w], (int)b0[w], d0, false);
        if (ex.dot[1]) {
            const u32x4 b1 = *(const u32x4*)(ex.B[1] + foff);
#pragma unroll
            for (int w = 0; w < 4; ++w) d1 = __builtin_amdgcn_sdot4((int)ov[w], (int)b1[w], d1, false);
        }
        // every lane of a live row is live (rows are whole groups of lanes), so the shuffles stay inside the row
        for (int o = 1; o < (1 << lpr_log2); o <<= 1) {
            d0 += __shfl_xor(d0, o, 64);
            d1 += __shfl_xor(d1, o, 64);
        }
        if (part == 0) {
            const bool neg = ex.anti && (row & 1);
            ex.dot[0][row] = neg ? -d0 : d0;
            if (ex.dot[1]) ex.dot[1][row] = neg ? -d1 : d1;
        }
    }
    if (part == 0) {
        if (ex.zero[0]) ex.zero[0][row] = 0;
        if (ex.zero[1]) ex.zero[1][row] = 0;
    }
}

// y[row] = I8(emb[t] + ((A[id][t] * +-B[id]) >> corr_shift)), t = tokens[row]; the odd member of an
// antithetic pair carries the negated B.
__global__ __launch_bounds__(256) void embed_i8_kernel(const int8_t* __restrict__ emb, const uint8_t* __restrict__ tokens,
                                                       const int8_t* __restrict__ A, const int8_t* __restrict__ B,
                                                       int8_t* __restrict__ y, int64_t rows, int lpr_log2, int d_log2,
                                                       int anti, int corr_shift)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = gid >> lpr_log2;
    if (row >= rows) return;
    const int part = (int)(gid & ((1 << lpr_log2) - 1));
    const int64_t id = anti ? (row >> 1) : row;
    const int t = tokens[row];
    int a = A[(size_t)id * 256 + t];
    if (anti && (row & 1)) a = -a;
    const u32x4 bv = *(const u32x4*)(B + ((size_t)id << d_log2) + (size_t)part * 16);
    const u32x4 ev = *(const u32x4*)(emb + ((size_t)t << d_log2) + (size_t)part * 16);
    u32x4 ov;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t bw = bv[w], ew = ev[w];
        uint32_t o = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) o |= (uint32_t)(sat127(sbyte(ew, b) + ((a * sbyte(bw, b)) >> corr_shift)) & 0xFF) << (8 * b);
        ov[w] = o;
    }
    *(u32x4*)(y + ((size_t)row << d_log2) + (size_t)part * 16) = ov;
}

// Log-likelihood of the target token in 1/16 bit (App. "Fitness Calculation in Integer Types").  EXP2 is a
// 256-entry table; LOG2 is not stored (the paper's table would have 2^28 entries) but inverted exactly:
// round(16 log2 s) is the largest k whose threshold ceil(2^((k - 1/2) / 16)) is at most s, found by bisection
// over 512 thresholds in LDS.  16 lanes share a row of 256 logits.
__global__ __launch_bounds__(256) void loglik_i8_kernel(const int8_t* __restrict__ logits, const uint8_t* __restrict__ targets,
                                                        const int* __restrict__ lut, int64_t rows, int accumulate,
                                                        int* __restrict__ out)
{
    __shared__ int s_exp[256];
    __shared__ int s_thr[512];
    const int tid = threadIdx.x;
    s_exp[tid] = lut[tid];
    s_thr[tid] = lut[256 + tid];
    s_thr[256 + tid] = lut[512 + tid];
    __syncthreads();
    const int64_t gid = (int64_t)blockIdx.x * 256 + tid;
    const int64_t row = gid >> 4;
    const int part = (int)(gid & 15);
    int sum = 0;
    if (row < rows) {
        const u32x4 yv = *(const u32x4*)(logits + row * 256 + part * 16);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t yw = yv[w];
#pragma unroll
            for (int b = 0; b < 4; ++b) sum += s_exp[sbyte(yw, b) + 128];
        }
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o, 64);
    if (row >= rows || part != 0) return;
    int lo = 0, hi = 511;   // invariant: s_thr[lo] <= sum; the answer is the largest such index
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_thr[mid] <= sum) lo = mid;
        else hi = mid - 1;
    }
    const int o = ((int)logits[row * 256 + targets[row]] + 128) - (lo - 64);
    out[row] = accumulate ? out[row] + o : o;
}

egg_status launch_loglik_i8(eggroll_ctx* c, int64_t rows, const int8_t* logits, const uint8_t* targets, int accumulate, int32_t* out)
{
    if (!c->lut.p) {
        // tables in double on the host, once per context: EXP2[i] = round(16 * 2^(i/16)); threshold k is the
        // smallest integer s with 16 log2 s >= k - 1/2 (never an exact tie: 2^((2k-1)/32) is irrational)
        std::vector<int> h(256 + 512);
        for (int i = 0; i < 256; ++i) h[i] = (int)nearbyint(16.0 * exp2(i / 16.0));
        for (int k = 0; k < 512; ++k) {
            const double v = ceil(exp2((k - 0.5) / 16.0));
            h[256 + k] = v < 2147483647.0 ? (int)v : 2147483647;
        }
        egg_status st = reserve(c, c->lut, h.size() * sizeof(int));
        if (st != EGG_OK) return st;
        if ((st = check_hip(c, hipMemcpy(c->lut.p, h.data(), h.size() * sizeof(int), hipMemcpyHostToDevice), "log-likelihood tables")) != EGG_OK) return st;
    }
    if (rows == 0) return EGG_OK;
    KernelScope ks(c, "loglik_i8");
    const int64_t threads = rows * 16;
    hipLaunchKernelGGL(loglik_i8_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream, logits, targets,
                       (const int*)c->lut.p, rows, accumulate, out);
    return check_hip(c, hipGetLastError(), "loglik_i8 launch");
}

static int ilog2(int v)
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

egg_status launch_layernorm_i8(eggroll_ctx* c, const int8_t* add, int8_t* y, const int8_t* ln, int8_t* u, int64_t rows, int D,
                               const LnExtras* extras)
{
    if (rows == 0) return EGG_OK;
    KernelScope ks(c, "resid_layernorm_i8");
    const int lpr = ilog2(D / 16);
    const int64_t threads = rows << lpr;
    hipLaunchKernelGGL(resid_ln_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream, add, y, ln, u, rows, lpr, ilog2(D),
                       extras ? *extras : LnExtras());
    return check_hip(c, hipGetLastError(), "resid_layernorm_i8 launch");
}

static egg_status launch_embed(eggroll_ctx* c, const int8_t* emb, const uint8_t* tokens, const int8_t* A, const int8_t* B,
                               int8_t* y, int64_t rows, int D, int anti, int corr_shift)
{
    if (rows == 0) return EGG_OK;
    KernelScope ks(c, "embed_i8");
    const int lpr = ilog2(D / 16);
    const int64_t threads = rows << lpr;
    hipLaunchKernelGGL(embed_i8_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream, emb, tokens, A, B, y, rows, lpr,
                       ilog2(D), anti, corr_shift);
    return check_hip(c, hipGetLastError(), "embed_i8 launch");
}

egg_status launch_embed_i8(eggroll_ctx* c, egg_key key, const egg_shape& s, int int_bound, int corr_shift, const int8_t* emb,
                           const uint8_t* tokens, int8_t* Y)
{
    const int D = s.d_in;
    const int64_t rows = s.member_count;
    const int anti = s.antithetic ? 1 : 0;
    const int64_t ids = anti ? rows / 2 : rows;
    const uint32_t first_id = (uint32_t)(anti ? s.member_begin / 2 : s.member_begin);
    egg_status st;
    if ((st = reserve(c, c->i8_a, (size_t)ids * 256)) != EGG_OK) return st;
    if ((st = reserve(c, c->i8_b, (size_t)ids * D)) != EGG_OK) return st;
    int8_t *A = (int8_t*)c->i8_a.p, *B = (int8_t*)c->i8_b.p;
    if ((st = launch_noise(c, make_stream_key(key.seed, key.step, key.layer, 0), first_id, ids, 256, EGG_I8, EGG_UNIFORM_INT, int_bound, A)) != EGG_OK) return st;
    if ((st = launch_noise(c, make_stream_key(key.seed, key.step, key.layer, 1), first_id, ids, D, EGG_I8, EGG_UNIFORM_INT, int_bound, B)) != EGG_OK) return st;
    return launch_embed(c, emb, tokens, A, B, Y, rows, D, anti, corr_shift);
}

// Scratch of one forward call: the rank-1 factors of all 6 L + 2 perturbed parameters (generated once per
// call: a member's perturbation is fixed while it is evaluated, Alg. 1), the activations of one time
// step, and a second copy of the recurrent state to ping-pong with S_out.
egg_status launch_egg_forward_i8(eggroll_ctx* c, egg_key key, const egg_shape& s, int L, int int_bound, int corr_shift, int T,
                                 const egg_model_i8& P, const uint8_t* tokens, const int8_t* S_in, int8_t* S_out,
                                 int8_t* logits)
{
    const int D = s.d_in;
    const int64_t rows = s.member_count;
    const int anti = s.antithetic ? 1 : 0;
    const int64_t ids = anti ? rows / 2 : rows;
    const uint32_t first_id = (uint32_t)(anti ? s.member_begin / 2 : s.member_begin);
    const int os_d = 4 + ilog2(D) / 2, os_4d = os_d + 1;   // 16 sqrt(n) as a shift, n = D and 4 D
    auto pad = [](size_t b) { return (b + 255) & ~size_t(255); };
    const size_t fD = pad((size_t)ids * D), f4D = pad((size_t)ids * 4 * D), f256 = pad((size_t)ids * 256);
    const size_t act = pad((size_t)rows * D), dots = pad((size_t)rows * sizeof(int));
    const size_t per_layer = 8 * fD + 2 * (f4D + fD);
    const size_t n_dots = 4 + 2 * (size_t)L;   // u.B_Wf, u.B_Wh, f^.B_Uh, one for the MLP and the head; s.B_Uf twice per layer
    const size_t total = 2 * (f256 + fD) + (size_t)L * per_layer   // factors
                         + 7 * act + 4 * act                        // y, u, y', a1, a3, f, f^; MLP hidden
                         + n_dots * dots + (T > 1 ? (size_t)L * act : 0);
    egg_status st;
    if ((st = reserve(c, c->gru, total)) != EGG_OK) return st;
    char* p = (char*)c->gru.p;
    auto take = [&](size_t b) { char* q = p; p += b; return (int8_t*)q; };
    auto gen = [&](uint32_t layer, int which, int n, int8_t* out) {
        return launch_noise(c, make_stream_key(key.seed, key.step, layer, which), first_id, ids, n, EGG_I8, EGG_UNIFORM_INT, int_bound, out);
    };
    int8_t* embA = take(f256); int8_t* embB = take(fD);
    int8_t* headA = take(f256); int8_t* headB = take(fD);
    const uint32_t head_layer = key.layer + 1u + 6u * (uint32_t)L;
    if ((st = gen(key.layer, 0, 256, embA)) != EGG_OK || (st = gen(key.layer, 1, D, embB)) != EGG_OK) return st;
    if ((st = gen(head_layer, 0, 256, headA)) != EGG_OK || (st = gen(head_layer, 1, D, headB)) != EGG_OK) return st;
    struct LayerFactors { int8_t *A[4], *B[4], *A1, *B1, *A2, *B2; };
    std::vector<LayerFactors> F((size_t)L);
    for (int i = 0; i < L; ++i) {
        const uint32_t base = key.layer + 1u + 6u * (uint32_t)i;
        for (int m = 0; m < 4; ++m) {
            F[i].A[m] = take(fD); F[i].B[m] = take(fD);
            if ((st = gen(base + m, 0, D, F[i].A[m])) != EGG_OK || (st = gen(base + m, 1, D, F[i].B[m])) != EGG_OK) return st;
        }
        F[i].A1 = take(f4D); F[i].B1 = take(fD); F[i].A2 = take(fD); F[i].B2 = take(f4D);
        if ((st = gen(base + 4, 0, 4 * D, F[i].A1)) != EGG_OK || (st = gen(base + 4, 1, D, F[i].B1)) != EGG_OK) return st;
        if ((st = gen(base + 5, 0, D, F[i].A2)) != EGG_OK || (st = gen(base + 5, 1, 4 * D, F[i].B2)) != EGG_OK) return st;
    }
    int8_t *y = take(act), *u = take(act), *yp = take(act), *a1 = take(act), *a3 = take(act), *f = take(act), *fh = take(act);
    int8_t* hid = take(4 * act);
    int* dot[4];
    for (int m = 0; m < 4; ++m) dot[m] = (int*)take(dots);
    std::vector<int*> dot_s(2 * (size_t)L);   // [layer][parity of the time step that reads it]
    for (auto& d : dot_s) d = (int*)take(dots);
    int8_t* S_alt = T > 1 ? take((size_t)L * act) : nullptr;
    const size_t DD = (size_t)D * D, state_stride = (size_t)rows * D;

    // Every dot product u . B that a matmul needs is a by-product of whatever wrote u: the normalisation
    // pass (u . B_Wf, u . B_Wh, u . B_mlp1, u . B_head), the first gate's epilogue (f^ . B_Uh), the last GRU
    // epilogue (h . B_Uf for the next time step) and the first MLP matmul's epilogue (hidden . B_mlp2).
    // Only s . B_Uf of the state the caller passes in is computed by a pass of its own, at the first time step.
    for (int t = 0; t < T; ++t) {
        // the last time step writes S_out; the ones before it alternate so that no step reads what it writes
        const int8_t* s_from = t == 0 ? S_in : (((T - t) & 1) ? S_alt : S_out);
        int8_t* s_to = ((T - 1 - t) & 1) ? S_alt : S_out;
        const size_t from_stride = t == 0 ? state_stride : (s_from == S_alt ? act : state_stride);
        const size_t to_stride = s_to == S_alt ? act : state_stride;
        if ((st = launch_embed(c, P.emb, tokens + (size_t)t * rows, embA, embB, y, rows, D, anti, corr_shift)) != EGG_OK) return st;
        const int8_t* add = nullptr;
        for (int i = 0; i < L; ++i) {
            int* ds_now = dot_s[2 * (size_t)i + (t & 1)];
            int* ds_next = t + 1 < T ? dot_s[2 * (size_t)i + ((t + 1) & 1)] : nullptr;
            LnExtras e1;
            e1.anti = anti;
            e1.B[0] = F[i].B[0]; e1.dot[0] = dot[0];   // u . B_Wf
            e1.B[1] = F[i].B[2]; e1.dot[1] = dot[2];   // u . B_Wh
            e1.zero[0] = dot[3]; e1.zero[1] = ds_next;
            if ((st = launch_layernorm_i8(c, add, y, P.ln1 + (size_t)i * D, u, rows, D, &e1)) != EGG_OK) return st;
            GruStep g;
            for (int m = 0; m < 4; ++m) { g.A[m] = F[i].A[m]; g.B[m] = F[i].B[m]; g.W[m] = P.gru_w + ((size_t)i * 4 + m) * DD; g.dot[m] = dot[m]; }
            g.dot[1] = ds_now;
            g.bf = P.gru_b + (size_t)i * 2 * D; g.bh = g.bf + D;
            g.a1 = a1; g.a3 = a3; g.f = f; g.fh = fh;
            g.u_dots_ready = true; g.s_dot_ready = t > 0; g.fh_dot_zeroed = true; g.dot_s_next = ds_next;
            int8_t* h = s_to + (size_t)i * to_stride;
            if ((st = launch_gru_step(c, g, anti, rows, D, int_bound, corr_shift, os_d, u, s_from + (size_t)i * from_stride, h)) != EGG_OK) return st;
            LnExtras e2;
            e2.anti = anti;
            e2.B[0] = F[i].B1; e2.dot[0] = dot[0];     // u . B_mlp1
            e2.zero[0] = dot[1];                        // hidden . B_mlp2, accumulated by the first MLP matmul
            if ((st = launch_layernorm_i8(c, h, y, P.ln2 + (size_t)i * D, u, rows, D, &e2)) != EGG_OK) return st;
            if ((st = launch_i8_matmul(c, F[i].A1, F[i].B1, anti, rows, 4 * D, D, int_bound, corr_shift, os_d, P.mlp1 + (size_t)i * 4 * DD, u, hid, dot[0], true, nullptr, F[i].B2, dot[1])) != EGG_OK) return st;
            if ((st = launch_i8_matmul(c, F[i].A2, F[i].B2, anti, rows, D, 4 * D, int_bound, corr_shift, os_4d, P.mlp2 + (size_t)i * 4 * DD, hid, yp, dot[1], true, nullptr)) != EGG_OK) return st;
            add = yp;
        }
        LnExtras eo;
        eo.anti = anti;
        eo.B[0] = headB; eo.dot[0] = dot[0];
        if ((st = launch_layernorm_i8(c, add, y, P.ln_out, u, rows, D, &eo)) != EGG_OK) return st;
        if ((st = launch_i8_matmul(c, headA, headB, anti, rows, 256, D, int_bound, corr_shift, os_d, P.head, u, logits + (size_t)t * rows * 256, dot[0], true, nullptr)) != EGG_OK) return st;
    }
    return EGG_OK;
}

}  // namespace egg

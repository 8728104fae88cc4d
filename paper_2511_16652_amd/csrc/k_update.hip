// EGGROLL update direction (EGGROLL UPDATE box; Sec. 4.2):
//   G = scale * sum_i f_i A_i B_i^T = scale * (diag(f~) A~)^T B~,  A~ in R^{K x d_out}, B~ in R^{K x d_in},
//   K = N*r, row kappa = i*r + l holds A_i[:, l] (resp. B_i[:, l]), f~ repeats f r times.
// Two steps: (1) a pack pass turns the [member][d][r] factors (the forward's caches, or freshly
// regenerated ones) into K-packed panels -- 16-byte chunks of consecutive kappa for one column --
// with the fitness folded into the A panel; (2) the MFMA NT core contracts the panels over K.
// bf16 factors are packed as fp16 (11 significant bits instead of 8 for f_i*a): a bf16 value of magnitude
// >= 2^-14 is exact in fp16; below that it lands on fp16's subnormal grid (absolute error <= 2^-25) and below
// 2^-25 it becomes zero -- about 5e-5 of N(0,1) draws, each contributing an absolute error <= 2^-25 to a product
// of typical size 1.  The A panel holds (f_i / fnorm) a with |f_i / fnorm| <= 1, so members whose |f_i| is far
// below max|f| lose relative precision the same way: the error per term is bounded by 2^-25 max|f|, i.e. it is
// relative to the largest fitness, not to f_i.  fp32 factors stay fp32.  No atomics: each G entry has one owner
// and a fixed summation order, so the result is run-to-run identical.
#include "common.hpp"
#include "gemm_core.hpp"

namespace egg {

// fnorm[0] = 2^ceil(log2(max|f|)) (1 if all zero), fnorm[1] = 1/fnorm[0].  Folding f/fnorm[0] into the
// fp16 panel and fnorm[0] into the epilogue scale is exact (a power of two) and keeps f_i*a inside
// the fp16 range whatever the magnitude of the fitness values.
__global__ __launch_bounds__(1024) void fitness_norm_kernel(const float* __restrict__ f, int64_t n, float* __restrict__ fnorm)
{
    __shared__ float red[16];
    float m = 0.f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, fabsf(f[i]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float mx = red[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) mx = fmaxf(mx, red[w]);
        float p = 1.f;
        if (mx > 0.f && mx < 3.0e38f) {
            int e;
            (void)frexpf(mx, &e);  // mx = frac * 2^e, frac in [0.5, 1)
            p = ldexpf(1.f, e);
        }
        fnorm[0] = p;
        fnorm[1] = 1.f / p;
    }
}

// out chunk (kg, col) at (kg*d + col)*16 bytes holds kappa = kg*EPC .. +EPC-1 of column `col`.
template <bool BF16>
__global__ __launch_bounds__(256) void pack_kernel(const void* __restrict__ src, const float* __restrict__ fitness,
                                                   const float* __restrict__ fnorm, int64_t members, int d, int rank, int64_t kgroups,
                                                   void* __restrict__ out)
{
    constexpr int EPC = BF16 ? 8 : 4;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= kgroups * d) return;
    const int64_t kg = gid / d;
    const int col = (int)(gid - kg * d);
    const int64_t K = members * rank;
    const float finv = fitness ? fnorm[1] : 1.f;
    float v[EPC];
    if constexpr (BF16) {
        // rank 2, 4 or 8: the 8 values are 8 / rank members x rank contiguous bf16; one load per member, issued
        // unconditionally from clamped addresses (members past the end count with factor 0)
        if (rank == 2 || rank == 4 || rank == 8) {
            uint32_t w[4];
            float fs[4];
            bool in[4];  // the member of word h exists
            if (rank == 8) {
                const int64_t i = kg, ic = min(i, members - 1);
                const u32x4 t = *(const u32x4*)((const uint16_t*)src + (ic * d + col) * 8);
                w[0] = t[0]; w[1] = t[1]; w[2] = t[2]; w[3] = t[3];
                fs[0] = fs[1] = fs[2] = fs[3] = fitness ? fitness[ic] * finv : 1.f;
                in[0] = in[1] = in[2] = in[3] = i < members;
            } else if (rank == 4) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int64_t i = kg * 2 + h, ic = min(i, members - 1);
                    const uint2 t = *(const uint2*)((const uint16_t*)src + (ic * d + col) * 4);
                    w[2 * h] = t.x; w[2 * h + 1] = t.y;
                    fs[2 * h] = fs[2 * h + 1] = fitness ? fitness[ic] * finv : 1.f;
                    in[2 * h] = in[2 * h + 1] = i < members;
                }
            } else {
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const int64_t i = kg * 4 + h, ic = min(i, members - 1);
                    w[h] = *(const uint32_t*)((const uint16_t*)src + (ic * d + col) * 2);
                    fs[h] = fitness ? fitness[ic] * finv : 1.f;
                    in[h] = i < members;
                }
            }
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            u32x4 o;
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                h2 p;
                p[0] = (_Float16)(in[h] ? bf16_lo(w[h]) * fs[h] : 0.f);  // round to nearest even; past the last member: +0
                p[1] = (_Float16)(in[h] ? bf16_hi(w[h]) * fs[h] : 0.f);
                o[h] = __builtin_bit_cast(uint32_t, p);
            }
            ((u32x4*)out)[gid] = o;
            return;
        }
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
        const int64_t kappa = kg * EPC + e;
        float x = 0.f;
        if (kappa < K) {
            const int64_t i = kappa / rank;
            const int l = (int)(kappa - i * rank);
            const int64_t off = (i * d + col) * rank + l;
            if constexpr (BF16) x = __uint_as_float((uint32_t)((const uint16_t*)src)[off] << 16);
            else x = ((const float*)src)[off];
            if (fitness) x *= fitness[i] * finv;
        }
        v[e] = x;
    }
    if constexpr (BF16) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h2 p;
            p[0] = (_Float16)v[2 * e];  // round to nearest even
            p[1] = (_Float16)v[2 * e + 1];
            o[e] = __builtin_bit_cast(uint32_t, p);
        }
        ((u32x4*)out)[gid] = o;
    } else {
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = __float_as_uint(v[e]);
        ((u32x4*)out)[gid] = o;
    }
}

// Rank-1 fast path of the pack pass: a thread turns an EPC x EPC block (EPC members x EPC columns,
// one 16-byte load per member) into EPC output chunks that are contiguous in the panel, so both the
// reads and the writes of a wave are fully coalesced.  Needs d % EPC == 0.
template <bool BF16>
__global__ __launch_bounds__(256) void pack_r1_kernel(const void* __restrict__ src, const float* __restrict__ fitness,
                                                      const float* __restrict__ fnorm, int64_t members, int d,
                                                      int64_t kgroups, void* __restrict__ out)
{
    constexpr int EPC = BF16 ? 8 : 4;
    const int cgroups = d / EPC;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= kgroups * cgroups) return;
    const int64_t kg = gid / cgroups;
    const int col0 = (int)(gid - kg * cgroups) * EPC;
    const float finv = fitness ? fnorm[1] : 1.f;
    float x[EPC][EPC];  // [member][column]
    // every load of the thread goes out before the first use (unconditional, from clamped member numbers; members past
    // the end count with factor 0, written as +0)
    u32x4 raw[EPC];
    float fsv[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
        const int64_t ic = min(kg * EPC + e, members - 1);
        raw[e] = *(const u32x4*)((const char*)src + (ic * d + col0) * (BF16 ? 2 : 4));
        fsv[e] = fitness ? fitness[ic] * finv : 1.f;
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
        const bool in = kg * EPC + e < members;
        const u32x4 v = in ? raw[e] : u32x4{0u, 0u, 0u, 0u};
        const float fs = in ? fsv[e] : 0.f;
        if constexpr (BF16) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                x[e][2 * w] = bf16_lo(v[w]) * fs;
                x[e][2 * w + 1] = bf16_hi(v[w]) * fs;
            }
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) x[e][w] = __uint_as_float(v[w]) * fs;
        }
    }
    u32x4* o = (u32x4*)out + kg * d + col0;
#pragma unroll
    for (int cc = 0; cc < EPC; ++cc) {
        u32x4 r;
        if constexpr (BF16) {
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                h2 p;
                p[0] = (_Float16)x[2 * w][cc];  // round to nearest even
                p[1] = (_Float16)x[2 * w + 1][cc];
                r[w] = __builtin_bit_cast(uint32_t, p);
            }
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) r[w] = __float_as_uint(x[w][cc]);
        }
        o[cc] = r;
    }
}

// Rank-1 bf16 factors without caches: regenerate straight into the K-packed fp16 panel.  A thread owns
// one column pair (2jp, 2jp+1) of 8 consecutive members -- eight Threefry blocks, the same (member,
// block) addressing every other kernel uses -- and writes the two finished 16-byte chunks, which are
// neighbours in the panel: no [member][d] intermediate is written or re-read.
__global__ __launch_bounds__(256) void gen_pack_r1_kernel(StreamKey key, uint32_t member_begin, const float* __restrict__ fitness,
                                                          const float* __restrict__ fnorm, int64_t members, int d,
                                                          int64_t kgroups, u32x4* __restrict__ out)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const int pairs = d >> 1;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= kgroups * pairs) return;
    const int64_t kg = gid / pairs;
    const int jp = (int)(gid - kg * pairs);
    const float finv = fitness ? fnorm[1] : 1.f;
    float lo[8], hi[8];  // columns 2jp and 2jp+1 of the 8 members
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int64_t i = kg * 8 + e;
        lo[e] = hi[e] = 0.f;
        if (i < members) {
            uint32_t w0, w1;
            noise_words(key, member_begin + (uint32_t)i, (uint32_t)jp, w0, w1);
            float z0, z1;
            normal_pair<false>(w0, w1, z0, z1);
            const uint32_t pk = pack_bf16x2(z0, z1);  // the factors are bf16 values
            const float fs = fitness ? fitness[i] * finv : 1.f;
            lo[e] = bf16_lo(pk) * fs;
            hi[e] = bf16_hi(pk) * fs;
        }
    }
    u32x4 c0, c1;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        h2 p, q;
        p[0] = (_Float16)lo[2 * w]; p[1] = (_Float16)lo[2 * w + 1];  // round to nearest even
        q[0] = (_Float16)hi[2 * w]; q[1] = (_Float16)hi[2 * w + 1];
        c0[w] = __builtin_bit_cast(uint32_t, p);
        c1[w] = __builtin_bit_cast(uint32_t, q);
    }
    u32x4* o = out + kg * d + 2 * jp;
    o[0] = c0;
    o[1] = c1;
}

struct UpdArgs {
    float* G;
    void* W;
    const float* fnorm;
    int d_out, d_in;
    float scale, lr;
    int accumulate, w_bf16;
};

// MBLK: row blocks (of 32) per wave tile.  G is row-major [d_out][d_in] and a column n is one k: the 32 lanes of a
// half-wave already write 32 consecutive floats of one G row, so no staging is needed.
template <int MBLK>
struct UpdEpiT {
    typedef float value_t;
    typedef UpdArgs Args;
    const Args a;
    float scale;
    // W += lr G: the lane's MBLK x 16 elements of W in the current column block, read in one batch when the block begins
    // (unconditional loads from clamped addresses; one load and one full wait per element otherwise)
    float wv[MBLK * 16];
    int row0 = 0;  // the lane's first row of the wave tile
    static constexpr __host__ __device__ int lds_per_wave(int) { return 0; }
    __device__ __forceinline__ UpdEpiT(const Args& a_, char*, int) : a(a_) { scale = a.scale * a.fnorm[0]; }
    __device__ __forceinline__ void column(int, bool) {}
    template <int J>
    __device__ __forceinline__ void column_at(int n, bool)
    {
        if (!a.W) return;
        const int64_t nc = min(n, a.d_in - 1);
        if (a.w_bf16) {
            const uint16_t* w = (const uint16_t*)a.W + nc;
#pragma unroll
            for (int k = 0; k < MBLK * 16; ++k) wv[k] = bf16_bits_to_f32(w[(int64_t)min(row0 + (k >> 4) * 32 + ((k >> 2) & 3) * 8 + (k & 3), a.d_out - 1) * a.d_in]);
        } else {
            const float* w = (const float*)a.W + nc;
#pragma unroll
            for (int k = 0; k < MBLK * 16; ++k) wv[k] = w[(int64_t)min(row0 + (k >> 4) * 32 + ((k >> 2) & 3) * 8 + (k & 3), a.d_out - 1) * a.d_in];
        }
    }
    template <int WTM>
    __device__ __forceinline__ void flush(int, int, int) {}
    template <int NT, int BM, int BN>
    __device__ __forceinline__ bool tile_begin(char*, int, int, int, int) { return false; }
    template <class MT, int MB, int NB>
    __device__ __forceinline__ void extra_mma(typename MT::acc_t (&)[MB][NB], int, int, int, int) {}
    template <int MB, int NB>
    __device__ __forceinline__ void prefetch(int mw0, int, int lane, int)
    {
        static_assert(MB == MBLK, "row blocks per wave tile");
        row0 = mw0 + (lane >> 5) * 4;
    }
    // rows m .. m + 3 (row block I, group Q of the block) of column n
    template <int I, int Q>
    __device__ __forceinline__ void store4_blk(int m, int n, const float (&v)[4], bool valid, int)
    {
        if (!valid || m >= a.d_out) return;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t idx = (int64_t)(m + e) * a.d_in + n;
            float g = scale * v[e];
            if (a.accumulate) g += a.G[idx];
            a.G[idx] = g;
            if (a.W) {
                const float w_new = fmaf(a.lr, g, wv[(I * 4 + Q) * 4 + e]);
                if (a.w_bf16) ((uint16_t*)a.W)[idx] = f32_to_bf16_bits(w_new);
                else ((float*)a.W)[idx] = w_new;
            }
        }
    }
};

template <class MT, int BM, int BN, int WM, int WN>
static egg_status launch_upd_gemm(eggroll_ctx* c, const char* name, const Operand& P, const Operand& Q, int kchunks,
                                  const UpdArgs& ea)
{
    const int tiles_m = (P.rows + BM - 1) / BM, tiles_n = (Q.rows + BN - 1) / BN;
    const size_t lds = gemm_lds_bytes<BM, BN>();
    if (!operand_offsets_fit(P, BM) || !operand_offsets_fit(Q, BN)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    static_assert(MT::BLK == 32, "the epilogue indexes 32-row blocks");
    auto kern = gemm_nt_kernel<MT, BM, BN, WM, WN, true, UpdEpiT<BM / WM / 32>>;
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, (size_t)lds, "gemm smem attr");
    if (st != EGG_OK) return st;
    KernelScope ks(c, name);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(WM * WN * 64), lds, c->stream, P, Q, kchunks,
                       tiles_m, tiles_n, 0, (const char*)c->zero_page.p, ea);
    return check_hip(c, hipGetLastError(), name);
}

egg_status launch_update(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                         egg_dtype noise_dtype, const float* fitness, float scale, int accumulate, float* G, void* W,
                         egg_dtype w_dtype, float lr, const void* A_cache, const void* B_cache, bool b_panel)
{
    const bool bf = noise_dtype == EGG_BF16;
    const int esz = bf ? 2 : 4, epc = bf ? 8 : 4;
    const int64_t K = s.member_count * (int64_t)s.rank;
    const int64_t kgroups = (K + epc - 1) / epc;
    if (kgroups > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "population * rank too large");
    egg_status st;

    // factors in [member][d][r] layout: the caller's caches, or regenerated into scratch
    // (rank-1 bf16 without caches regenerates straight into the packed panels instead)
    const bool gen_packed = !A_cache && bf && s.rank == 1 && s.d_out % 2 == 0 && s.d_in % 2 == 0;
    const void* A_src = A_cache;
    const void* B_src = B_cache;
    if (!A_src && !gen_packed) {
        const size_t na = (size_t)s.member_count * s.d_out * s.rank * esz, nb = (size_t)s.member_count * s.d_in * s.rank * esz;
        if ((st = reserve(c, c->a_buf, na)) != EGG_OK) return st;
        if ((st = reserve(c, c->b_buf, nb)) != EGG_OK) return st;
        if ((st = launch_noise(c, ka, (uint32_t)s.member_begin, s.member_count, (int64_t)s.d_out * s.rank, noise_dtype, EGG_NORMAL, 0, c->a_buf.p)) != EGG_OK) return st;
        if ((st = launch_noise(c, kb, (uint32_t)s.member_begin, s.member_count, (int64_t)s.d_in * s.rank, noise_dtype, EGG_NORMAL, 0, c->b_buf.p)) != EGG_OK) return st;
        A_src = c->a_buf.p;
        B_src = c->b_buf.p;
    }

    if ((st = reserve(c, c->fnorm, 256)) != EGG_OK) return st;
    float* fnorm = (float*)c->fnorm.p;
    {
        KernelScope ks(c, "fitness_norm");
        hipLaunchKernelGGL(fitness_norm_kernel, dim3(1), dim3(1024), 0, c->stream, fitness, s.member_count, fnorm);
    }
    if ((st = reserve(c, c->pack_a, (size_t)kgroups * s.d_out * 16)) != EGG_OK) return st;
    // b_panel: the caller's B_cache already is the packed panel (written by the forward pass); only A is generated
    if (!b_panel && (st = reserve(c, c->pack_b, (size_t)kgroups * s.d_in * 16)) != EGG_OK) return st;
    {
        const int64_t ta = kgroups * s.d_out, tb = kgroups * s.d_in;
        if ((ta + 255) / 256 > 0x7FFFFFFF || (tb + 255) / 256 > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "pack grid too large");
        KernelScope ks(c, "update_pack");
        auto pack = [&](const void* src, const float* fit, int d, void* dst) {
            if (s.rank == 1 && d % epc == 0) {
                const int64_t n = kgroups * (d / epc);
                const dim3 g((unsigned)((n + 255) / 256)), b(256);
                if (bf) hipLaunchKernelGGL(pack_r1_kernel<true>, g, b, 0, c->stream, src, fit, fnorm, s.member_count, d, kgroups, dst);
                else hipLaunchKernelGGL(pack_r1_kernel<false>, g, b, 0, c->stream, src, fit, fnorm, s.member_count, d, kgroups, dst);
            } else {
                const int64_t n = kgroups * d;
                const dim3 g((unsigned)((n + 255) / 256)), b(256);
                if (bf) hipLaunchKernelGGL(pack_kernel<true>, g, b, 0, c->stream, src, fit, fnorm, s.member_count, d, s.rank, kgroups, dst);
                else hipLaunchKernelGGL(pack_kernel<false>, g, b, 0, c->stream, src, fit, fnorm, s.member_count, d, s.rank, kgroups, dst);
            }
        };
        auto gen_pack = [&](const StreamKey& k, const float* fit, int d, void* dst) {
            const int64_t n = kgroups * (d / 2);
            hipLaunchKernelGGL(gen_pack_r1_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, k,
                               (uint32_t)s.member_begin, fit, fnorm, s.member_count, d, kgroups, (u32x4*)dst);
        };
        if (gen_packed) {
            gen_pack(ka, fitness, s.d_out, c->pack_a.p);
            if (!b_panel) gen_pack(kb, nullptr, s.d_in, c->pack_b.p);
        } else {
            pack(A_src, fitness, s.d_out, c->pack_a.p);
            pack(B_src, nullptr, s.d_in, c->pack_b.p);
        }
        if ((st = check_hip(c, hipGetLastError(), "pack launch")) != EGG_OK) return st;
    }

    Operand P{(const char*)c->pack_a.p, 16, (int64_t)s.d_out * 16, s.d_out};
    Operand Q{(const char*)(b_panel ? B_cache : c->pack_b.p), 16, (int64_t)s.d_in * 16, s.d_in};
    UpdArgs ea{G, W, fnorm, s.d_out, s.d_in, scale, lr, accumulate, w_dtype == EGG_BF16 ? 1 : 0};
    if (bf) {
        const int64_t big_tiles = ((s.d_out + 255) / 256) * (int64_t)((s.d_in + 255) / 256);
        if (big_tiles >= 192) return launch_upd_gemm<MmaF16, 256, 256, 2, 4>(c, "update_gemm_f16", P, Q, (int)kgroups, ea);
        return launch_upd_gemm<MmaF16, 128, 128, 2, 2>(c, "update_gemm_f16_small", P, Q, (int)kgroups, ea);
    }
    return launch_upd_gemm<MmaF32, 128, 128, 2, 2>(c, "update_gemm_f32", P, Q, (int)kgroups, ea);
}

}  // namespace egg

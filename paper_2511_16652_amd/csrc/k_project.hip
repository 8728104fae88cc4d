// Projection pre-pass of the population forward:  t[q][l] = sum_k X[q][k] * B_i[k][l]
// (Sec. 4.2: for r = 1 "a batch of N vector-vector dot products of length d_in"; the B x r
// intermediate of the arithmetic-intensity appendix).  One workgroup per member: B_i is regenerated
// once into LDS (and optionally kept in the caller's cache), then the member's S rows are streamed
// against it, one wave per row.  HBM-bound on X for large S, integer-ALU bound (noise) for S = 1.
// With antithetic pairs a workgroup owns a pair: the factors are generated once for its 2S rows.
#include "common.hpp"

namespace egg {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// d_in is walked in panels of `panel` columns (a multiple of the 16-byte chunk, all of d_in when B_i fits the LDS budget):
// per panel B_i[k0 .. k0 + panel) is regenerated into LDS and the member's rows are streamed against it; with more than
// one panel the partial sums are carried in t itself (a row is always handled by the same wave).
template <bool BF16, int RANK>
__global__ __launch_bounds__(256) void project_kernel(StreamKey kb, uint32_t member_begin, int S, int anti_rows, int d_in, int panel,
                                                      const void* __restrict__ X, float* __restrict__ t,
                                                      void* __restrict__ B_cache)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x;
    const int64_t ml = blockIdx.x;  // local member
    const uint32_t member = member_begin + (uint32_t)ml;
    constexpr int EPC = BF16 ? 8 : 4;  // elements per 16-byte chunk of X
    // bf16 with more than one rank term: the panel sits in LDS rank-major ([l][column]), so that a 16-byte read holds the
    // same 8 columns as the chunk of the row and each pair of columns is one packed dot product (v_dot2c_f32_bf16)
    // instead of two unpacked multiply-adds: the pass was vector-ALU bound on unpacking (2.5 TB/s at rank 4).
    constexpr bool TRANSPOSED = BF16 && RANK >= 2;
    const int lane = tid & 63, wave = tid >> 6;

    for (int k0 = 0; k0 < d_in; k0 += panel) {
        const int kn = min(panel, d_in - k0);     // columns of this panel
        const int n = kn * RANK;                  // even: d_in and panel are multiples of 4
        const int first = k0 * RANK;              // flat index of the panel's first factor entry (even)
        if (k0) __syncthreads();                  // every wave is done with the previous panel
        // ---- phase 1: B_i panel -> LDS (storage dtype), optional cache ---------------------------
        for (int b = tid; b < (n >> 1); b += 256) {
            const int gb = (first >> 1) + b;      // Threefry block of the member's vector
            uint32_t w0, w1;
            noise_words(kb, member, (uint32_t)gb, w0, w1);
            float z0, z1;
            normal_pair<!BF16>(w0, w1, z0, z1);
            if constexpr (BF16) {
                const uint32_t pk = pack_bf16x2(z0, z1);
                if constexpr (TRANSPOSED) {
                    // flat entries 2b, 2b+1 = (column 2b / RANK, rank terms l, l+1): rank-major in LDS, columns contiguous
                    const int col = (2 * b) / RANK, l = (2 * b) % RANK;
                    ((uint16_t*)smem)[l * kn + col] = (uint16_t)(pk & 0xFFFFu);
                    ((uint16_t*)smem)[(l + 1) * kn + col] = (uint16_t)(pk >> 16);
                } else {
                    ((uint32_t*)smem)[b] = pk;
                }
                if (B_cache) ((uint32_t*)B_cache)[ml * (int64_t)((d_in * RANK) >> 1) + gb] = pk;
            } else {
                ((float2*)smem)[b] = make_float2(z0, z1);
                if (B_cache) ((float2*)B_cache)[ml * (int64_t)((d_in * RANK) >> 1) + gb] = make_float2(z0, z1);
            }
        }
        __syncthreads();

        // ---- phase 2: one wave per row ------------------------------------------------------------
        const int chunks = kn / EPC;
        for (int s = wave; s < S; s += 4) {
            const int64_t row = ml * S + s;
            const uint4* xr = (const uint4*)((const char*)X + (row * (int64_t)d_in + k0) * (BF16 ? 2 : 4));
            float acc[RANK];
#pragma unroll
            for (int l = 0; l < RANK; ++l) acc[l] = 0.f;
            // (four iterations at a time, so that a lane has four 16-byte loads of the row in flight: with one, the pass
            // ran at 2.5 TB/s on rows of 8192 values; the order of the additions is unchanged)
#pragma unroll 4
            for (int ch = lane; ch < chunks; ch += 64) {
                const uint4 xv = xr[ch];
                if constexpr (TRANSPOSED) {
                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                    const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                    for (int l = 0; l < RANK; ++l) {
                        const uint4 q = *(const uint4*)((const uint16_t*)smem + (int64_t)l * kn + (int64_t)ch * 8);
                        const uint32_t bw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc[l] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xw[e]), __builtin_bit_cast(bf16x2, bw[e]), acc[l], false);
                    }
                    continue;
                }
                float x[EPC];
                if constexpr (BF16) {
                    const uint32_t w[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        x[2 * e] = __uint_as_float(w[e] << 16);
                        x[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
                    }
                } else {
                    x[0] = __uint_as_float(xv.x); x[1] = __uint_as_float(xv.y);
                    x[2] = __uint_as_float(xv.z); x[3] = __uint_as_float(xv.w);
                }
                // B_i[k][l] for the chunk's k range: EPC*RANK consecutive elements = RANK 16-byte reads
                const uint4* bp = (const uint4*)smem + (int64_t)ch * RANK;
#pragma unroll
                for (int v = 0; v < RANK; ++v) {
                    const uint4 q = bp[v];
                    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
                    // the 16 bytes hold flat entries v*EPC .. of the chunk: entry f belongs to column f / RANK, rank term f % RANK
                    if constexpr (BF16) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int f = v * 8 + e;
                            const float bv = (e & 1) ? __uint_as_float(w[e >> 1] & 0xFFFF0000u) : __uint_as_float(w[e >> 1] << 16);
                            acc[f % RANK] = fmaf(x[f / RANK], bv, acc[f % RANK]);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int f = v * 4 + e;
                            acc[f % RANK] = fmaf(x[f / RANK], __uint_as_float(w[e]), acc[f % RANK]);
                        }
                    }
                }
            }
#pragma unroll
            for (int l = 0; l < RANK; ++l) {
                float v = acc[l];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
                // antithetic pairs: the workgroup owns both members of a pair (2 x anti_rows rows); the second
                // member is evaluated at -sigma, which is folded into its projections
                if (lane == 0) {
                    const float sv = (anti_rows && s >= anti_rows) ? -v : v;
                    t[row * RANK + l] = k0 ? t[row * RANK + l] + sv : sv;
                }
            }
        }
    }
}

// One row per member and rank 1: nothing is shared between rows, so B_i never needs to sit in LDS.
// Each thread multiplies the factor pairs it generates with the matching x pair on the fly; one
// shuffle reduction per wave and a 4-entry LDS reduction finish the dot product.
template <bool BF16>
__global__ __launch_bounds__(256) void project_row_kernel(StreamKey kb, uint32_t member_begin, int d_in,
                                                          const void* __restrict__ X, float* __restrict__ t,
                                                          void* __restrict__ B_cache)
{
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const int64_t ml = blockIdx.x;
    const uint32_t member = member_begin + (uint32_t)ml;
    const int pairs = d_in >> 1;
    float acc = 0.f;
    for (int b = tid; b < pairs; b += 256) {
        uint32_t w0, w1;
        noise_words(kb, member, (uint32_t)b, w0, w1);
        float z0, z1;
        normal_pair<!BF16>(w0, w1, z0, z1);
        if constexpr (BF16) {
            const uint32_t pk = pack_bf16x2(z0, z1);
            const uint32_t xv = ((const uint32_t*)X)[ml * pairs + b];
            acc = fmaf(bf16_lo(xv), bf16_lo(pk), acc);
            acc = fmaf(bf16_hi(xv), bf16_hi(pk), acc);
            if (B_cache) ((uint32_t*)B_cache)[ml * pairs + b] = pk;
        } else {
            const float2 xv = ((const float2*)X)[ml * pairs + b];
            acc = fmaf(xv.x, z0, acc);
            acc = fmaf(xv.y, z1, acc);
            if (B_cache) ((float2*)B_cache)[ml * pairs + b] = make_float2(z0, z1);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) t[ml] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The same projection for 8 consecutive members per workgroup, with B leaving the kernel as the K-packed fp16
// panel the update contracts ([member / 8][k][member % 8]).  512 threads: thread (b, half) generates the column
// pair (2b, 2b+1) of members 4 half .. 4 half + 3 and stores its 8 bytes of the two 16-byte chunks, which are
// neighbours in the panel.  The first 256 threads (half 0) and the last 256 (half 1) each hold the 256 b-lanes
// in the order of project_row_kernel, and every member's partial sums go through the same shuffle tree and the
// same final additions, so t is bit-identical to that kernel's.
__global__ __launch_bounds__(512) void project_row8_kernel(StreamKey kb, uint32_t member_begin, int64_t members, int d_in,
                                                           const void* __restrict__ X, float* __restrict__ t,
                                                           u32x4* __restrict__ panel)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    __shared__ float red[4][8];
    const int tid = threadIdx.x;
    const int half = tid >> 8, bl = tid & 255;
    const int64_t g = blockIdx.x;
    const int pairs = d_in >> 1;
    float acc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = 0.f;
    for (int b = bl; b < pairs; b += 256) {
        float lo[4], hi[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t i = g * 8 + half * 4 + e;
            lo[e] = hi[e] = 0.f;
            if (i < members) {
                uint32_t w0, w1;
                noise_words(kb, member_begin + (uint32_t)i, (uint32_t)b, w0, w1);
                float z0, z1;
                normal_pair<false>(w0, w1, z0, z1);
                const uint32_t pk = pack_bf16x2(z0, z1);
                const uint32_t xv = ((const uint32_t*)X)[i * pairs + b];
                acc[e] = fmaf(bf16_lo(xv), bf16_lo(pk), acc[e]);
                acc[e] = fmaf(bf16_hi(xv), bf16_hi(pk), acc[e]);
                lo[e] = bf16_lo(pk);
                hi[e] = bf16_hi(pk);
            }
        }
        uint2 c0, c1;
        {
            h2 p, q;
            p[0] = (_Float16)lo[0]; p[1] = (_Float16)lo[1];
            q[0] = (_Float16)lo[2]; q[1] = (_Float16)lo[3];
            c0.x = __builtin_bit_cast(uint32_t, p); c0.y = __builtin_bit_cast(uint32_t, q);
            p[0] = (_Float16)hi[0]; p[1] = (_Float16)hi[1];
            q[0] = (_Float16)hi[2]; q[1] = (_Float16)hi[3];
            c1.x = __builtin_bit_cast(uint32_t, p); c1.y = __builtin_bit_cast(uint32_t, q);
        }
        uint2* o = (uint2*)(panel + g * d_in + 2 * b) + half;   // bytes 8 half .. 8 half + 7 of chunk 2b
        o[0] = c0;
        o[2] = c1;                                              // the same bytes of chunk 2b + 1
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) acc[e] += __shfl_xor(acc[e], off, 64);
    }
    if ((tid & 63) == 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) red[bl >> 6][half * 4 + e] = acc[e];
    }
    __syncthreads();
    if (tid < 8 && g * 8 + tid < members) t[g * 8 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
}

template <bool BF16>
static egg_status launch_project_t(eggroll_ctx* c, const StreamKey& kb, const egg_shape& shape, const void* X, float* t,
                                   void* B_cache, bool panel)
{
    if (panel && B_cache) {
        if (!BF16 || shape.rank != 1 || shape.rows_per_member != 1 || shape.antithetic)
            return fail(c, EGG_EUNSUPPORTED, "the panel cache layout needs bf16, rank 1, one row per member, no antithetic pairs");
        const int64_t groups = (shape.member_count + 7) / 8;
        if (groups > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "too many members in one call");
        KernelScope ks(c, "project");
        hipLaunchKernelGGL(project_row8_kernel, dim3((unsigned)groups), dim3(512), 0, c->stream, kb, (uint32_t)shape.member_begin,
                           shape.member_count, shape.d_in, X, t, (u32x4*)B_cache);
        return check_hip(c, hipGetLastError(), "project launch");
    }
    egg_shape s = shape;  // the noise view: pairs as members of 2S rows when antithetic
    const int anti_rows = shape.antithetic ? shape.rows_per_member : 0;
    if (shape.antithetic) {
        s.member_begin /= 2;
        s.member_count /= 2;
        s.rows_per_member *= 2;
    }
    // B_i panels of at most 128 KB in LDS: all of d_in when it fits, else the largest multiple of 64 columns
    const int esz = BF16 ? 2 : 4;
    int kpanel = s.d_in;
    if ((size_t)s.d_in * s.rank * esz > 128 * 1024) kpanel = (int)(128 * 1024 / ((size_t)s.rank * esz)) / 64 * 64;
    const size_t lds = (size_t)kpanel * s.rank * esz;
    const dim3 g((unsigned)s.member_count), b(256);
    if (s.member_count > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "too many members in one call");
    const uint32_t mb = (uint32_t)s.member_begin;
    if (s.rank == 1 && s.rows_per_member == 1) {
        KernelScope ks(c, "project");
        hipLaunchKernelGGL(project_row_kernel<BF16>, g, b, 0, c->stream, kb, mb, s.d_in, X, t, B_cache);
        return check_hip(c, hipGetLastError(), "project launch");
    }
#define EGG_LAUNCH_PROJECT(R)                                                                                        \
    {                                                                                                                \
        auto kern = project_kernel<BF16, R>;                                                                         \
        if (lds > 48 * 1024) {                                                                                       \
            egg_status st = ensure_dynamic_lds(c, (const void*)kern, (size_t)lds, "project smem attr"); \
            if (st != EGG_OK) return st;                                                                             \
        }                                                                                                            \
        KernelScope ks(c, "project");                                                                                \
        hipLaunchKernelGGL(kern, g, b, lds, c->stream, kb, mb, s.rows_per_member, anti_rows, s.d_in, kpanel, X, t, B_cache);            \
    }
    switch (s.rank) {
        case 1: EGG_LAUNCH_PROJECT(1) break;
        case 2: EGG_LAUNCH_PROJECT(2) break;
        case 4: EGG_LAUNCH_PROJECT(4) break;
        case 8: EGG_LAUNCH_PROJECT(8) break;
        default: EGG_LAUNCH_PROJECT(16) break;
    }
#undef EGG_LAUNCH_PROJECT
    return check_hip(c, hipGetLastError(), "project launch");
}

egg_status launch_project(eggroll_ctx* c, const StreamKey& kb, const egg_shape& s, egg_dtype io, const void* X,
                          float* t, void* B_cache, bool panel)
{
    return io == EGG_BF16 ? launch_project_t<true>(c, kb, s, X, t, B_cache, panel)
                          : launch_project_t<false>(c, kb, s, X, t, B_cache, panel);
}

}  // namespace egg

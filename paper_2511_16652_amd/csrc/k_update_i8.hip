// Integer parameter update of the int8 model (App. "Parameter Update" of the integer pretraining
// section), bit-exact:
//   E = (diag(F) A)^T B    int8 x int8 -> int32 over the population, F_i in {-1, 0, 1}
//   theta <- clamp(theta + sign(E) [|E| >= threshold], -127, 127)      one bin per step
// Three steps: the factors are regenerated into scratch ([member][d] int8); a pack pass turns them
// into K-packed panels (16 consecutive members of one column per 16-byte chunk) with F folded into
// the A panel (a sign flip or a zero: still int8); the int8 MFMA NT core contracts the panels over
// the members.  Small weight matrices give few tiles, so K is split over several groups of
// workgroups; each group stores its int32 partial E, and a last elementwise pass adds the partials
// (integer addition: the result does not depend on the order) and applies the threshold.  With
// one split the epilogue applies it directly.  (Combining the partial tiles with atomics was
// measured 20x slower than the contraction itself: 64 scattered 4-byte atomics per instruction.)
#include "common.hpp"
#include "gemm_core.hpp"
#include <algorithm>

namespace egg {

// A thread turns a 16 x 16 block (16 members x 16 columns, one 16-byte load per member) into 16
// output chunks that are contiguous in the panel.  Needs d % 16 == 0.  Members past the end and
// members of fitness 0 contribute zero bytes.
__global__ __launch_bounds__(256) void pack_i8_kernel(const int8_t* __restrict__ src, const int8_t* __restrict__ F,
                                                      int64_t members, int d, int64_t kgroups, u32x4* __restrict__ out)
{
    const int cgroups = d / 16;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= kgroups * cgroups) return;
    const int64_t kg = gid / cgroups;
    const int col0 = (int)(gid - kg * cgroups) * 16;
    u32x4 x[16];  // [member] -> 16 column bytes, already multiplied by the member's fitness
    // all 16 loads (and the 16 fitness bytes) go out before the first use: unconditional, from clamped member numbers --
    // a load under "if (i < members)" is a branch and gets a full wait of its own
    int fit[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int64_t i = kg * 16 + e, ic = min(i, members - 1);
        x[e] = *(const u32x4*)(src + ic * d + col0);
        fit[e] = F ? (int)F[ic] : 1;
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int64_t i = kg * 16 + e;
        const u32x4 v = x[e];
        const int f = i < members ? fit[e] : 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            // bytewise negation without a carry between bytes: -b = (b ^ 0xFF) + 1 (no byte is -128)
            const uint32_t n = v[w] ^ 0xFFFFFFFFu;
            const uint32_t neg = ((n & 0x7F7F7F7Fu) + 0x01010101u) ^ (n & 0x80808080u);
            x[e][w] = f > 0 ? v[w] : (f < 0 ? neg : 0u);
        }
    }
    u32x4* o = out + kg * d + col0;
#pragma unroll
    for (int cc = 0; cc < 16; ++cc) {
        u32x4 r;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) word |= ((x[4 * w + b][cc >> 2] >> (8 * (cc & 3))) & 0xFFu) << (8 * b);
            r[w] = word;
        }
        o[cc] = r;
    }
}

// one bin towards sign(e) where |e| reaches the threshold; four entries per word
__device__ __forceinline__ uint32_t move4(uint32_t theta4, const i32x4& e, int threshold)
{
    uint32_t out = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int v = e[b];
        const int mag = v < 0 ? -v : v;  // |E| < 2^31 is guaranteed by the host-side size check
        int t = (int)(int8_t)(theta4 >> (8 * b));
        if (v != 0 && mag >= threshold) t += v > 0 ? 1 : -1;
        t = min(127, max(-127, t));
        out |= ((uint32_t)t & 0xFFu) << (8 * b);
    }
    return out;
}

// elementwise pass after a split-K contraction: adds the partial E of every split, 16 entries per thread
__global__ __launch_bounds__(256) void apply_threshold_kernel(const i32x4* __restrict__ parts, int nsplit, int64_t split_stride,
                                                              i32x4* __restrict__ E_out, u32x4* __restrict__ theta, int64_t n16,
                                                              int threshold)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    i32x4 e[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) e[w] = parts[4 * i + w];
    for (int sp = 1; sp < nsplit; ++sp) {
#pragma unroll
        for (int w = 0; w < 4; ++w) e[w] += parts[sp * split_stride + 4 * i + w];
    }
    u32x4 t = theta[i];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (E_out) E_out[4 * i + w] = e[w];
        t[w] = move4(t[w], e[w], threshold);
    }
    theta[i] = t;
}

// Epilogue of the contraction.  Rows of the product are columns k of theta (P = B panel), its
// columns are rows j of theta (Q = F*A panel): a lane of the MFMA layout owns 4 consecutive k of
// one j.  The int32 accumulators of a 32-row block are parked in the wave's LDS slice and re-read
// row-wise, so that a lane finishes 16 consecutive entries of one theta row with 16-byte accesses.
struct I8UpdEpi {
    typedef int value_t;
    struct Args {
        int32_t* E;      // one split: optional output [d_out][d_in]; split-K: partial buffers [split][d_out][d_in]
        int8_t* theta;   // [d_out][d_in]
        int d_out, d_in, threshold;
        int split;       // != 0: only store this split's partial E
        int tiles;       // workgroups per split
    };
    const Args a;
    char* const stage;
    const int lane;
    int row_pitch;

    static constexpr __host__ __device__ int pitch(int wtm) { return wtm * 4 + 16; }
    static constexpr __host__ __device__ int lds_per_wave(int wtm) { return 32 * pitch(wtm); }
    __device__ __forceinline__ I8UpdEpi(const Args& a_, char* slice, int lane_) : a(a_), stage(slice), lane(lane_), row_pitch(0) {}
    template <int NT, int BM, int BN>
    __device__ __forceinline__ bool tile_begin(char*, int, int, int, int) { return false; }
    template <class MT, int MB, int NB>
    __device__ __forceinline__ void extra_mma(typename MT::acc_t (&)[MB][NB], int, int, int, int) {}
    template <int MB, int NB>
    __device__ __forceinline__ void prefetch(int, int, int, int) { row_pitch = pitch(MB * 32); }
    __device__ __forceinline__ void column(int, bool) {}
    __device__ __forceinline__ void store4(int, int, const int (&v)[4], bool, int ml)
    {
        *(i32x4*)(stage + (lane & 31) * row_pitch + ml * 4) = i32x4{v[0], v[1], v[2], v[3]};
    }
    template <int WTM>
    __device__ __forceinline__ void flush(int mw0, int nb0, int n_rows)
    {
        constexpr int P = pitch(WTM), CPR = WTM / 16, PASSES = WTM / 32;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes have landed
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < PASSES; ++it) {
            const int c = it * 64 + lane;
            const int row = c / CPR, mc = (c % CPR) * 16;
            const int j = nb0 + row, k = mw0 + mc;
            if (j < n_rows && k < a.d_in) {  // d_in is a multiple of 16
                const char* src = stage + row * P + mc * 4;
                const int64_t idx = (int64_t)j * a.d_in + k;
                i32x4 e[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) e[w] = *(const i32x4*)(src + w * 16);
                if (a.split) {
                    int32_t* part = a.E + (int64_t)(blockIdx.x / a.tiles) * a.d_out * a.d_in;
#pragma unroll
                    for (int w = 0; w < 4; ++w) *(i32x4*)(part + idx + 4 * w) = e[w];
                } else {
                    if (a.E) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) *(i32x4*)(a.E + idx + 4 * w) = e[w];
                    }
                    u32x4 t = *(const u32x4*)(a.theta + idx);
#pragma unroll
                    for (int w = 0; w < 4; ++w) t[w] = move4(t[w], e[w], a.threshold);
                    *(u32x4*)(a.theta + idx) = t;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();  // the slice is reused by the next row block
    }
};

template <int BM, int BN, int WM, int WN>
static egg_status launch_i8_upd_gemm(eggroll_ctx* c, const Operand& P, const Operand& Q, int kchunks, int per_split, int nsplit,
                                     I8UpdEpi::Args ea)
{
    const int tiles_m = (P.rows + BM - 1) / BM, tiles_n = (Q.rows + BN - 1) / BN;
    const size_t lds = std::max(gemm_lds_bytes<BM, BN>(), (size_t)WM * WN * I8UpdEpi::lds_per_wave(BM / WM));
    if (!operand_offsets_fit(P, BM) || !operand_offsets_fit(Q, BN)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    auto kern = gemm_nt_kernel<MmaI8, BM, BN, WM, WN, true, I8UpdEpi, (BM * BN <= 128 * 128 ? 2 : 1)>;
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, (size_t)lds, "gemm smem attr");
    if (st != EGG_OK) return st;
    ea.tiles = tiles_m * tiles_n;
    KernelScope ks(c, "update_gemm_i8");
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n * nsplit)), dim3(WM * WN * 64), lds, c->stream, P, Q,
                       kchunks, tiles_m, tiles_n, nsplit > 1 ? per_split : 0, (const char*)c->zero_page.p, ea);
    return check_hip(c, hipGetLastError(), "update_gemm_i8");
}

egg_status launch_update_i8(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                            int int_bound, const int8_t* F, int32_t threshold, int8_t* theta, int32_t* E_out)
{
    const int64_t N = s.member_count;
    const int64_t kgroups = (N + 15) / 16;
    if (kgroups > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "population too large");
    egg_status st;
    if ((st = reserve(c, c->i8_a, (size_t)N * s.d_out)) != EGG_OK) return st;
    if ((st = reserve(c, c->i8_b, (size_t)N * s.d_in)) != EGG_OK) return st;
    if ((st = reserve(c, c->pack_a, (size_t)kgroups * s.d_out * 16)) != EGG_OK) return st;
    if ((st = reserve(c, c->pack_b, (size_t)kgroups * s.d_in * 16)) != EGG_OK) return st;
    if ((st = launch_noise(c, ka, (uint32_t)s.member_begin, N, s.d_out, EGG_I8, EGG_UNIFORM_INT, int_bound, c->i8_a.p)) != EGG_OK) return st;
    if ((st = launch_noise(c, kb, (uint32_t)s.member_begin, N, s.d_in, EGG_I8, EGG_UNIFORM_INT, int_bound, c->i8_b.p)) != EGG_OK) return st;
    {
        KernelScope ks(c, "update_pack_i8");
        const int64_t na = kgroups * (s.d_out / 16), nb = kgroups * (s.d_in / 16);
        if ((na + 255) / 256 > 0x7FFFFFFF || (nb + 255) / 256 > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "pack grid too large");
        hipLaunchKernelGGL(pack_i8_kernel, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, c->stream, (const int8_t*)c->i8_a.p, F,
                           N, s.d_out, kgroups, (u32x4*)c->pack_a.p);
        hipLaunchKernelGGL(pack_i8_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, c->stream, (const int8_t*)c->i8_b.p,
                           (const int8_t*)nullptr, N, s.d_in, kgroups, (u32x4*)c->pack_b.p);
        if ((st = check_hip(c, hipGetLastError(), "pack_i8 launch")) != EGG_OK) return st;
    }

    // rows of the product = columns k of theta (B panel), columns = rows j of theta (F*A panel)
    Operand P{(const char*)c->pack_b.p, 16, (int64_t)s.d_in * 16, s.d_in};
    Operand Q{(const char*)c->pack_a.p, 16, (int64_t)s.d_out * 16, s.d_out};
    const int64_t big_tiles = ((s.d_out + 255) / 256) * (int64_t)((s.d_in + 255) / 256);
    const int64_t small_tiles = ((s.d_out + 127) / 128) * (int64_t)((s.d_in + 127) / 128);
    // enough workgroups for two per CU; a split owns whole 8-chunk K-stages (128 members)
    int per_split = 0, nsplit = 1;
    if (big_tiles < 192) {
        int64_t want = std::min<int64_t>((512 + small_tiles - 1) / small_tiles, (kgroups + 7) / 8);
        if (want > 1) {
            per_split = (int)((((kgroups + want - 1) / want) + 7) & ~int64_t(7));
            nsplit = (int)((kgroups + per_split - 1) / per_split);
        }
    }
    const int64_t n16 = (int64_t)s.d_out * s.d_in / 16;
    I8UpdEpi::Args ea{E_out, theta, s.d_out, s.d_in, threshold, 0, 0};
    if (nsplit > 1) {
        if ((st = reserve(c, c->t_buf, (size_t)nsplit * s.d_out * s.d_in * sizeof(int32_t))) != EGG_OK) return st;
        ea.E = (int32_t*)c->t_buf.p;
        ea.split = 1;
    }
    if (big_tiles >= 192) st = launch_i8_upd_gemm<256, 256, 2, 4>(c, P, Q, (int)kgroups, 0, 1, ea);
    else st = launch_i8_upd_gemm<128, 128, 2, 2>(c, P, Q, (int)kgroups, per_split, nsplit, ea);
    if (st != EGG_OK) return st;
    if (nsplit > 1) {
        KernelScope ks(c, "apply_threshold");
        hipLaunchKernelGGL(apply_threshold_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, c->stream,
                           (const i32x4*)c->t_buf.p, nsplit, n16 * 4, (i32x4*)E_out, (u32x4*)theta, n16, threshold);
        if ((st = check_hip(c, hipGetLastError(), "apply_threshold launch")) != EGG_OK) return st;
    }
    return EGG_OK;
}

}  // namespace egg

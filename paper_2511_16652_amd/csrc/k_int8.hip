// Integer perturbed matmul of the int8 recurrent model, bit-exact
// (App. "Matrix Multiplication": u @ M = I8(uM / (16 sqrt n)), a right shift for n = 4^d;
//  App. "Adding EGGROLL Perturbations": I8((u theta^T + ((u . B) I32(A) >> (4 + sigma_hat))) / (16 sqrt n))).
// Per step: one wave-per-row int8 dot kernel for u . B_i, then the int8 MFMA NT core for u theta^T
// whose epilogue adds the shifted rank-1 term, shifts, saturates to [-127, 127] and stores int8.
// The factors are fixed while a member is evaluated (Alg. 1), so they are generated once per call
// into scratch and re-read from L2/HBM at every step.
#include "common.hpp"
#include "gemm_core.hpp"

namespace egg {

// dots[row] = sum_k H[row][k] * B[row][k]   (int8 x int8 -> int32), one wave per row
__global__ __launch_bounds__(256) void dot_i8_kernel(const int8_t* __restrict__ H, const int8_t* __restrict__ B,
                                                     int64_t rows, int d, int* __restrict__ dots)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const u32x4* h = (const u32x4*)(H + row * d);
    const u32x4* b = (const u32x4*)(B + row * d);
    int acc = 0;
    for (int ch = lane; ch < (d >> 4); ch += 64) {
        const u32x4 hv = h[ch], bv = b[ch];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int x = (int)(int8_t)(hv[w] >> (8 * q));
                const int y = (int)(int8_t)(bv[w] >> (8 * q));
                acc += x * y;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) dots[row] = acc;
}

// Epilogue of the integer step.  A lane owns, per 32-column block, the outputs h'[n][m..m+3] of 4*MB
// groups; the matching bytes of A_i (for the correction) and of B_i (for the NEXT step's u . B) are
// fetched at kernel start, so that no global-memory latency sits behind the last MFMA.  The next
// step's dot product is accumulated here: per column the lane sums h'_j * B_i[j] over its rows, the
// two half-waves are combined, and one integer atomicAdd per (wave, column) lands in dots_next --
// integer addition is associative, so the result does not depend on the order of the atomics.
__global__ __launch_bounds__(256) void zero_i32_kernel(int* __restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

struct I8Epi {
    typedef int value_t;
    struct Args {
        const int8_t* A;  // [rows][d] factors
        const int8_t* B;  // [rows][d] factors
        const int* dots;  // [rows]  u . B of this step
        int* dots_next;   // [rows]  accumulates u' . B for the next step (zeroed by the host), or NULL
        int8_t* H_out;    // [rows][d]
        int d, corr_shift, out_shift;
    };
    const Args a;
    int dot[2];
    uint32_t pa[2][2][4], pb[2][2][4];  // prefetched bytes of A_i and B_i: [row block][column block][q]
    int part;                           // running partial of the next dot for the current column block
    int cur_j, cur_iq;
    bool have_pf;                       // small tiles prefetch; the 256x256 tile has no registers to spare

    static constexpr __host__ __device__ int lds_per_wave(int) { return 0; }
    __device__ __forceinline__ I8Epi(const Args& a_, char*, int) : a(a_), part(0), cur_j(-1), cur_iq(0), have_pf(false) {}
    template <int NT, int BM, int BN>
    __device__ __forceinline__ bool tile_begin(char*, int, int, int, int) { return false; }
    template <class MT, int MB, int NB>
    __device__ __forceinline__ void extra_mma(typename MT::acc_t (&)[MB][NB], int, int, int, int) {}

    template <int MB, int NB>
    __device__ __forceinline__ void prefetch(int mw0, int nw0, int lane, int n_rows)
    {
        static_assert(MB <= 4 && NB <= 2, "prefetch storage");
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int n = min(nw0 + j * 32 + (lane & 31), n_rows - 1);
            dot[j] = a.dots[n];
            if constexpr (MB > 2) continue;
            have_pf = true;
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int m = min(mw0 + i * 32 + q * 8 + (lane >> 5) * 4, a.d - 4);
                    const int64_t off = (int64_t)n * a.d + m;
                    pa[i][j][q] = *(const uint32_t*)(a.A + off);
                    pb[i][j][q] = a.dots_next ? *(const uint32_t*)(a.B + off) : 0u;
                }
        }
    }
    __device__ __forceinline__ void column(int, bool)
    {
        ++cur_j;
        cur_iq = 0;
        part = 0;
    }
    __device__ __forceinline__ void store4(int m, int n, const int (&v)[4], bool valid, int)
    {
        const int i = cur_iq >> 2, q = cur_iq & 3;
        ++cur_iq;
        if (!valid || m >= a.d) return;
        // cur_j, i, q are compile-time constants after unrolling; the selects below fold away
        uint32_t a4 = 0, b4 = 0;
        const int dj = cur_j == 0 ? dot[0] : dot[1];
        if (have_pf) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq)
                        if (jj == cur_j && ii == i && qq == q) {
                            a4 = pa[ii][jj][qq];
                            b4 = pb[ii][jj][qq];
                        }
        } else {
            const int64_t off = (int64_t)n * a.d + m;
            a4 = *(const uint32_t*)(a.A + off);
            b4 = a.dots_next ? *(const uint32_t*)(a.B + off) : 0u;
        }
        uint32_t out = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int ae = (int)(int8_t)(a4 >> (8 * e));
            const int corr = (dj * ae) >> a.corr_shift;  // arithmetic shift: floor
            int y = (v[e] + corr) >> a.out_shift;
            y = min(127, max(-127, y));
            out |= ((uint32_t)y & 0xFFu) << (8 * e);
            part += y * (int)(int8_t)(b4 >> (8 * e));
        }
        *(uint32_t*)(a.H_out + (int64_t)n * a.d + m) = out;
    }
    template <int WTM>
    __device__ __forceinline__ void flush(int, int nb0, int n_rows)
    {
        if (!a.dots_next) return;
        int p = part + __shfl_xor(part, 32, 64);  // the two half-waves hold different rows of the same column
        const int lane = threadIdx.x & 63;
        const int n = nb0 + lane;
        if (lane < 32 && n < n_rows) atomicAdd(a.dots_next + n, p);
    }
};

template <int BM, int BN, int WM, int WN>
static egg_status launch_i8_gemm(eggroll_ctx* c, const Operand& P, const Operand& Q, int kchunks, const I8Epi::Args& ea)
{
    const int tiles_m = (P.rows + BM - 1) / BM, tiles_n = (Q.rows + BN - 1) / BN;
    const size_t lds = gemm_lds_bytes<BM, BN>();
    if (!operand_offsets_fit(P, BM) || !operand_offsets_fit(Q, BN)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    auto kern = gemm_nt_kernel<MmaI8, BM, BN, WM, WN, false, 1, I8Epi>;
    egg_status st = check_hip(c, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds), "gemm smem attr");
    if (st != EGG_OK) return st;
    KernelScope ks(c, "forward_gemm_i8");
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(WM * WN * 64), lds, c->stream, P, Q, kchunks,
                       tiles_m, tiles_n, (const char*)c->zero_page.p, ea);
    return check_hip(c, hipGetLastError(), "forward_gemm_i8");
}

egg_status launch_forward_i8(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                             int int_bound, int corr_shift, int out_shift, int steps, const int8_t* W,
                             const int8_t* H_in, int8_t* H_out)
{
    const int d = s.d_in;
    const int64_t rows = s.member_count;
    const size_t hbytes = (size_t)rows * d;
    egg_status st;
    if ((st = reserve(c, c->i8_a, hbytes)) != EGG_OK) return st;
    if ((st = reserve(c, c->i8_b, hbytes)) != EGG_OK) return st;
    if ((st = reserve(c, c->i8_h, 2 * ((hbytes + 255) & ~size_t(255)))) != EGG_OK) return st;
    // one row of dot products per step: step t reads row t (filled by the dot kernel for t = 0, by the
    // previous step's epilogue otherwise) and accumulates row t+1
    const size_t dot_row = ((size_t)rows * sizeof(int) + 255) & ~size_t(255);
    if ((st = reserve(c, c->t_buf, dot_row * (size_t)(steps + 1))) != EGG_OK) return st;
    int8_t* A = (int8_t*)c->i8_a.p;
    int8_t* B = (int8_t*)c->i8_b.p;
    int8_t* scratch[2] = {(int8_t*)c->i8_h.p, (int8_t*)c->i8_h.p + ((hbytes + 255) & ~size_t(255))};
    char* dots_base = (char*)c->t_buf.p;

    if ((st = launch_noise(c, ka, (uint32_t)s.member_begin, rows, d, EGG_I8, EGG_UNIFORM_INT, int_bound, A)) != EGG_OK) return st;
    if ((st = launch_noise(c, kb, (uint32_t)s.member_begin, rows, d, EGG_I8, EGG_UNIFORM_INT, int_bound, B)) != EGG_OK) return st;
    {   // a fill kernel rather than a memset node, so that the call can sit inside a captured graph
        const int64_t nz = (int64_t)(dot_row / sizeof(int)) * (steps + 1);
        KernelScope ks(c, "zero_dots");
        hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, c->stream, (int*)dots_base, nz);
    }
    {
        KernelScope ks(c, "dot_i8");
        hipLaunchKernelGGL(dot_i8_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->stream, H_in, B, rows, d, (int*)dots_base);
    }
    if ((st = check_hip(c, hipGetLastError(), "dot_i8 launch")) != EGG_OK) return st;

    const int64_t big_tiles = ((d + 255) / 256) * ((rows + 255) / 256);
    const int8_t* src = H_in;
    for (int t = 0; t < steps; ++t) {
        int8_t* dst = (t == steps - 1) ? H_out : scratch[t & 1];
        const bool alias = (dst == src);  // only possible for steps == 1 with H_out == H_in
        if (alias) dst = scratch[0];
        Operand P{(const char*)W, (int64_t)d, 16, d};
        Operand Q{(const char*)src, (int64_t)d, 16, (int)rows};
        I8Epi::Args ea{A, B, (const int*)(dots_base + dot_row * t), t + 1 < steps ? (int*)(dots_base + dot_row * (t + 1)) : nullptr,
                       dst, d, corr_shift, out_shift};
        st = big_tiles >= 192 ? launch_i8_gemm<256, 256, 2, 4>(c, P, Q, d / 16, ea) : launch_i8_gemm<128, 128, 2, 2>(c, P, Q, d / 16, ea);
        if (st != EGG_OK) return st;
        if (alias) {
            if ((st = check_hip(c, hipMemcpyAsync(H_out, dst, hbytes, hipMemcpyDeviceToDevice, c->stream), "copy back")) != EGG_OK) return st;
        }
        src = dst;
    }
    return EGG_OK;
}

}  // namespace egg

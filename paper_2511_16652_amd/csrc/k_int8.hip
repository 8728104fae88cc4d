// Integer perturbed matmul of the int8 recurrent model, bit-exact
// (App. "Matrix Multiplication": u @ M = I8(uM / (16 sqrt n)), a right shift for n = 4^d;
//  App. "Adding EGGROLL Perturbations": I8((u theta^T + ((u . B) I32(A) >> (4 + sigma_hat))) / (16 sqrt n))).
// Per step: the int8 MFMA NT core computes u theta^T; its epilogue adds the shifted rank-1 term,
// shifts, saturates to [-127, 127], stores int8 and accumulates the next step's u . B_i (the first
// step's dot products come from a wave-per-row dot kernel).
// The factors are fixed while a member is evaluated (Alg. 1), so they are generated once per call
// into scratch and re-read from L2/HBM at every step.
#include "common.hpp"
#include "gemm_core.hpp"
#include <algorithm>

namespace egg {

// Row dot products  d0 = X0 . B0,  d1 = X0 . B1 (optional),  d2 = X1 . B2 (optional)   (int8 x int8 -> int32):
// G lanes per row (16 for short rows, so that every lane has a 16-byte chunk to read; a whole wave otherwise),
// v_dot4 on packed bytes.  Several products in one pass share the loads of X0 (the GRU cell needs three).
// anti: rows 2p, 2p+1 share the factors of pair p, and the odd row uses -B_p.
template <int G>
__global__ __launch_bounds__(256) void dots_i8_kernel(const int8_t* __restrict__ X0, const int8_t* __restrict__ B0,
                                                      const int8_t* __restrict__ B1, const int8_t* __restrict__ X1,
                                                      const int8_t* __restrict__ B2, int64_t rows, int d, int anti,
                                                      int* __restrict__ d0, int* __restrict__ d1, int* __restrict__ d2)
{
    const int lig = threadIdx.x % G;
    const int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
    int acc0 = 0, acc1 = 0, acc2 = 0;
    if (row < rows) {
        const int64_t frow = (anti ? row >> 1 : row) * d;
        const u32x4* x0 = (const u32x4*)(X0 + row * d);
        const u32x4* b0 = (const u32x4*)(B0 + frow);
        for (int ch = lig; ch < (d >> 4); ch += G) {
            const u32x4 xv = x0[ch], bv = b0[ch];
#pragma unroll
            for (int w = 0; w < 4; ++w) acc0 = __builtin_amdgcn_sdot4((int)xv[w], (int)bv[w], acc0, false);
            if (B1) {
                const u32x4 cv = ((const u32x4*)(B1 + frow))[ch];
#pragma unroll
                for (int w = 0; w < 4; ++w) acc1 = __builtin_amdgcn_sdot4((int)xv[w], (int)cv[w], acc1, false);
            }
            if (B2) {
                const u32x4 yv = ((const u32x4*)(X1 + row * d))[ch], ev = ((const u32x4*)(B2 + frow))[ch];
#pragma unroll
                for (int w = 0; w < 4; ++w) acc2 = __builtin_amdgcn_sdot4((int)yv[w], (int)ev[w], acc2, false);
            }
        }
    }
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) {
        acc0 += __shfl_xor(acc0, off, 64);
        acc1 += __shfl_xor(acc1, off, 64);
        acc2 += __shfl_xor(acc2, off, 64);
    }
    if (lig == 0 && row < rows) {
        const bool neg = anti && (row & 1);
        d0[row] = neg ? -acc0 : acc0;
        if (B1) d1[row] = neg ? -acc1 : acc1;
        if (B2) d2[row] = neg ? -acc2 : acc2;
    }
}

egg_status launch_dots_i8(eggroll_ctx* c, const int8_t* X0, const int8_t* B0, const int8_t* B1, const int8_t* X1, const int8_t* B2,
                          int64_t rows, int d, int anti, int* d0, int* d1, int* d2)
{
    KernelScope ks(c, "dot_i8");
    if (d <= 1024)
        hipLaunchKernelGGL(dots_i8_kernel<16>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, c->stream, X0, B0, B1, X1, B2, rows, d, anti, d0, d1, d2);
    else
        hipLaunchKernelGGL(dots_i8_kernel<64>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->stream, X0, B0, B1, X1, B2, rows, d, anti, d0, d1, d2);
    return check_hip(c, hipGetLastError(), "dot_i8 launch");
}

__global__ __launch_bounds__(256) void zero_i32_kernel(int* __restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(256) void zero2_i32_kernel(int* __restrict__ p0, int* __restrict__ p1, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        p0[i] = 0;
        if (p1) p1[i] = 0;
    }
}

// a fill kernel rather than a memset node, so that callers can sit inside a captured graph
egg_status launch_zero_i32(eggroll_ctx* c, int* p0, int* p1, int64_t n)
{
    KernelScope ks(c, "zero_dots");
    hipLaunchKernelGGL(zero2_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, p0, p1, n);
    return check_hip(c, hipGetLastError(), "zero_dots launch");
}

// Epilogue of the integer step.  The MFMA layout gives a lane 4 consecutive outputs of one row of
// h' at a time, i.e. 4-byte accesses 1 KB apart; instead the int32 accumulators of a 32-row block
// are parked in the wave's LDS slice and re-read row-wise, so that a lane finishes 16 consecutive
// outputs of one row: one 16-byte load each of A_i (correction) and B_i (the NEXT step's u . B), one
// 16-byte store of h'.  Wave tiles of 64 columns fetch those factor bytes and the dot products at
// kernel start, so that no global-memory latency sits behind the last MFMA.  The next step's dot
// product is accumulated here: a lane sums h'_j * B_i[j] over its 16 outputs, the lanes of a row are
// combined by shuffles, and one integer atomicAdd per (wave, row) lands in dots_next -- integer
// addition is associative, so the result does not depend on the order of the atomics.
struct I8Args {
    const int8_t* A;  // [rows][d] factors
    const int8_t* B;  // [rows][d] factors that the NEXT matmul dots this one's output with (read only when dots_next)
    const int* dots;  // [rows]  u . B of this step
    int* dots_next;   // [rows]  accumulates u' . B for the next matmul (zeroed beforehand), or NULL; with gate 1 u' is f^
    int8_t* H_out;    // [rows][d]
    int d, corr_shift, out_shift;
    int anti;  // antithetic pairs: rows 2p, 2p+1 read the factors of pair p; the odd row uses -B_p
    // GRU gating fused behind the matmul (App. "GRU"); y = this matmul's I8 result, all operands [rows][d]:
    //   gate 1:  f = I8(other + y + bias)  -> H_out,   f^ = I8(((f + 127) state) >> 8)  -> out2
    //   gate 2:  h^ = I8(other + y + bias),  h = I8(state + I8(((f + 127)(h^ - state)) >> 8))  -> H_out
    int gate;
    const int8_t* g_other;
    const int8_t* g_state;
    const int8_t* g_f;
    const int8_t* g_bias;  // [d]
    int8_t* g_out2;
};

// Stores and no-return atomics issued from inline asm, for the row-streaming kernel.  The compiler's waitcnt
// pass treats vmcnt as in-order only while nothing but loads is pending; one store it knows of turns every
// later use of a loaded register into s_waitcnt vmcnt(0), which would drain the loads of later blocks at
// each epilogue.  Operations it does not know of can only make its counted waits stricter (they occupy
// counter slots), never weaker.  Nothing in the kernel reads these locations back.
__device__ __forceinline__ void store16_untracked(void* p, const u32x4& v)
{
    // the two wait states cover the hazard between a store of more than 64 bits and a VALU write of its data
    // registers, which the compiler's hazard recognizer handles for its own stores but cannot see inside asm
    asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void atomic_add_untracked(int* p, int v)
{
    asm volatile("global_atomic_add %0, %1, off" ::"v"(p), "v"(v) : "memory");
}

// MODE < 0: gate mode and next-dot accumulation are read from the arguments at run time (general core).
// MODE >= 0: both are compile-time constants (gate = MODE & 3, next-dot = MODE >> 2), which strips the other
// variants' code and their uniform branches from a kernel whose time goes into issuing the epilogue.  These
// kernels also use the folded form of the arithmetic (the launcher checks that it cannot overflow):
//     (acc + (p >> cs)) >> os  =  ((acc << cs) + p) >> (cs + os)           nested floors of integers
//     clamp(t >> sh, -127, 127) = clamp(t, -127 << sh, (128 << sh) - 1) >> sh    the shift is monotonic
// i.e. multiply, shift-add, clamp, shift.  (Shifting each result straight into its byte of the output word
// with a hand-written SDWA destination select was tried and removed: the hazard recognizer does not look
// inside inline asm, and gfx950 needs a wait state between a partial-register write and the next read of
// that register, so back-to-back byte writes into one word occasionally read a stale word.)
// SWZ: the staging rows are exactly one wave-tile row of int32 wide (no padding) and the 16-byte slot of a row is
// XOR-swizzled with the row number instead: the transposing accesses stay conflict-free and the slice shrinks to
// 32 * 4 * WTM bytes (what lets the row-streaming kernel keep a three-deep ring at two workgroups per CU).
template <bool DOT24, int MODE = -1, bool SWZ = false>
struct I8Epi {
    typedef int value_t;
    typedef I8Args Args;
    static constexpr int MAX_PF_PASSES = 2;  // wave tiles up to 64 wide prefetch
    __device__ __forceinline__ int gate() const { return MODE >= 0 ? (MODE & 3) : a.gate; }
    __device__ __forceinline__ bool has_next() const { return MODE >= 0 ? (MODE >> 2) != 0 : a.dots_next != nullptr; }
    Args a;
    char* stage;
    int lane;
    u32x4 pa[2][MAX_PF_PASSES], pb[2][MAX_PF_PASSES];  // prefetched bytes of A_i and B_i: [row block][pass]
    int pdot[2][MAX_PF_PASSES];
    int cur_j;
    int row_pitch;  // pitch(wave tile width), fixed by prefetch() at kernel start

    static constexpr __host__ __device__ int pitch(int wtm) { return SWZ ? wtm * 4 : wtm * 4 + 16; }
    static constexpr __host__ __device__ int lds_per_wave(int wtm) { return 32 * pitch(wtm); }
    __device__ __forceinline__ I8Epi(const Args& a_, char* slice, int lane_) : a(a_), stage(slice), lane(lane_), cur_j(-1) {}
    template <int NT, int BM, int BN>
    __device__ __forceinline__ bool tile_begin(char*, int, int, int, int) { return false; }
    template <class MT, int MB, int NB>
    __device__ __forceinline__ void extra_mma(typename MT::acc_t (&)[MB][NB], int, int, int, int) {}

    // pass `it` of a 32-row block: the row (inside the block) and first column (inside the wave tile) of this lane
    template <int WTM>
    __device__ __forceinline__ void pass_coords(int it, int& row, int& mc) const
    {
        constexpr int CPR = WTM / 16;  // 16-byte output chunks per row
        const int c = it * 64 + lane;
        row = c / CPR;
        mc = (c % CPR) * 16;
    }
    template <int WTM>
    __device__ __forceinline__ void fetch(int mw0, int nb0, int it, int n_rows, u32x4& av, u32x4& bv, int& dv) const
    {
        int row, mc;
        pass_coords<WTM>(it, row, mc);
        const int n = min(nb0 + row, n_rows - 1);
        const int m = min(mw0 + mc, a.d - 16);
        const int64_t off = (int64_t)(a.anti ? n >> 1 : n) * a.d + m;
        av = *(const u32x4*)(a.A + off);
        if (has_next()) bv = *(const u32x4*)(a.B + off);
        else bv = u32x4{0u, 0u, 0u, 0u};
        dv = a.dots[n];
    }

    template <int MB, int NB>
    __device__ __forceinline__ void prefetch(int mw0, int nw0, int, int n_rows)
    {
        static_assert(NB <= 2, "prefetch storage");
        row_pitch = pitch(MB * 32);
        if constexpr (MB <= MAX_PF_PASSES) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int it = 0; it < MB; ++it) fetch<MB * 32>(mw0, nw0 + j * 32, it, n_rows, pa[j][it], pb[j][it], pdot[j][it]);
        }
    }
    __device__ __forceinline__ void column(int, bool) { ++cur_j; }
    // Makes the prefetched registers "used" here, so that the one wait for them sits at this point, where only
    // loads are in flight and the compiler waits by count; a first use behind the epilogue's stores would wait
    // for every outstanding memory operation, the loads of later blocks included.
    __device__ __forceinline__ void touch_prefetched()
    {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int it = 0; it < MAX_PF_PASSES; ++it) {
                asm volatile("" ::"v"(pa[j][it]), "v"(pdot[j][it]));
                if (has_next()) asm volatile("" ::"v"(pb[j][it]));
            }
    }
    __device__ __forceinline__ void store4(int, int, const int (&v)[4], bool, int ml)
    {
        const int r = lane & 31;
        *(i32x4*)(stage + r * row_pitch + (SWZ ? (ml * 4) ^ ((r & 15) << 4) : ml * 4)) = i32x4{v[0], v[1], v[2], v[3]};
    }

    // one lane's 16 outputs of row nb0 + row: correction, shift, saturate, store, next-dot partial
    template <int WTM>
    __device__ __forceinline__ void finish_pass(int it, int mw0, int nb0, int n_rows, const u32x4& av, const u32x4& bv, int dv)
    {
        constexpr int P = pitch(WTM), CPR = WTM / 16;
        int row, mc;
        pass_coords<WTM>(it, row, mc);
        const int n = nb0 + row, m = mw0 + mc;
        const bool ok = n < n_rows && m < a.d;
        const char* src = stage + row * P + mc * 4;
        const int64_t idx = (int64_t)min(n, n_rows - 1) * a.d + min(m, a.d - 16);
        u32x4 gv_o = {0u, 0u, 0u, 0u}, gv_s = gv_o, gv_f = gv_o, gv_b = gv_o, out2 = gv_o;
        if (gate()) {  // issued first: their latency hides under the accumulator arithmetic below
            gv_o = *(const u32x4*)(a.g_other + idx);
            gv_s = *(const u32x4*)(a.g_state + idx);
            gv_b = *(const u32x4*)(a.g_bias + min(m, a.d - 16));
            if (gate() == 2) gv_f = *(const u32x4*)(a.g_f + idx);
        }
        u32x4 out;
        int part = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const i32x4 acc4 = SWZ ? *(const i32x4*)(stage + row * P + ((mc * 4 + w * 16) ^ ((row & 15) << 4)))
                                   : *(const i32x4*)(src + w * 16);
            int y[4];
            if constexpr (MODE >= 0) {
                const int sh = a.corr_shift + a.out_shift;
                const int lo = -(127 << sh), hi = (128 << sh) - 1;
                int t[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ae = (int)(int8_t)(av[w] >> (8 * e));
                    const int prod = DOT24 ? __mul24(dv, ae) : dv * ae;
                    t[e] = min(hi, max(lo, (int)((uint32_t)acc4[e] << a.corr_shift) + prod));
                    y[e] = t[e] >> sh;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ae = (int)(int8_t)(av[w] >> (8 * e));
                    // |u . B| < 2^23 was checked on the host when DOT24: the full-rate 24-bit multiply is exact
                    const int prod = DOT24 ? __mul24(dv, ae) : dv * ae;
                    const int corr = prod >> a.corr_shift;  // arithmetic shift: floor
                    y[e] = min(127, max(-127, (acc4[e] + corr) >> a.out_shift));
                }
            }
            if (gate()) {
                int y2[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int sj = (int)(int8_t)(gv_s[w] >> (8 * e));
                    const int sum = min(127, max(-127, (int)(int8_t)(gv_o[w] >> (8 * e)) + y[e] + (int)(int8_t)(gv_b[w] >> (8 * e))));
                    if (gate() == 1) {
                        y[e] = sum;                                                   // f
                        y2[e] = min(127, max(-127, ((sum + 127) * sj) >> 8));         // f^
                    } else {
                        const int fj = (int)(int8_t)(gv_f[w] >> (8 * e));
                        const int delta = min(127, max(-127, ((fj + 127) * (sum - sj)) >> 8));
                        y[e] = min(127, max(-127, sj + delta));                      // h
                        y2[e] = 0;
                    }
                }
                out2[w] = __builtin_amdgcn_perm((uint32_t)y2[1], (uint32_t)y2[0], 0x0c0c0400u) |
                          __builtin_amdgcn_perm((uint32_t)y2[3], (uint32_t)y2[2], 0x04000c0cu);
            }
            // low bytes of y[0..3] -> one word (byte selectors 0-3: second operand, 4-7: first, 0x0c: zero)
            const uint32_t o = __builtin_amdgcn_perm((uint32_t)y[1], (uint32_t)y[0], 0x0c0c0400u) |
                               __builtin_amdgcn_perm((uint32_t)y[3], (uint32_t)y[2], 0x04000c0cu);
            out[w] = o;
            part = __builtin_amdgcn_sdot4((int)(gate() == 1 ? out2[w] : o), (int)bv[w], part, false);
        }
        if constexpr (MODE >= 0) {
            if (ok) store16_untracked(a.H_out + (int64_t)n * a.d + m, out);
            if (ok && gate() == 1) store16_untracked(a.g_out2 + (int64_t)n * a.d + m, out2);
        } else {
            if (ok) *(u32x4*)(a.H_out + (int64_t)n * a.d + m) = out;
            if (ok && gate() == 1) *(u32x4*)(a.g_out2 + (int64_t)n * a.d + m) = out2;
        }
        if (has_next()) {
            if (!ok) part = 0;
            if (a.anti && (n & 1)) part = -part;  // h' . (-B_p)
#pragma unroll
            for (int off = 1; off < CPR; off <<= 1) part += __shfl_xor(part, off, 64);
            if (mc == 0 && n < n_rows) {
                if constexpr (MODE >= 0) atomic_add_untracked(a.dots_next + n, part);
                else atomicAdd(a.dots_next + n, part);
            }
        }
    }

    template <int WTM>
    __device__ __forceinline__ void flush(int mw0, int nb0, int n_rows)
    {
        constexpr int PASSES = WTM / 32;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes have landed
        __builtin_amdgcn_wave_barrier();
        if constexpr (PASSES <= MAX_PF_PASSES) {
            // cur_j is a compile-time constant after unrolling; the select folds away
#pragma unroll
            for (int it = 0; it < PASSES; ++it) {
                if (cur_j == 0) finish_pass<WTM>(it, mw0, nb0, n_rows, pa[0][it], pb[0][it], pdot[0][it]);
                else finish_pass<WTM>(it, mw0, nb0, n_rows, pa[1][it], pb[1][it], pdot[1][it]);
            }
        } else {
            // wide tiles have no registers to spare across the main loop: fetch pass by pass
#pragma unroll
            for (int it = 0; it < PASSES; ++it) {
                u32x4 av, bv;
                int dv;
                fetch<WTM>(mw0, nb0, it, n_rows, av, bv, dv);
                finish_pass<WTM>(it, mw0, nb0, n_rows, av, bv, dv);
            }
        }
        __builtin_amdgcn_wave_barrier();  // the slice is reused by the next row block
    }
};

template <int BM, int BN, int WM, int WN, class Epi>
static egg_status launch_i8_gemm(eggroll_ctx* c, const Operand& P, const Operand& Q, int kchunks, const typename Epi::Args& ea)
{
    const int tiles_m = (P.rows + BM - 1) / BM, tiles_n = (Q.rows + BN - 1) / BN;
    const size_t lds = std::max(gemm_lds_bytes<BM, BN>(), (size_t)WM * WN * Epi::lds_per_wave(BM / WM));
    if (!operand_offsets_fit(P, BM) || !operand_offsets_fit(Q, BN)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    auto kern = gemm_nt_kernel<MmaI8, BM, BN, WM, WN, false, Epi, (BM * BN <= 128 * 128 ? 2 : 1)>;
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, (size_t)lds, "gemm smem attr");
    if (st != EGG_OK) return st;
    KernelScope ks(c, "forward_gemm_i8");
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(WM * WN * 64), lds, c->stream, P, Q, kchunks,
                       tiles_m, tiles_n, 0, (const char*)c->zero_page.p, ea);
    return check_hip(c, hipGetLastError(), "forward_gemm_i8");
}

// Workgroup barrier without the memory fences of __syncthreads(): those wait for every outstanding global load
// and store of the wave -- the loads of later blocks and the epilogue's stores, which the row-streaming kernel
// keeps in flight across its barriers.  What the barrier has to order there is LDS traffic only: the ring is
// written by direct-to-LDS loads whose arrival the kernel confirms itself (s_waitcnt vmcnt) before the barrier,
// and read by ds_read instructions whose results the MFMAs have consumed before the barrier that frees a buffer.
// The empty asm statements keep the compiler from moving memory accesses across it.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Row-streaming form of the matmul for d_in = 256 (the integer model's width): K is so short that a tile
// of the general core is all prologue and epilogue, so here a workgroup is persistent instead.  Its four
// waves keep the MFMA fragments of a 256-row slice of theta in registers for the whole kernel (64 rows x
// 256 bytes per wave = 64 VGPRs), and blocks of 64 activation rows stream through a three-deep LDS ring
// filled by direct-to-LDS loads.  The waves of this kernel spend about half their life in s_waitcnt (measured),
// so the order of an iteration is built around keeping loads in flight:
//     multiply block b  ->  barrier (its buffer is free)  ->  epilogue of b  ->  fetch the factor bytes and
//     dot products of b+1 into the registers the epilogue just finished with  ->  issue the loads of b+3 into
//     the freed buffer  ->  wait until only that prefetch and those loads are outstanding  ->  barrier.
// Loads complete in issue order among themselves, so the last wait proves that block b+1 has landed
// and that the epilogue's stores are done (after which a use of the prefetched registers waits by count and
// leaves block b+3's loads in flight through the next multiply and epilogue).  Every load named in that count
// is issued unconditionally.  Column slices of a wider theta (the 4D x D matrix of the MLP) that read the same
// rows sit on the same XCD, next to each other in launch order, so that the second to fourth read of a row
// block hits that XCD's L2.
// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding (vmcnt is split over
// bits 3:0 and 15:14; the other counters are left at "do not wait")
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

template <class Epi>
__global__ __launch_bounds__(256, 2) void stream_i8_kernel(const int8_t* __restrict__ W, int d_out, Operand Q, int tiles_m,
                                                           int nstreams, int nblocks, int conservative, typename Epi::Args ea)
{
    constexpr int BN = 64, NT = 256, WTM = 64, MB = 2, NB = 2, PITCH = 128, RING = 3;
    constexpr int HALF = BN * PITCH;  // 64 rows x one 128-byte half of K
    constexpr int BUF = 2 * HALF;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int tm = q % tiles_m;
    const int stream = xcd * (nstreams >> 3) + q / tiles_m;
    const int m0 = tm * 256, mw0 = m0 + wave * WTM;
    char* const slice = lds + RING * BUF + wave * Epi::lds_per_wave(WTM);

    // theta fragments: lane reads row (lane & 31) of a 32-row block, chunk 2 ks + (lane >> 5) of each K half
    u32x4 wf[2][4][MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        const int row = min(mw0 + i * 32 + (lane & 31), d_out - 1);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) wf[h][ks][i] = *(const u32x4*)(W + (size_t)row * 256 + (h * 8 + 2 * ks + (lane >> 5)) * 16);
    }
    const int frow = lane & 31, fsw = (frow >> 1) & 7;
    int foff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) foff[ks] = frow * PITCH + (((2 * ks + (lane >> 5)) ^ fsw) << 4);

    DmaLoader<BN, NT, false> lq;
    auto issue = [&](int nb, int buf) {   // four loads per lane, unconditional
        const int n0 = nb * BN;
        lq.init(Q, n0, tid);
        const char* g = Q.base + (int64_t)n0 * Q.row_stride;
        lq.load(g, 0, 16, nullptr, lds + buf * BUF, wave);
        lq.load(g + 128, 8, 16, nullptr, lds + buf * BUF + HALF, wave);
    };

    int nb = stream;
    if (nb >= nblocks) return;
    issue(nb, 0);
    if (nb + nstreams < nblocks) issue(nb + nstreams, 1);
    if (nb + 2 * nstreams < nblocks) issue(nb + 2 * nstreams, 2);
    Epi epi(ea, slice, lane);
    epi.template prefetch<MB, NB>(mw0, nb * BN, lane, Q.rows);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    lds_barrier();
    int cur = 0;
    for (; nb < nblocks; nb += nstreams) {
        const char* buf = lds + cur * BUF;   // block nb is in LDS: every wave confirmed its share before the last barrier
        i32x16 acc[MB][NB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4 fb[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) fb[j] = *(const u32x4*)(buf + h * HALF + j * 32 * PITCH + foff[ks]);
#pragma unroll
                for (int i = 0; i < MB; ++i)
#pragma unroll
                    for (int j = 0; j < NB; ++j) MmaI8::mma(wf[h][ks][i], fb[j], acc[i][j]);
            }
        lds_barrier();  // every wave has read block nb: its buffer is free
        epi.touch_prefetched();
        const int n0 = nb * BN;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int n = n0 + j * 32 + (lane & 31);
            const bool nvalid = n < Q.rows;
            epi.column(n, nvalid);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int ml = i * 32 + qq * 8 + (lane >> 5) * 4;
                    int v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * qq + e];
                    epi.store4(mw0 + ml, n, v, nvalid, ml);
                }
            epi.template flush<WTM>(mw0, n0 + j * 32, Q.rows);
        }
        const int nb1 = nb + nstreams, nb3 = nb + 3 * nstreams;
        epi = Epi(ea, slice, lane);   // its registers are dead: the next block's factor bytes load straight into them
        if (nb3 < nblocks) {
            epi.template prefetch<MB, NB>(mw0, nb1 * BN, lane, Q.rows);   // 2 or 3 loads for each of its 4 passes
            issue(nb3, cur);
            // Block nb+1 (issued two iterations ago) must have landed; what may stay in flight, in issue order: the
            // ring loads of block nb+2, the factor prefetch of block nb+1 just issued, the ring loads of block nb+3.
            // The counts are those of the source (fetch() loads A_i, B_i and the dot product, plus B_next with a
            // next-dot epilogue; issue() is two DmaLoader passes); the conservative form waits for everything and
            // exists so that a test can hold the counted form against it bit for bit.
            constexpr int RING_LOADS = 2 * DmaLoader<BN, NT, false>::L;
            constexpr int PF_LOADS_PLAIN = MB * NB * 2, PF_LOADS_NEXT = MB * NB * 3;
            static_assert(2 * RING_LOADS + PF_LOADS_NEXT == 20 && 2 * RING_LOADS + PF_LOADS_PLAIN == 16, "outstanding-load budget of the ring");
            if (conservative) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            else if (epi.has_next()) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * RING_LOADS + PF_LOADS_NEXT));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * RING_LOADS + PF_LOADS_PLAIN));
        } else {
            if (nb1 < nblocks) epi.template prefetch<MB, NB>(mw0, nb1 * BN, lane, Q.rows);
            __builtin_amdgcn_s_waitcnt(0x0F70);  // the last blocks: everything
        }
        cur = cur == RING - 1 ? 0 : cur + 1;
        lds_barrier();  // all waves have confirmed their share of block nb+1
    }
}

template <class Epi>
static egg_status launch_i8_stream(eggroll_ctx* c, const int8_t* W, int d_out, const Operand& Q, const typename Epi::Args& ea)
{
    const int tiles_m = (d_out + 255) / 256;
    const int nblocks = (Q.rows + 63) / 64;
    int nstreams = std::max(8, (512 / tiles_m) & ~7);
    nstreams = std::min(nstreams, (nblocks + 7) & ~7);
    const size_t lds = 3 * 2 * 64 * 128 + 4 * Epi::lds_per_wave(64);   // ring of three blocks + the waves' staging slices
    if (!operand_offsets_fit(Q, 64)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    auto kern = stream_i8_kernel<Epi>;
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, (size_t)lds, "stream smem attr");
    if (st != EGG_OK) return st;
    KernelScope ks(c, "forward_stream_i8");
    hipLaunchKernelGGL(kern, dim3((unsigned)(nstreams * tiles_m)), dim3(256), lds, c->stream, W, d_out, Q, tiles_m, nstreams, nblocks,
                       c->conservative_waits ? 1 : 0, ea);
    return check_hip(c, hipGetLastError(), "forward_stream_i8");
}

// Kernel choice for one integer matmul: the row-streaming kernel at the integer model's width, otherwise the
// general core with 256 x 256 tiles when those fill the chip, else 128 x 128 tiles (two workgroups per CU).
static egg_status dispatch_i8(eggroll_ctx* c, const int8_t* W, int d_out, int d_in, int64_t rows, int int_bound, const Operand& Q,
                              const I8Args& ea)
{
    // |u . B_i| <= d_in * 127 * (largest noise magnitude): below 2^23 the correction product fits the 24-bit multiplier
    const int nmax = noise_max(int_bound);
    const bool dot24 = (int64_t)d_in * 127 * nmax < (int64_t(1) << 23);
    // the streaming kernel folds the two shifts into one: needs |acc| 2^cs + |dot A| inside int32 and clamp bounds that fit
    const int sh = ea.corr_shift + ea.out_shift;
    const bool fold_ok = sh <= 23 && (((int64_t)d_in * 127 * 127) << ea.corr_shift) + (int64_t)d_in * 127 * nmax * nmax < (int64_t(1) << 31);
    if (d_in == 256 && rows >= 2048 && fold_ok)
    {
        const int mode = ea.gate | (ea.dots_next ? 4 : 0);
        switch (mode) {
#define EGG_STREAM_CASE(M) \
            case M: return dot24 ? launch_i8_stream<I8Epi<true, M, true>>(c, W, d_out, Q, ea) : launch_i8_stream<I8Epi<false, M, true>>(c, W, d_out, Q, ea);
            EGG_STREAM_CASE(0) EGG_STREAM_CASE(1) EGG_STREAM_CASE(2) EGG_STREAM_CASE(4) EGG_STREAM_CASE(5) EGG_STREAM_CASE(6)
#undef EGG_STREAM_CASE
            default: return fail(c, EGG_EINVAL, "gate mode %d", ea.gate);
        }
    }
    const int64_t big_tiles = ((d_out + 255) / 256) * ((rows + 255) / 256);
    Operand P{(const char*)W, (int64_t)d_in, 16, d_out};
    // ungated matmuls (the recurrence of the single-matrix cell, the MLP's second matrix) get the epilogue with
    // compile-time mode when the folded arithmetic is safe; gated ones at other widths keep the run-time form
    const int mode = (ea.gate == 0 && fold_ok) ? (ea.dots_next ? 4 : 0) : -1;
#define EGG_GEMM_CASE(BM, BN, WM, WN, M) \
    if (mode == M) return dot24 ? launch_i8_gemm<BM, BN, WM, WN, I8Epi<true, M>>(c, P, Q, d_in / 16, ea) : launch_i8_gemm<BM, BN, WM, WN, I8Epi<false, M>>(c, P, Q, d_in / 16, ea);
    if (big_tiles >= 192) {
        EGG_GEMM_CASE(256, 256, 2, 4, 0) EGG_GEMM_CASE(256, 256, 2, 4, 4) EGG_GEMM_CASE(256, 256, 2, 4, -1)
    }
    EGG_GEMM_CASE(128, 128, 2, 2, 0) EGG_GEMM_CASE(128, 128, 2, 2, 4) EGG_GEMM_CASE(128, 128, 2, 2, -1)
#undef EGG_GEMM_CASE
    return fail(c, EGG_EINVAL, "no kernel for this mode");
}

// One perturbed integer matmul on factor buffers that already exist:  dst = I8((src W^T + ((src . B) A >> cs)) >> os).
// dots: `rows` int32, computed here unless dots_ready.  With dots_next (zeroed by the caller) the epilogue also accumulates
// the dot products of the output rows (of f^ under gate 1) with B_next, factors of the matmul that consumes them.  Used by the GRU cell, whose factors are generated once per call.
egg_status launch_i8_matmul(eggroll_ctx* c, const int8_t* A, const int8_t* B, int anti, int64_t rows, int d_out, int d_in,
                            int int_bound, int corr_shift, int out_shift, const int8_t* W, const int8_t* src, int8_t* dst,
                            int* dots, bool dots_ready, const I8Gate* gate, const int8_t* B_next, int* dots_next)
{
    egg_status st;
    if (!dots_ready && (st = launch_dots_i8(c, src, B, nullptr, nullptr, nullptr, rows, d_in, anti, dots, nullptr, nullptr)) != EGG_OK) return st;
    Operand Q{(const char*)src, (int64_t)d_in, 16, (int)rows};
    I8Args ea{A, B_next, dots, dots_next, dst, d_out, corr_shift, out_shift, anti, 0, nullptr, nullptr, nullptr, nullptr, nullptr};
    if (gate) {
        ea.gate = gate->mode;
        ea.g_other = gate->other; ea.g_state = gate->state; ea.g_f = gate->f; ea.g_bias = gate->bias; ea.g_out2 = gate->out2;
    }
    return dispatch_i8(c, W, d_out, d_in, rows, int_bound, Q, ea);
}

egg_status launch_forward_i8(eggroll_ctx* c, const StreamKey& ka, const StreamKey& kb, const egg_shape& s,
                             int int_bound, int corr_shift, int out_shift, int steps, const int8_t* W,
                             const int8_t* H_in, int8_t* H_out)
{
    const int d_in = s.d_in, d_out = s.d_out;  // more than one step feeds h' back in: the API checks d_out == d_in
    const int64_t rows = s.member_count;
    const int anti = s.antithetic ? 1 : 0;
    const int64_t noise_ids = anti ? rows / 2 : rows;
    const uint32_t first_id = (uint32_t)(anti ? s.member_begin / 2 : s.member_begin);
    const size_t obytes = (size_t)rows * d_out;
    egg_status st;
    if ((st = reserve(c, c->i8_a, (size_t)noise_ids * d_out)) != EGG_OK) return st;
    if ((st = reserve(c, c->i8_b, (size_t)noise_ids * d_in)) != EGG_OK) return st;
    if ((st = reserve(c, c->i8_h, 2 * ((obytes + 255) & ~size_t(255)))) != EGG_OK) return st;
    // one row of dot products per step: step t reads row t (filled by the dot kernel for t = 0, by the
    // previous step's epilogue otherwise) and accumulates row t+1
    const size_t dot_row = ((size_t)rows * sizeof(int) + 255) & ~size_t(255);
    if ((st = reserve(c, c->t_buf, dot_row * (size_t)(steps + 1))) != EGG_OK) return st;
    int8_t* A = (int8_t*)c->i8_a.p;
    int8_t* B = (int8_t*)c->i8_b.p;
    int8_t* scratch[2] = {(int8_t*)c->i8_h.p, (int8_t*)c->i8_h.p + ((obytes + 255) & ~size_t(255))};
    char* dots_base = (char*)c->t_buf.p;

    if ((st = launch_noise(c, ka, first_id, noise_ids, d_out, EGG_I8, EGG_UNIFORM_INT, int_bound, A)) != EGG_OK) return st;
    if ((st = launch_noise(c, kb, first_id, noise_ids, d_in, EGG_I8, EGG_UNIFORM_INT, int_bound, B)) != EGG_OK) return st;
    if (steps > 1) {   // a fill kernel rather than a memset node, so that the call can sit inside a captured graph
        const int64_t nz = (int64_t)(dot_row / sizeof(int)) * (steps + 1);
        KernelScope ks(c, "zero_dots");
        hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, c->stream, (int*)dots_base, nz);
    }
    if ((st = launch_dots_i8(c, H_in, B, nullptr, nullptr, nullptr, rows, d_in, anti, (int*)dots_base, nullptr, nullptr)) != EGG_OK) return st;

    const int8_t* src = H_in;
    for (int t = 0; t < steps; ++t) {
        int8_t* dst = (t == steps - 1) ? H_out : scratch[t & 1];
        const bool alias = (dst == src);  // only possible for steps == 1 with H_out == H_in
        if (alias) dst = scratch[0];
        Operand Q{(const char*)src, (int64_t)d_in, 16, (int)rows};
        // the epilogue's row length is d_out (rows of A_i and of h'); with a next step d_out == d_in, so B_i fits too
        I8Args ea{A, B, (const int*)(dots_base + dot_row * t), t + 1 < steps ? (int*)(dots_base + dot_row * (t + 1)) : nullptr,
                       dst, d_out, corr_shift, out_shift, anti, 0, nullptr, nullptr, nullptr, nullptr, nullptr};
        st = dispatch_i8(c, W, d_out, d_in, rows, int_bound, Q, ea);
        if (st != EGG_OK) return st;
        if (alias) {
            if ((st = check_hip(c, hipMemcpyAsync(H_out, dst, obytes, hipMemcpyDeviceToDevice, c->stream), "copy back")) != EGG_OK) return st;
        }
        src = dst;
    }
    return EGG_OK;
}

}  // namespace egg

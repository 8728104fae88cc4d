// MFMA "NT" GEMM core for gfx950:  C[m][n] = sum_k P[m][k] * Q[n][k]
//
// Both operands are addressed as 16-byte K-chunks (8 bf16/fp16, 16 int8 or 4 fp32 values that are
// consecutive in K), so one core serves
//   - the shared GEMM of the population forward  (P = W rows, Q = X rows, both row-major), Sec. 4.2
//   - the update contraction (diag(f)A)^T B over K = N*r (P, Q = K-packed factor panels), Sec. 4.2
//   - the int8 x int8 -> int32 matmul of the integer model, App. "Matrix Multiplication".
// A workgroup owns a BM x BN tile of C; 64-wide waves own 32x32 MFMA blocks of it.  K advances in
// tiles of 8 chunks (128 bytes per row), double-buffered in LDS.  Rows of an LDS tile are 128 bytes
// with the chunk slot XOR-swizzled by (row>>1)&7, which makes the 16-byte fragment reads of any 16
// neighbouring rows hit distinct banks; the swizzle is applied on the global side so that
// direct-to-LDS loads (which place lane t's 16 bytes at base + 16 t) can be used.
// The epilogue is a functor that receives, per lane, 4 consecutive rows m..m+3 of one column n:
// that is exactly one aligned group of factor entries A_i[m..m+3][:] for the member of column n.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace egg {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte K-chunk
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

struct Operand {
    const char* base;    // device pointer to row 0, chunk 0
    int64_t row_stride;  // bytes between consecutive rows
    int64_t kc_stride;   // bytes between consecutive 16-byte K-chunks of a row
    int rows;            // valid rows
};

struct MmaBf16 {
    static constexpr int MFMA_PER_MMA = 1;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
struct MmaF16 {
    static constexpr int MFMA_PER_MMA = 1;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
struct MmaI8 {
    static constexpr int MFMA_PER_MMA = 1;
    typedef i32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    }
};
struct MmaF32 {  // a 16-byte chunk holds 4 k-values: four 32x32x2 products
    static constexpr int MFMA_PER_MMA = 4;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[0]), __uint_as_float(b[0]), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[1]), __uint_as_float(b[1]), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[2]), __uint_as_float(b[2]), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[3]), __uint_as_float(b[3]), c, 0, 0, 0);
    }
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so ids that are congruent
// mod 8 share an L2.  Give each XCD a contiguous run of tiles, and walk tiles in groups of GM rows
// so that a run covers a compact block of C (few distinct P and Q panels per L2).
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int& tm, int& tn)
{
    const int total = tiles_m * tiles_n;
    if ((total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);
    const int GM = 4;
    const int per_group = GM * tiles_n;
    const int g = pid / per_group;
    const int first_m = g * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_group = pid - g * per_group;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

// Global -> LDS movement of one K-tile (BM + BN rows of 128 bytes).  Load `it` of a thread covers
// chunk-linear index it*NT + tid: row = idx/8, LDS slot = idx%8.  Addresses are a wave-uniform
// 64-bit base (tile origin + K offset, kept in scalar registers) plus a loop-invariant 32-bit
// per-lane offset.  DIRECT uses the LDS-DMA form of the global load (lane t of a wave lands at
// base + 16 t); otherwise the tile is staged in registers and written with ds_write_b128.
template <int BM, int BN, int NT, bool DIRECT>
struct Loader {
    static constexpr int LP = BM * 8 / NT, LQ = BN * 8 / NT;
    u32x4 rp[DIRECT ? 1 : LP], rq[DIRECT ? 1 : LQ];

    template <int L>
    __device__ __forceinline__ void side(const char* base, const uint32_t (&off)[L], const int (&chunk)[L], int kfirst,
                                         int kchunks, bool tail, char* sdst, const char* zero_page, int wave,
                                         u32x4 (&regs)[DIRECT ? 1 : L])
    {
#pragma unroll
        for (int it = 0; it < L; ++it) {
            const char* g = base + (uint64_t)off[it];
            if (tail && kfirst + chunk[it] >= kchunks) g = zero_page;
            if constexpr (DIRECT) {
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                                 (lds_ptr_t)(sdst + (it * NT + wave * 64) * 16), 16, 0, 0);
            } else {
                regs[it] = *(const u32x4*)g;
            }
        }
    }

    __device__ __forceinline__ void issue(int kt, int kchunks, char* sbase, const char* pb, const char* qb,
                                          const uint32_t (&po)[LP], const uint32_t (&qo)[LQ], const int (&cp)[LP],
                                          const int (&cq)[LQ], int64_t pstep, int64_t qstep, const char* zero_page,
                                          int wave)
    {
        const char* pk = pb + (int64_t)kt * pstep;
        const char* qk = qb + (int64_t)kt * qstep;
        if (kt * 8 + 8 <= kchunks) {  // full K-tile: no predicate on the loads
            side<LP>(pk, po, cp, kt * 8, kchunks, false, sbase, zero_page, wave, rp);
            side<LQ>(qk, qo, cq, kt * 8, kchunks, false, sbase + BM * 128, zero_page, wave, rq);
        } else {
            side<LP>(pk, po, cp, kt * 8, kchunks, true, sbase, zero_page, wave, rp);
            side<LQ>(qk, qo, cq, kt * 8, kchunks, true, sbase + BM * 128, zero_page, wave, rq);
        }
    }
    __device__ __forceinline__ void commit(char* sbase, int tid)
    {
        if constexpr (!DIRECT) {
#pragma unroll
            for (int it = 0; it < LP; ++it) *(u32x4*)(sbase + (it * NT + tid) * 16) = rp[it];
#pragma unroll
            for (int it = 0; it < LQ; ++it) *(u32x4*)(sbase + BM * 128 + (it * NT + tid) * 16) = rq[it];
        }
    }
};

// Largest per-lane byte offset the loader forms must fit 32 bits (checked on the host).
inline bool operand_offsets_fit(const Operand& o, int tile_rows)
{
    return (int64_t)tile_rows * o.row_stride + 8 * o.kc_stride < (int64_t(1) << 32);
}

// Epi requirements:
//   struct Args (trivially copyable);  __device__ Epi(const Args&, char* lds_scratch);
//   __device__ void column(int n, bool valid);                       called once per owned column
//   __device__ void store4(int m, int n, const T (&v)[4], bool col_valid);   rows m..m+3 of column n
//
// Main loop, per K-tile (4 MFMA k-steps): the fragments of k-step s+1 are read from LDS while the
// MFMAs of k-step s run (two fragment register sets); the global->LDS loads of the next K-tile are
// issued right after the barrier that retires the previous one, so they have a whole tile of MFMA
// work to land; the single barrier per K-tile sits in the middle of the last k-step.
template <class MT, int BM, int BN, int WM, int WN, bool DIRECT, class Epi>
__global__ __launch_bounds__(WM* WN * 64, 1) void gemm_nt_kernel(Operand P, Operand Q, int kchunks, int tiles_m,
                                                                   int tiles_n, const char* zero_page,
                                                                   typename Epi::Args ea)
{
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MB = WTM / 32, NB = WTN / 32;
    constexpr int LP = BM * 8 / NT, LQ = BN * 8 / NT;  // 16-byte loads per thread per K-tile
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile rows must divide over the threads");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tiles are made of 32x32 blocks");
    constexpr int STAGE_BYTES = (BM + BN) * 128;

    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;

    int tm, tn;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- global -> LDS addressing -------------------------------------------------------------
    // load `it` of this thread covers chunk-linear index c = it*NT + tid of the tile:
    // row = c / 8, LDS slot = c % 8, global chunk = slot ^ ((row>>1)&7).
    const char* pb = P.base + (int64_t)m0 * P.row_stride;
    const char* qb = Q.base + (int64_t)n0 * Q.row_stride;
    uint32_t po[LP], qo[LQ];
    int cp[LP], cq[LQ];  // global chunk index (0..7) of each load, for the K tail
#pragma unroll
    for (int it = 0; it < LP; ++it) {
        const int c = it * NT + tid;
        const int row = c >> 3;
        cp[it] = (c & 7) ^ ((row >> 1) & 7);
        const int rl = min(row, P.rows - 1 - m0);  // rows past the end re-read the last valid row
        po[it] = (uint32_t)((int64_t)rl * P.row_stride + (int64_t)cp[it] * P.kc_stride);
    }
#pragma unroll
    for (int it = 0; it < LQ; ++it) {
        const int c = it * NT + tid;
        const int row = c >> 3;
        cq[it] = (c & 7) ^ ((row >> 1) & 7);
        const int rl = min(row, Q.rows - 1 - n0);
        qo[it] = (uint32_t)((int64_t)rl * Q.row_stride + (int64_t)cq[it] * Q.kc_stride);
    }
    const int64_t pstep = 8 * P.kc_stride, qstep = 8 * Q.kc_stride;

    // ---- LDS fragment addressing ----------------------------------------------------------------
    // lane reads row (lane&31) of a 32-row block, chunk 2*ks + (lane>>5); rows of a block start at a
    // multiple of 32, so the swizzle term depends on the lane only.
    const int frow = lane & 31;
    const int fsw = (frow >> 1) & 7;
    int foff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) foff[ks] = frow * 128 + (((2 * ks + (lane >> 5)) ^ fsw) << 4);
    const int a_base = wm * WTM * 128;
    const int b_base = BM * 128 + wn * WTN * 128;

    typename MT::acc_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int KT = (kchunks + 7) >> 3;
    Loader<BM, BN, NT, DIRECT> ld;
    u32x4 fa[2][MB], fb[2][NB];

#define EGG_READ_FRAGS(BUF, STAGE, KS)                                                                         \
    {                                                                                                          \
        const char* sa_ = lds + (STAGE)*STAGE_BYTES + a_base + foff[KS];                                       \
        const char* sb_ = lds + (STAGE)*STAGE_BYTES + b_base + foff[KS];                                       \
        _Pragma("unroll") for (int i = 0; i < MB; ++i) fa[BUF][i] = *(const u32x4*)(sa_ + i * 32 * 128);       \
        _Pragma("unroll") for (int j = 0; j < NB; ++j) fb[BUF][j] = *(const u32x4*)(sb_ + j * 32 * 128);       \
    }
#define EGG_MMA_ROWS(BUF, I0, I1)                                                                              \
    _Pragma("unroll") for (int i = I0; i < I1; ++i) _Pragma("unroll") for (int j = 0; j < NB; ++j)             \
        MT::mma(fa[BUF][i], fb[BUF][j], acc[i][j]);
// interleave: one LDS fragment read behind each of the first MB+NB MFMAs of a k-step
#define EGG_SCHED_STEP()                                                                                       \
    _Pragma("unroll") for (int r_ = 0; r_ < MB + NB; ++r_) {                                                   \
        __builtin_amdgcn_sched_group_barrier(0x008, MT::MFMA_PER_MMA, 0);                                      \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                     \
    }                                                                                                          \
    __builtin_amdgcn_sched_group_barrier(0x008, (MB * NB - MB - NB) * MT::MFMA_PER_MMA, 0);

    ld.issue(0, kchunks, lds, pb, qb, po, qo, cp, cq, pstep, qstep, zero_page, wave);
    ld.commit(lds, tid);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): direct-to-LDS data has landed
    __syncthreads();
    EGG_READ_FRAGS(0, 0, 0)

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        char* nxt = lds + (cur ^ 1) * STAGE_BYTES;
        if (more) ld.issue(kt + 1, kchunks, nxt, pb, qb, po, qo, cp, cq, pstep, qstep, zero_page, wave);
        EGG_READ_FRAGS(1, cur, 1)
        EGG_MMA_ROWS(0, 0, MB)
        EGG_SCHED_STEP()
        EGG_READ_FRAGS(0, cur, 2)
        EGG_MMA_ROWS(1, 0, MB)
        EGG_SCHED_STEP()
        EGG_READ_FRAGS(1, cur, 3)
        EGG_MMA_ROWS(0, 0, MB)
        EGG_SCHED_STEP()
        EGG_MMA_ROWS(1, 0, MB / 2)
        if (more) ld.commit(nxt, tid);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (more) EGG_READ_FRAGS(0, cur ^ 1, 0)
        EGG_MMA_ROWS(1, MB / 2, MB)
    }
#undef EGG_READ_FRAGS
#undef EGG_MMA_ROWS
#undef EGG_SCHED_STEP

    // ---- epilogue -------------------------------------------------------------------------------
    Epi epi(ea, lds);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int n = n0 + wn * WTN + j * 32 + (lane & 31);
        const bool nvalid = n < Q.rows;
        epi.column(n, nvalid);
#pragma unroll
        for (int i = 0; i < MB; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = m0 + wm * WTM + i * 32 + q * 8 + (lane >> 5) * 4;
                typename Epi::value_t v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
                epi.store4(m, n, v, nvalid);
            }
        }
    }
}

}  // namespace egg

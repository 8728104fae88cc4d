// MFMA "NT" GEMM core for gfx950:  C[m][n] = sum_k P[m][k] * Q[n][k]
//
// Both operands are addressed as 16-byte K-chunks (8 bf16/fp16, 16 int8 or 4 fp32 values that are
// consecutive in K), so one core serves
//   - the shared GEMM of the population forward  (P = W rows, Q = X rows, both row-major), Sec. 4.2
//   - the update contraction (diag(f)A)^T B over K = N*r (P, Q = K-packed factor panels), Sec. 4.2
//   - the int8 x int8 -> int32 matmul of the integer model, App. "Matrix Multiplication".
// A workgroup owns a BM x BN tile of C; 64-wide waves own 32x32 MFMA blocks of it.  K advances in
// stages of 8 chunks (128 bytes per row) double-buffered in LDS and filled by direct-to-LDS loads
// (global_load_lds, 16 bytes per lane): the loads of stage kt+2 are issued right behind the barrier
// that retires stage kt's buffer and land while stage kt+1 is multiplied.  Nothing is staged in
// registers and no ds_write is issued.  (Measured at 4096^3 bf16: 103 us against 117 us for the earlier
// register-staged form -- global_load_dwordx4 one stage ahead, ds_write_b128 -- whose LDS instruction
// count and LDS wait cycles were twice those of the vendor library's kernel; the stage-synchronous form
// of the direct load alone already streams 16.8 TB/s from L2 into LDS.)
// Stage layouts: row-major operands keep 128-byte rows with the chunk slot XOR-swizzled by (row>>1)&7,
// which makes the 16-byte fragment reads of any 16 neighbouring rows hit distinct banks; K-packed
// operands use a chunk-major stage ([chunk][row][16 B]) whose fragment reads are 32 consecutive slots.
// The epilogue is a functor that receives, per lane, 4 consecutive rows m..m+3 of one column n:
// that is exactly one aligned group of factor entries A_i[m..m+3][:] for the member of column n.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace egg {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
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
    static constexpr int BLK = 32;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
// The same contraction from 16x16x32 blocks.  Both shapes retire 1024 flops per cycle and CU and read the same
// fragment bytes from LDS, but on ordinary (non-constant) operands the chip clocks higher under the 16x16x32 form:
// measured with MFMAs alone 2.0 PFLOP/s against 1.7, and 1.40 against 1.22 inside this kernel's loop structure
// (fragment reads, one barrier and 64 KB of direct-to-LDS loads per stage).
struct MmaBf16Blk16 {
    static constexpr int MFMA_PER_MMA = 1;
    static constexpr int BLK = 16;
    typedef f32x4 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
struct MmaF16 {
    static constexpr int MFMA_PER_MMA = 1;
    static constexpr int BLK = 32;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
struct MmaI8 {
    static constexpr int MFMA_PER_MMA = 1;
    static constexpr int BLK = 32;
    typedef i32x16 acc_t;
    static __device__ __forceinline__ void mma(const u32x4& a, const u32x4& b, acc_t& c)
    {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    }
};
struct MmaF32 {  // a 16-byte chunk holds 4 k-values: four 32x32x2 products
    static constexpr int MFMA_PER_MMA = 4;
    static constexpr int BLK = 32;
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

// f(integral_constant<int, J>) for J = FIRST .. LAST-1, unrolled by construction
template <int FIRST, int LAST, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (FIRST < LAST) {
        f(std::integral_constant<int, FIRST>{});
        static_for<FIRST + 1, LAST>(f);
    }
}

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

// Global -> LDS movement of one K-stage (ROWS rows x 8 chunks of 16 bytes) by direct-to-LDS loads: lane i
// of a wave's load lands at LDS base + 16 i, so slot idx = it*NT + tid sits at byte 16 idx of the operand's
// half of the stage, and the lane fetches the chunk that belongs there:
//   row-major operands (KMAJOR = false): row idx/8, position idx%8 holds chunk k = (idx%8) ^ swizzle(row);
//                                        8 neighbouring lanes cover the 128 contiguous bytes of one row;
//   K-packed operands  (KMAJOR = true) : row idx % ROWS of chunk idx / ROWS;
//                                        64 lanes read 64 consecutive rows of one chunk plane: 1 KB.
// Addresses are a wave-uniform 64-bit base (tile origin + K offset, kept in scalar registers) plus a
// loop-invariant 32-bit per-lane offset.
typedef __attribute__((address_space(3))) void egg_lds_void;
typedef __attribute__((address_space(1))) const void egg_glb_void;
// TAIL = false: the caller guarantees that K is a whole number of stages (no zero-page redirection, and the
// chunk numbers need not be kept).
template <int ROWS, int NT, bool KMAJOR, bool TAIL = true>
struct DmaLoader {
    static constexpr int L = ROWS * 8 / NT;
    uint32_t off[L];
    int chunk[TAIL ? L : 1];
    __device__ __forceinline__ void init(const Operand& o, int row0, int tid)
    {
#pragma unroll
        for (int it = 0; it < L; ++it) {
            const int idx = it * NT + tid;
            const int row = KMAJOR ? idx % ROWS : idx >> 3;
            const int ch = KMAJOR ? idx / ROWS : (idx & 7) ^ ((row >> 1) & 7);
            if constexpr (TAIL) chunk[it] = ch;
            const int rl = min(row, o.rows - 1 - row0);  // rows past the end re-read the last valid row
            off[it] = (uint32_t)((int64_t)rl * o.row_stride + (int64_t)ch * o.kc_stride);
        }
    }
    // chunks past the end of K (only possible in the last stage) read the zero page instead
    __device__ __forceinline__ void load(const char* base, int kfirst, int kchunks, const char* zero_page, char* sdst, int wave) const
    {
#pragma unroll
        for (int it = 0; it < L; ++it) {
            const char* g = base + (uint64_t)off[it];
            if constexpr (TAIL) {
                if (kfirst + chunk[it] >= kchunks) g = zero_page;
            }
            __builtin_amdgcn_global_load_lds((egg_glb_void*)g, (egg_lds_void*)(sdst + (it * NT + wave * 64) * 16), 16, 0, 0);
        }
    }
};

// Largest per-lane byte offset the loader forms must fit 32 bits (checked on the host).
inline bool operand_offsets_fit(const Operand& o, int tile_rows)
{
    return (int64_t)tile_rows * o.row_stride + 8 * o.kc_stride < (int64_t(1) << 32);
}

template <int BM, int BN>
constexpr size_t gemm_lds_bytes()
{
    return (size_t)2 * (BM + BN) * 128;
}

// ---- main-loop pieces of the 16x16x32 form, shared by the one-tile kernel and the persistent kernel below ------
// A stage holds two k-steps of 32; each is multiplied in two units of MB/2 block rows, so a stage is four units
// of equal MFMA time.  The A fragments are double-buffered per unit, the B fragments per k-step; every unit reads
// the A fragments of the next one, units 0 and 3 also the B fragments of the next k-step.  The barrier sits in the
// middle of unit 3; all fragment reads of the stage have returned there (lgkmcnt(0)), so the loads that follow it
// may overwrite the buffer.  (The macros use the kernels' local names.)
#define EGG_READ_A(BUF, STAGE, KS_, H_)                                                                        \
    {                                                                                                          \
        const char* sa_ = lds + (STAGE)*STAGE_BYTES + a_base + foff[KS_] + (H_)*HB * BLK * PITCH;              \
        _Pragma("unroll") for (int i = 0; i < HB; ++i) fa[BUF][i] = *(const u32x4*)(sa_ + i * BLK * PITCH);    \
    }
#define EGG_READ_B(BUF, STAGE, KS_)                                                                            \
    {                                                                                                          \
        const char* sb_ = lds + (STAGE)*STAGE_BYTES + b_base + foff[KS_];                                      \
        _Pragma("unroll") for (int j = 0; j < NB; ++j) fb[BUF][j] = *(const u32x4*)(sb_ + j * BLK * PITCH);    \
    }
#define EGG_MMA_UNIT(ABUF, BBUF, H_, I0, I1)                                                                   \
    _Pragma("unroll") for (int i = I0; i < I1; ++i) _Pragma("unroll") for (int j = 0; j < NB; ++j)             \
        MT::mma(fa[ABUF][i], fb[BBUF][j], acc[(H_)*HB + i][j]);
// one LDS read behind each of the first NR_ MFMAs of a unit
#define EGG_SCHED16(NR_)                                                                                       \
    _Pragma("unroll") for (int r_ = 0; r_ < HB * NB; ++r_) {                                                   \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                     \
        if (r_ < (NR_)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                     \
    }
#define EGG_ITER16(KT_, NEXT, LOAD2)                                                                           \
    {                                                                                                          \
        const int cur_ = (KT_)&1;                                                                              \
        const int lk_ = (KT_) + 2;                                                                             \
        EGG_READ_A(1, cur_, 0, 1)                                                                              \
        EGG_READ_B(1, cur_, 1)                                                                                 \
        EGG_MMA_UNIT(0, 0, 0, 0, HB)                                                                           \
        EGG_SCHED16(HB + NB)                                                                                   \
        EGG_READ_A(0, cur_, 1, 0)                                                                              \
        EGG_MMA_UNIT(1, 0, 1, 0, HB)                                                                           \
        EGG_SCHED16(HB)                                                                                        \
        EGG_READ_A(1, cur_, 1, 1)                                                                              \
        EGG_MMA_UNIT(0, 1, 0, 0, HB)                                                                           \
        EGG_SCHED16(HB)                                                                                        \
        EGG_MMA_UNIT(1, 1, 1, 0, HB / 2)                                                                       \
        __builtin_amdgcn_s_waitcnt(0x0070); /* vmcnt(0) lgkmcnt(0): own direct loads landed, own reads done */ \
        __syncthreads();                                                                                       \
        if (LOAD2) {                                                                                           \
            lp.load(pb + (int64_t)lk_ * pstep, lk_ * 8, kchunks, zero_page, lds + cur_ * STAGE_BYTES, wave);   \
            lq.load(qb + (int64_t)lk_ * qstep, lk_ * 8, kchunks, zero_page, lds + cur_ * STAGE_BYTES + BM * PITCH, wave); \
        }                                                                                                      \
        if (NEXT) {                                                                                            \
            EGG_READ_A(0, cur_ ^ 1, 0, 0)                                                                      \
            EGG_READ_B(0, cur_ ^ 1, 0)                                                                         \
        }                                                                                                      \
        EGG_MMA_UNIT(1, 1, 1, HB / 2, HB)                                                                      \
    }

// Epi requirements:
//   struct Args (trivially copyable);  static constexpr int lds_per_wave(int wtm);
//   __device__ Epi(const Args&, char* wave_lds_slice, int lane);
//   __device__ void column(int n, bool valid);                       called once per owned column (persistent kernel: column_at<J>, store4_at<I, J>)
//   __device__ void store4(int m, int n, const T (&v)[4], bool col_valid, int ml);  rows m..m+3 of column n
//   template <int WTM> __device__ void flush(int mw0, int nb0, int n_rows);   after each 32-column block
//   template <int MB, int NB> __device__ void prefetch(int mw0, int nw0, int lane, int n_rows);   late in the main loop
//   template <class MT, int MB, int NB> __device__ void extra_mma(acc_t (&acc)[MB][NB], int mw0, int nw0, int lane, int n_rows);
//   template <int NT, int BM, int BN> __device__ bool tile_begin(char* lds_tail, int m0, int n0, int tid, int n_rows);
//       called by all threads before the per-wave part; returns whether a barrier is needed
//
// Main loop, per K-stage (4 MFMA k-steps): the fragments of k-step s+1 are read from LDS while the
// MFMAs of k-step s run (two fragment register sets).  The single barrier of the stage sits in the
// middle of k-step 3; right behind it the direct-to-LDS loads of stage kt+2 go out into the buffer the
// barrier retired, and the first fragments of stage kt+1 are read.
// KMAJOR: both operands are K-packed panels (chunk-major stages); otherwise row-major operands.
// an epilogue may take the column block as a compile-time index (column_at<J>) instead of column()
template <class E, int J, class = void>
struct has_column_at : std::false_type {};
template <class E, int J>
struct has_column_at<E, J, std::void_t<decltype(std::declval<E&>().template column_at<J>(0, true))>> : std::true_type {};
// ... and the row block and group of a store (store4_blk<I, Q>) instead of store4()
template <class E, class = void>
struct has_store4_blk : std::false_type {};
template <class E>
struct has_store4_blk<E, std::void_t<decltype(&E::template store4_blk<0, 0>)>> : std::true_type {};
template <int I, int Q, class E, class V>
__device__ __forceinline__ void epi_store4(E& e, int m, int n, const V (&v)[4], bool valid, int ml)
{
    if constexpr (has_store4_blk<E>::value) e.template store4_blk<I, Q>(m, n, v, valid, ml);
    else e.store4(m, n, v, valid, ml);
}
template <int J, class E>
__device__ __forceinline__ void epi_column(E& e, int n, bool valid)
{
    if constexpr (has_column_at<E, J>::value) e.template column_at<J>(n, valid);
    else e.column(n, valid);
}

template <class MT, int BM, int BN, int WM, int WN, bool KMAJOR, class Epi, int WG_PER_CU = 1>
__global__ __launch_bounds__(WM* WN * 64, WG_PER_CU) void gemm_nt_kernel(Operand P, Operand Q, int kchunks, int tiles_m,
                                                                   int tiles_n, int ksplit, const char* zero_page,
                                                                   typename Epi::Args ea)
{
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int BLK = MT::BLK;  // rows and columns of one MFMA block
    constexpr int MB = WTM / BLK, NB = WTN / BLK;
    constexpr int PITCH = 128;  // bytes per LDS row
    constexpr int STAGE_BYTES = (BM + BN) * PITCH;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "stage rows must divide over the threads");
    static_assert(BLK == 32 || BLK == 16, "MFMA block shapes: 32x32 (K = 16 per step) or 16x16 (K = 32 per step)");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && MB % 2 == 0, "wave tiles are made of whole MFMA blocks");
    static_assert(BLK == 32 || !KMAJOR, "the 16x16 form is written for row-major operands");

    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;

    // split-K (ksplit > 0): consecutive groups of tiles_m * tiles_n workgroups own consecutive ranges of
    // ksplit K-chunks; the epilogue stores partial tiles that a later pass combines
    int tile_id = blockIdx.x, kbeg = 0;
    if (ksplit > 0) {
        const int tiles = tiles_m * tiles_n;
        const int sp = tile_id / tiles;
        tile_id -= sp * tiles;
        kbeg = sp * ksplit;
        kchunks = min(kchunks - kbeg, ksplit);
    }
    int tm, tn;
    tile_coords(tile_id, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    // The epilogue may fetch small per-tile side data ahead of time instead of paying global-memory
    // latency behind the last MFMA: its prefetch hook runs before the last K-stage.
    Epi epi(ea, lds + wave * Epi::lds_per_wave(WTM), lane);
#define EGG_EPI_PREFETCH epi.template prefetch<MB, NB>(m0 + wm * WTM, n0 + wn * WTN, lane, Q.rows);

    const char* pb = P.base + (int64_t)m0 * P.row_stride + (int64_t)kbeg * P.kc_stride;
    const char* qb = Q.base + (int64_t)n0 * Q.row_stride + (int64_t)kbeg * Q.kc_stride;
    DmaLoader<BM, NT, KMAJOR> lp;
    DmaLoader<BN, NT, KMAJOR> lq;
    lp.init(P, m0, tid);
    lq.init(Q, n0, tid);
    const int64_t pstep = 8 * P.kc_stride, qstep = 8 * Q.kc_stride;

    // ---- LDS fragment addressing ----------------------------------------------------------------
    // lane reads row (lane&31) of a 32-row block, chunk 2*ks + (lane>>5); rows of a block start at a
    // multiple of 32, so the swizzle term depends on the lane only.
    // (16x16 blocks: row (lane&15), chunk 4*ks + (lane>>4), two k-steps per stage)
    constexpr int KSTEPS = BLK == 32 ? 4 : 2;          // MFMA k-steps per stage
    constexpr int CPS = 8 / KSTEPS;                    // 16-byte chunks per k-step and row
    const int frow = lane & (BLK - 1);
    const int fsw = (frow >> 1) & 7;
    int foff[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) foff[ks] = frow * PITCH + (((CPS * ks + lane / BLK) ^ fsw) << 4);
    const int a_base = wm * WTM * PITCH;
    const int b_base = BM * PITCH + wn * WTN * PITCH;
    // chunk-major stages: chunk c of row r at (c * ROWS + r) * 16 inside the operand's half of the stage
    const int a_row16 = (wm * WTM + frow) * 16, b_row16 = BM * PITCH + (wn * WTN + frow) * 16;

    typename MT::acc_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < BLK * BLK / 64; ++e) acc[i][j][e] = 0;

    const int KT = (kchunks + 7) >> 3;
  if constexpr (BLK == 32) {
    u32x4 fa[2][MB], fb[2][NB];

#define EGG_READ_FRAGS(BUF, STAGE, KS_)                                                                        \
    {                                                                                                          \
        const int c_ = 2 * (KS_) + (lane >> 5);                                                                \
        const char* sa_ = lds + (STAGE)*STAGE_BYTES + (KMAJOR ? a_row16 + c_ * BM * 16 : a_base + foff[KS_]);  \
        const char* sb_ = lds + (STAGE)*STAGE_BYTES + (KMAJOR ? b_row16 + c_ * BN * 16 : b_base + foff[KS_]);  \
        constexpr int BLK_ = KMAJOR ? 32 * 16 : 32 * PITCH;                                                    \
        _Pragma("unroll") for (int i = 0; i < MB; ++i) fa[BUF][i] = *(const u32x4*)(sa_ + i * BLK_);           \
        _Pragma("unroll") for (int j = 0; j < NB; ++j) fb[BUF][j] = *(const u32x4*)(sb_ + j * BLK_);           \
    }
#define EGG_MMA_ROWS(BUF, I0, I1)                                                                              \
    _Pragma("unroll") for (int i = I0; i < I1; ++i) _Pragma("unroll") for (int j = 0; j < NB; ++j)             \
        MT::mma(fa[BUF][i], fb[BUF][j], acc[i][j]);
// Scheduling patterns (sched_group_barrier masks: 0x008 MFMA, 0x100 LDS read, 0x200 LDS write,
// 0x020 VMEM read).  Every k-step pairs one LDS fragment read with each of its first MB+NB MFMAs;
// k-step 1 additionally spreads the ds_writes of the next stage, k-step 2 the global loads of the
// stage after it, so that neither forms a block of memory-only instructions before the barrier.
#define EGG_SCHED(MASK_A, N_A, MASK_B, N_B)                                                                    \
    {                                                                                                          \
        constexpr int NM_ = MB * NB * MT::MFMA_PER_MMA, NR_ = MB + NB;                                         \
        constexpr int PA_ = ((N_A) + NM_ - 1) / NM_, PB_ = ((N_B) + NM_ - 1) / NM_;                            \
        _Pragma("unroll") for (int r_ = 0; r_ < NM_; ++r_) {                                                   \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                 \
            if (r_ < NR_) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                   \
            if ((N_A) > 0 && r_ * PA_ < (N_A)) __builtin_amdgcn_sched_group_barrier(MASK_A, PA_, 0);           \
            if ((N_B) > 0 && r_ * PB_ < (N_B)) __builtin_amdgcn_sched_group_barrier(MASK_B, PB_, 0);           \
        }                                                                                                      \
    }
// One K-stage.  The barrier in k-step 3 retires this stage's buffer (every wave has read its last
// fragments from it), so the loads of stage kt+2 are issued right behind it, straight into that buffer,
// and have a whole stage of MFMA work to land: the next barrier waits for them.
#define EGG_ITER(KT_, NEXT, LOAD2)                                                                         \
    {                                                                                                          \
        const int cur_ = (KT_)&1;                                                                              \
        const int lk_ = (KT_) + 2;                                                                             \
        EGG_READ_FRAGS(1, cur_, 1)                                                                             \
        EGG_MMA_ROWS(0, 0, MB)                                                                                 \
        EGG_SCHED(0, 0, 0, 0)                                                                                  \
        EGG_READ_FRAGS(0, cur_, 2)                                                                             \
        EGG_MMA_ROWS(1, 0, MB)                                                                                 \
        EGG_SCHED(0, 0, 0, 0)                                                                                  \
        EGG_READ_FRAGS(1, cur_, 3)                                                                             \
        EGG_MMA_ROWS(0, 0, MB)                                                                                 \
        EGG_SCHED(0, 0, 0, 0)                                                                                  \
        EGG_MMA_ROWS(1, 0, MB / 2)                                                                             \
        __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0): this wave's direct-to-LDS loads have landed */        \
        __syncthreads();                                                                                       \
        if (LOAD2) {                                                                                           \
            lp.load(pb + (int64_t)lk_ * pstep, lk_ * 8, kchunks, zero_page, lds + cur_ * STAGE_BYTES, wave);   \
            lq.load(qb + (int64_t)lk_ * qstep, lk_ * 8, kchunks, zero_page, lds + cur_ * STAGE_BYTES + BM * PITCH, wave); \
        }                                                                                                      \
        if (NEXT) EGG_READ_FRAGS(0, cur_ ^ 1, 0)                                                               \
        EGG_MMA_ROWS(1, MB / 2, MB)                                                                            \
    }

    // prologue: stages 0 and 1 straight into the two buffers
    lp.load(pb, 0, kchunks, zero_page, lds, wave);
    lq.load(qb, 0, kchunks, zero_page, lds + BM * PITCH, wave);
    if (KT > 1) {
        lp.load(pb + pstep, 8, kchunks, zero_page, lds + STAGE_BYTES, wave);
        lq.load(qb + qstep, 8, kchunks, zero_page, lds + STAGE_BYTES + BM * PITCH, wave);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    EGG_READ_FRAGS(0, 0, 0)
    int kt = 0;
    for (; kt + 2 < KT; ++kt) EGG_ITER(kt, true, true)           // steady state
    if (kt + 1 < KT) { EGG_ITER(kt, true, false) ++kt; }          // the last stage is already on its way
    EGG_EPI_PREFETCH
    EGG_ITER(kt, false, false)                                    // last stage
#undef EGG_ITER
#undef EGG_SCHED
#undef EGG_READ_FRAGS
#undef EGG_MMA_ROWS
  } else {
    // 16x16x32 blocks: the units described above the kernel
    constexpr int HB = MB / 2;
    u32x4 fa[2][HB], fb[2][NB];
    static_assert(HB % 2 == 0, "unit 3 is split around the barrier");
    lp.load(pb, 0, kchunks, zero_page, lds, wave);
    lq.load(qb, 0, kchunks, zero_page, lds + BM * PITCH, wave);
    if (KT > 1) {
        lp.load(pb + pstep, 8, kchunks, zero_page, lds + STAGE_BYTES, wave);
        lq.load(qb + qstep, 8, kchunks, zero_page, lds + STAGE_BYTES + BM * PITCH, wave);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    EGG_READ_A(0, 0, 0, 0)
    EGG_READ_B(0, 0, 0)
    int kt = 0;
    for (; kt + 2 < KT; ++kt) EGG_ITER16(kt, true, true)
    if (kt + 1 < KT) { EGG_ITER16(kt, true, false) ++kt; }
    EGG_EPI_PREFETCH
    EGG_ITER16(kt, false, false)
  }

    // ---- epilogue -------------------------------------------------------------------------------
    // The LDS stages are dead now; each wave gets a private slice of them as staging space, so that
    // an epilogue can turn the MFMA layout (a lane owns 4 consecutive rows of one column) into
    // row-contiguous 16-byte stores.
    __syncthreads();
    // an epilogue may fold per-column-block rank-r terms into the accumulators with a few more MFMAs
    epi.template extra_mma<MT, MB, NB>(acc, m0 + wm * WTM, n0 + wn * WTN, lane, Q.rows);
    // workgroup-level hook: an epilogue may pull per-tile side data into the LDS behind the wave slices
    if (epi.template tile_begin<NT, BM, BN>(lds + WM * WN * Epi::lds_per_wave(WTM), m0, n0, tid, Q.rows)) __syncthreads();
    // (a compile-time loop: were the optimiser to leave it rolled, acc would be indexed at run time and live in scratch)
    static_for<0, NB>([&](auto jc) __attribute__((always_inline)) {
        constexpr int j = decltype(jc)::value;
        const int n = n0 + wn * WTN + j * BLK + (lane & (BLK - 1));
        const bool nvalid = n < Q.rows;
        epi_column<j>(epi, n, nvalid);
        static_for<0, MB>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            static_for<0, (BLK == 32 ? 4 : 1)>([&](auto qc) __attribute__((always_inline)) {
                constexpr int q = decltype(qc)::value;
                // 32x32 block: four groups of 4 rows, 8 apart, offset by the lane half; 16x16: rows 4 (lane>>4) ..+3
                const int ml = i * BLK + (BLK == 32 ? q * 8 + (lane >> 5) * 4 : (lane >> 4) * 4);  // row inside the wave tile
                typename Epi::value_t v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
                epi_store4<i, q>(epi, m0 + wm * WTM + ml, n, v, nvalid, ml);
            });
        });
        epi.template flush<WTM>(m0 + wm * WTM, n0 + wn * WTN + j * BLK, Q.rows);
    });
}

// Staging helper for epilogues whose output is row-major [n][m] with 2-byte elements: store4 parks a
// lane's 4 consecutive m-values of column n in the wave's LDS slice as row (n mod block size); flush writes
// the ROWS x WTM block out with 16-byte stores, 16 lanes per 256 contiguous bytes.
struct RowStager2B {
    char* base;
    int lane;
    int row;  // the lane's column of the MFMA block = row of the staged block: lane & (block size - 1)
    static constexpr __host__ __device__ int pitch(int wtm) { return wtm * 2 + 16; }
    static constexpr __host__ __device__ int bytes(int wtm) { return 32 * pitch(wtm); }
    __device__ __forceinline__ void put(int wtm_pitch, int ml, uint32_t lo, uint32_t hi) const
    {
        *(uint2*)(base + row * wtm_pitch + ml * 2) = make_uint2(lo, hi);
    }
    // out: element pointer of the row-major destination with `ld` elements per row; rows nb0..nb0+31
    // (valid below n_rows), columns mw0..mw0+WTM-1 (valid below m_cols, a multiple of 4)
    template <int WTM, int ROWS = 32>
    __device__ __forceinline__ void flush(uint16_t* out, int64_t ld, int mw0, int nb0, int n_rows, int m_cols) const
    {
        constexpr int P = pitch(WTM), CPR = WTM / 8;  // 16-byte chunks per row
        static_assert(ROWS * CPR % 64 == 0, "whole wave passes");
        __builtin_amdgcn_s_waitcnt(0xC07F);           // lgkmcnt(0): the wave's own LDS writes have landed
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < ROWS * CPR / 64; ++it) {
            const int c = it * 64 + lane;
            const int row = c / CPR, cc = c % CPR;
            const int n = nb0 + row, m = mw0 + cc * 8;
            if (n < n_rows && m < m_cols) {
                const u32x4 v = *(const u32x4*)(base + row * P + cc * 16);
                uint16_t* dst = out + (int64_t)n * ld + m;
                if (m + 8 <= m_cols) *(u32x4*)dst = v;
                else *(uint2*)dst = make_uint2(v[0], v[1]);
            }
        }
        __builtin_amdgcn_wave_barrier();  // the slice is reused by the next column block
    }
};


// The same staging in half the space: 16 rows (one 16x16 column block) of WTM 2-byte elements without padding,
// the 16-byte chunks of a row XOR-swizzled by the row number instead.  A store4 of 16 rows x 2 lane groups then
// covers 16 distinct chunks (all 64 banks once), and flush reads whole rows.  At WTM = 128 the eight waves of a
// workgroup need 32 KB: what a 160 KB LDS leaves beside two 64 KB stages, so a persistent kernel can stage one
// tile's output while the next tile's first stages are already landing.
struct RowStagerSwz {
    char* base;
    int lane;
    int row;
    static constexpr __host__ __device__ int pitch(int wtm) { return wtm * 2; }
    static constexpr __host__ __device__ int bytes(int wtm) { return 16 * pitch(wtm); }
    __device__ __forceinline__ void put(int wtm_pitch, int ml, uint32_t lo, uint32_t hi) const
    {
        const int chunks = wtm_pitch >> 4;  // per row, a power of two
        const int c = ((ml >> 3) ^ row) & (chunks - 1);
        *(uint2*)(base + row * wtm_pitch + (c << 4) + ((ml >> 2) & 1) * 8) = make_uint2(lo, hi);
    }
    template <int WTM, int ROWS = 16>
    __device__ __forceinline__ void flush(uint16_t* out, int64_t ld, int mw0, int nb0, int n_rows, int m_cols) const
    {
        static_assert(ROWS == 16, "one 16-column block at a time");
        constexpr int P = pitch(WTM), CPR = WTM / 8;
        static_assert(ROWS * CPR % 64 == 0 && (CPR & (CPR - 1)) == 0, "whole wave passes over power-of-two rows");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes have landed
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < ROWS * CPR / 64; ++it) {
            const int c = it * 64 + lane;
            const int r = c / CPR, cc = c % CPR;
            const int n = nb0 + r, m = mw0 + cc * 8;
            if (n < n_rows && m < m_cols) {
                const u32x4 v = *(const u32x4*)(base + r * P + (((cc ^ r) & (CPR - 1)) << 4));
                uint16_t* dst = out + (int64_t)n * ld + m;
                if (m + 8 <= m_cols) *(u32x4*)dst = v;
                else *(uint2*)dst = make_uint2(v[0], v[1]);
            }
        }
        __builtin_amdgcn_wave_barrier();  // the slice is reused by the next column block
    }
};

// Persistent form of the 16x16x32 kernel for epilogues that only store (no workgroup-level staging of side data):
// one workgroup per compute unit walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...  After the last MFMA of a
// tile the two stage buffers are free, so the direct-to-LDS loads of the NEXT tile's stages 0 and 1 go out first;
// the epilogue of the finished tile (staged through the 32 KB of LDS behind the stages) then runs while they land,
// and nothing waits for a workgroup to drain its stores, be retired and be replaced.  (Measured at K = 2048: the
// one-tile kernel spends 3 us of a tile on its prologue and 7 us from the first store to the next workgroup's
// first MFMA.)
template <class MT, int BM, int BN, int WM, int WN, class Epi>
__global__ __launch_bounds__(WM* WN * 64, 1) void gemm_nt_persistent_kernel(Operand P, Operand Q, int kchunks, int tiles_m,
                                                                      int tiles_n, const char* zero_page,
                                                                      typename Epi::Args ea)
{
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int BLK = MT::BLK;
    static_assert(BLK == 16, "written for the 16x16x32 form");
    constexpr int MB = WTM / BLK, NB = WTN / BLK, HB = MB / 2;
    constexpr int PITCH = 128;
    constexpr int STAGE_BYTES = (BM + BN) * PITCH;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0 && HB % 2 == 0, "tile shape");
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int total = tiles_m * tiles_n;
    const int64_t pstep = 8 * P.kc_stride, qstep = 8 * Q.kc_stride;
    const int KT = (kchunks + 7) >> 3;

    constexpr int KSTEPS = 2, CPS = 4;
    const int frow = lane & (BLK - 1);
    const int fsw = (frow >> 1) & 7;
    int foff[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) foff[ks] = frow * PITCH + (((CPS * ks + lane / BLK) ^ fsw) << 4);
    const int a_base = wm * WTM * PITCH;
    const int b_base = BM * PITCH + wn * WTN * PITCH;

    DmaLoader<BM, NT, false, false> lp;  // K is a whole number of stages (checked on the host)
    DmaLoader<BN, NT, false, false> lq;

    int tile = blockIdx.x;
    if (tile >= total) return;
    int tm, tn;
    tile_coords(tile, tiles_m, tiles_n, tm, tn);
    int m0 = tm * BM, n0 = tn * BN;
    const char* pb = P.base + (int64_t)m0 * P.row_stride;
    const char* qb = Q.base + (int64_t)n0 * Q.row_stride;
    lp.init(P, m0, tid);
    lq.init(Q, n0, tid);
#define EGG_FIRST_STAGES                                                                   \
    lp.load(pb, 0, kchunks, zero_page, lds, wave);                                         \
    lq.load(qb, 0, kchunks, zero_page, lds + BM * PITCH, wave);                            \
    if (KT > 1) {                                                                          \
        lp.load(pb + pstep, 8, kchunks, zero_page, lds + STAGE_BYTES, wave);               \
        lq.load(qb + qstep, 8, kchunks, zero_page, lds + STAGE_BYTES + BM * PITCH, wave);  \
    }
    EGG_FIRST_STAGES
    for (;;) {
        typename MT::acc_t acc[MB][NB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[i][j][e] = 0;
        u32x4 fa[2][HB], fb[2][NB];
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's part of stages 0 and 1 has landed
        __syncthreads();
        EGG_READ_A(0, 0, 0, 0)
        EGG_READ_B(0, 0, 0)
        int kt = 0;
        for (; kt + 2 < KT; ++kt) EGG_ITER16(kt, true, true)
        if (kt + 1 < KT) { EGG_ITER16(kt, true, false) ++kt; }
        // The epilogue object is built here, from a lane number the optimiser cannot trace back: otherwise the
        // per-lane staging and store addresses, which do not depend on the tile, are hoisted out of the tile loop
        // and held in registers (then spilled) through every main loop.
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        Epi epi(ea, lds + 2 * STAGE_BYTES + wave * Epi::lds_per_wave(WTM), lane_e);
        epi.template prefetch<MB, NB>(m0 + wm * WTM, n0 + wn * WTN, lane_e, Q.rows);
        EGG_ITER16(kt, false, false)

        // Rank-r terms folded into the accumulators first: their operands were fetched a stage ago, and a wait for
        // them placed behind the next tile's loads would wait for those as well (the counter retires in order).
        epi.template extra_mma<MT, MB, NB>(acc, m0 + wm * WTM, n0 + wn * WTN, lane_e, Q.rows);
        // the barrier of the last stage had every wave's last fragment reads behind it: both stage buffers are free
        const int cm0 = m0, cn0 = n0;  // the finished tile
        const int next = tile + (int)gridDim.x;
        {
            // Straight-line on purpose (past its last tile a workgroup fetches the finished tile's stages again, unused):
            // behind a branch the compiler can no longer count these loads, and every wait of the epilogue for a load of
            // its own would become a wait for all of them.
            tile_coords(next < total ? next : tile, tiles_m, tiles_n, tm, tn);
            m0 = tm * BM;
            n0 = tn * BN;
            pb = P.base + (int64_t)m0 * P.row_stride;
            qb = Q.base + (int64_t)n0 * Q.row_stride;
            lp.init(P, m0, tid);
            lq.init(Q, n0, tid);
            EGG_FIRST_STAGES
        }
        static_for<0, NB>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            const int n = cn0 + wn * WTN + j * BLK + (lane_e & (BLK - 1));
            const bool nvalid = n < Q.rows;
            epi.template column_at<j>(n, nvalid);
            static_for<0, MB>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value;
                const int ml = i * BLK + (lane_e >> 4) * 4;
                typename Epi::value_t v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][e];
                epi.template store4_at<i, j>(cm0 + wm * WTM + ml, n, v, nvalid, ml);
            });
            epi.template flush<WTM>(cm0 + wm * WTM, cn0 + wn * WTN + j * BLK, Q.rows);
        });
        if (next >= total) break;
        tile = next;
    }
#undef EGG_FIRST_STAGES
}

#undef EGG_ITER16
#undef EGG_SCHED16
#undef EGG_MMA_UNIT
#undef EGG_READ_A
#undef EGG_READ_B

}  // namespace egg

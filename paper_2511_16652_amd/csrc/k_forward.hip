// Population forward of one linear layer (Sec. 4.2):
//   Y = X W^T   (shared MFMA GEMM over all N*S rows)   +   (sigma/sqrt r) t A_i^T   (epilogue)
// The epilogue regenerates exactly the factor entries A_i[j..j+3][:] that the lane's four outputs
// need -- for one row per member every entry of A is produced exactly once over the grid -- applies
// the correction in fp32, optionally keeps A_i for the update, applies the activation and stores.
#include "common.hpp"
#include "gemm_core.hpp"

namespace egg {

// gelu(x) = x Phi(x) for outputs that are rounded to bf16.  Every vector-ALU slot of the epilogue is exposed time
// (one slot per element costs about 1 % of a K = 2048 tile), and the library erff costs about 27 of them.  Here
// Phi(x) - 1/2 is an odd degree-17 polynomial on [-4, 4] (least squares on Chebyshev nodes, pinned to 1/2 at the
// ends so that the clamp continues it with Phi = 0 and Phi = 1): 12 slots.  |error of gelu| <= 2e-5 inside
// (-3.8, 3.8) and <= 1.3e-4 at |x| = 4 (the neglected tail 4 Phi(-4)); a bf16 ulp of gelu is larger than that
// wherever |gelu(x)| > 0.03.  fp32 outputs keep erff.
// Four values at a time, step by step, so that the four Horner chains are independent neighbours in the
// instruction stream (a dependent fma cannot issue back to back).
__device__ __forceinline__ void gelu_bf16_grade4(float (&y)[4])
{
    float xc[4], x2[4], p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) xc[e] = __builtin_amdgcn_fmed3f(y[e], -4.0f, 4.0f);
#pragma unroll
    for (int e = 0; e < 4; ++e) x2[e] = xc[e] * xc[e];
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = fmaf(8.809068429e-11f, x2[e], -7.454938351e-09f);
#define EGG_GELU_STEP(C) _Pragma("unroll") for (int e = 0; e < 4; ++e) p[e] = fmaf(p[e], x2[e], C);
    EGG_GELU_STEP(2.826503707e-07f)
    EGG_GELU_STEP(-6.433988670e-06f)
    EGG_GELU_STEP(9.985887631e-05f)
    EGG_GELU_STEP(-1.137293224e-03f)
    EGG_GELU_STEP(9.882503528e-03f)
    EGG_GELU_STEP(-6.641100396e-02f)
    EGG_GELU_STEP(3.989198364e-01f)
#undef EGG_GELU_STEP
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] *= fmaf(xc[e], p[e], 0.5f);
}

// Arguments of the forward epilogue (the same for every instantiation).
struct FwdArgs {
    StreamKey ka;
    uint32_t member_begin;
    int S, d_out;
    float c;  // sigma / sqrt(r); 0 switches the correction off
    int act, y_bf16;
    void* Y;
    const float* t;
    void* A_buf;  // REGEN: optional cache to fill; otherwise the materialised factors to read
    int wtm_pitch;  // RowStager2B::pitch of the launched wave tile
    int stage_a;    // !REGEN: the tile's slice of A fits the LDS tail and is staged there
    int mma_corr;   // !REGEN, bf16, S % CORR_COLS == 0: the correction is folded in by one extra MFMA per block
    int pair_share; // REGEN with antithetic pairs: neighbouring lanes share their factors
    const void* resid;  // optional [R][d_out] of the output dtype, added after the activation (residual stream)
    const void* next_B;  // LEAN_PROJ: the next layer's factors B[member][d_out][rank] (bf16; its rank is this layer's)
    float* next_part;    // LEAN_PROJ: partial projections [d_out / 128 slabs][R][rank]
};

// Where the lane's factor entries A_i[m..m+3][0..RANK-1] come from:
//   REGEN  (rank 1, one row per member): regenerated in registers from the counter stream -- each
//          entry of A is needed by exactly one lane of the grid, so nothing is stored or re-read;
//   otherwise read from a materialised [member][d_out][RANK] buffer (written just before by the
//          noise kernel, the caller's A_cache if one was given): with S rows per member the buffer
//          is RANK/S of the output size, and every entry is generated once instead of S times.
// BLK: rows/columns of the MFMA block the kernel is built from (a lane owns column lane & (BLK-1) of a block).
// LEAN != 0: a store-only epilogue for bf16 outputs whose correction is either off (c == 0) or already folded into
// the accumulators by extra_mma; the activation and the residual are fixed at compile time (bit 1: GELU, bit 2:
// residual).  The general epilogue decides all of that at run time and carries the code of every case (counter RNG,
// erff, staged and direct factor reads) 32 times per wave: about 80 KB, more than the instruction cache that two
// compute units share, and it runs once per tile -- measured at 13 us behind a 50 us main loop, against 5 us for
// the lean form.
// bit 3 (LEAN_PROJ): the rows this layer stores are the input of the next perturbed layer, whose rank-1 projection
// t'[n] = sum_m Y[n][m] B'[m] is formed here from the very bf16 values that are stored, so that Y is not read again
// by a projection pass: a lane adds its 4 x 8 products per column, the four lane groups of a column are summed by two
// shuffles, and the sum over the wave tile's 128 rows goes to a slab-partial that a small pass adds up in fixed order.
enum { LEAN_ON = 1, LEAN_GELU = 2, LEAN_RESID = 4, LEAN_PROJ = 8 };
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// sum over the 16 lanes of a DPP row, left in every lane of the row
__device__ __forceinline__ float row_sum16(float x)
{
#define EGG_DPP_ADD(CTRL) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
    EGG_DPP_ADD(0xB1)   // quad_perm [1, 0, 3, 2]
    EGG_DPP_ADD(0x4E)   // quad_perm [2, 3, 0, 1]
    EGG_DPP_ADD(0x141)  // row_half_mirror: the other quad of the half row
    EGG_DPP_ADD(0x140)  // row_mirror: the other half row
#undef EGG_DPP_ADD
    return x;
}
template <bool BF16, int RANK, bool REGEN, int BLK = 32, int LEAN = 0>
struct FwdEpi {
    static_assert(LEAN == 0 || (BF16 && !REGEN), "the lean epilogue stores bf16 and regenerates nothing");
    typedef float value_t;
    typedef FwdArgs Args;
    static constexpr int A_STAGE_BYTES = 48 * 1024;
    static constexpr bool REGEN_MODE = REGEN;
    static constexpr bool IS_BF16 = BF16;
    static constexpr int RANK_ELEMS_BYTES = RANK * (BF16 ? 2 : 4);
    const Args a;
    // staging slices: bf16 Y block, and (REGEN, bf16) the A_i block kept for the update
    typedef std::conditional_t<LEAN != 0, RowStagerSwz, RowStager2B> stager_t;
    stager_t sty, sta;
    float tc[RANK];
    uint32_t member;
    int64_t ml_member;
    const char* a_tile = nullptr;  // staged A slice: [member - first_member][m - m0][RANK]
    int64_t first_member = 0;
    int tile_m0 = 0, tile_rows = 0;

    // When every column block belongs to one member (S a multiple of CORR_COLS), the rank-r correction of
    // a block is itself a small GEMM, Y[m][n] += sum_l A_i[m][l] * (c t[n][l]), and one more
    // MFMA per block adds it to the accumulators: 16 of its K-slots hold A_i[m][0..r) twice and
    // the fp32 value c*t split into two bf16 halves (hi, then lo = the rounding remainder), so the
    // products stay accurate to about 2^-16.  The epilogue that follows is then the plain store.
    static constexpr int AW = RANK >= 2 ? RANK / 2 : 1;  // 32-bit words of one A_i[m][0..RANK) row in bf16
    // register prefetch (general epilogue); rank 8 would not fit the register budget: it loads late.  The store-only
    // epilogue parks the operands in its LDS slice instead (see prefetch).
    static constexpr bool PREFETCH = RANK <= 4 && LEAN == 0;
    static constexpr int LDS_T = 0, LDS_A = 2048;  // byte offsets of t[64][RANK] fp32 and A_i[128][RANK] bf16 in the slice
    static constexpr int LDS_NB = 3072;            // LEAN_PROJ: the next layer's B'[128][RANK] bf16
    static constexpr bool PROJ = (LEAN & LEAN_PROJ) != 0;
    static_assert(!PROJ || RANK == 1 || RANK == 2 || RANK == 4, "the three runs of 256 RANK bytes fill the wave's 4 KB slice at rank 4");
    // Rank 1: B' of the lane's 4 rows of a row block as two bf16 pairs along the rows -- (r0, r1) and (r2, r3), the packing
    // of the values on their way to the store -- so that a column's share is two packed dot products per row block.
    // Rank 2 and 4 would need 16 RANK registers that way; there the products are formed when the staged rows are read back
    // for the store (flush): a lane then holds 8 consecutive outputs of one row, always the same 8 of the wave tile's 128,
    // and needs B' of those 8 only: bp[l][q] = (B'[8 cc + 2q][l], B'[8 cc + 2q + 1][l]), cc = lane % 16.
    static constexpr bool PROJ_ROWS = PROJ && RANK == 1, PROJ_FLUSH = PROJ && RANK > 1;
    uint32_t nb[PROJ_ROWS ? 8 : 1][2];
    uint32_t bp[PROJ_FLUSH ? RANK : 1][4];
    float tn = 0.f;  // rank 1: the lane's part of t'[n] for the current column
    // Store-only epilogue with residual: the lane's 8 residual pieces (4 bf16 each, one per row block) of the current
    // column block, and those of the next one, on their way while the current block is converted and staged.  Loaded
    // unconditionally from clamped addresses: a predicated load is a branch, and the counted waits behind a branch
    // degrade to "everything outstanding" -- the first version waited out one memory round trip per piece.
    static constexpr bool RESID = LEAN != 0 && (LEAN & LEAN_RESID) != 0;
    // Two sets, used alternately by the column blocks (named at compile time: no copies between them, which the scheduler
    // would be free to hoist, with their wait, to right behind the loads).
    uint2 rres[RESID ? 2 : 1][RESID ? 8 : 1];
    int res_m0 = 0, res_rows = 0;  // first row of the lane's pieces in the wave tile; rows of the output (for the clamp)
    template <int SET>
    __device__ __forceinline__ void load_residual(int n)
    {
        if constexpr (RESID) {
            const uint16_t* rrow = (const uint16_t*)a.resid + (int64_t)min(n, res_rows - 1) * a.d_out;
#pragma unroll
            for (int i = 0; i < 8; ++i) rres[SET][i] = *(const uint2*)(rrow + min(res_m0 + i * BLK, a.d_out - 4));
        }
    }
    // prefetched A rows of the lane, per (row block, group of CORR_COLS columns that share one member), and the
    // prefetched t of the lane's columns, per column block.  With 16x16 blocks a wave tile has twice the row
    // blocks; one member per 64 columns (the width of every wave tile launched here) keeps the register count.
    static constexpr int CORR_COLS = BLK == 32 ? 32 : 64;
    static constexpr int PF_MB = 128 / BLK, PF_NB = 128 / BLK, PF_NG = 128 / CORR_COLS;
    uint32_t pf_a[PREFETCH ? PF_MB : 1][PF_NG][AW];
    float pf_t[PF_NB][RANK];

    template <int NB>
    __device__ __forceinline__ void fetch_t(int nw0, int lane, int n_rows)
    {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int nc = min(nw0 + j * BLK + (lane & (BLK - 1)), n_rows - 1);
#pragma unroll
            for (int l = 0; l < RANK; ++l) pf_t[j][l] = a.t[(int64_t)nc * RANK + l];
        }
    }
    __device__ __forceinline__ void fetch_a(uint32_t (&dst)[AW], int m, int nblock0, int n_rows) const
    {
        const int64_t mlb = (int64_t)(min(nblock0, n_rows - 1) / a.S);  // the block's member (uniform)
        const uint16_t* src = (const uint16_t*)a.A_buf + (mlb * a.d_out + min(m, a.d_out - 1)) * RANK;
        if constexpr (RANK == 1) dst[0] = src[0];
        else if constexpr (RANK == 2) dst[0] = *(const uint32_t*)src;
        else if constexpr (RANK == 4) { const uint2 v = *(const uint2*)src; dst[0] = v.x; dst[1] = v.y; }
        else if constexpr (RANK == 8) { const u32x4 v = *(const u32x4*)src; dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3]; }
    }

    // issued at kernel start: the operands of extra_mma, so that their latency hides under the main loop
    template <int MB, int NB>
    __device__ __forceinline__ void prefetch(int mw0, int nw0, int lane, int n_rows)
    {
        if constexpr (LEAN != 0 && RANK <= 8) {
            // Store-only epilogue: the wave tile (128 rows x 64 columns, one member) needs t[nw0..+64)[0..r) and
            // A_i[mw0..+128)[0..r): two contiguous runs of 256 r bytes, brought into the wave's staging slice by 2 r
            // direct-to-LDS loads of one dword per lane.  No register holds them through the last stage; extra_mma
            // reads its fragments from the slice.  (The slice is idle here: the previous tile's flush is behind us.)
            static_assert(MB * BLK == 128 && NB * BLK == 64 && BLK == 16, "slice layout is that of a 128 x 64 wave tile");
            if (!a.mma_corr || nw0 >= n_rows || mw0 >= a.d_out) return;
            const int64_t member_l = (int64_t)nw0 / a.S;
            const uint32_t* tsrc = (const uint32_t*)(a.t + (int64_t)nw0 * RANK);
            const uint32_t* asrc = (const uint32_t*)((const uint16_t*)a.A_buf + (member_l * a.d_out + mw0) * RANK);
            const int t_last = min(n_rows - nw0, 64) * RANK - 1;           // last valid dword of the t run
            const int a_last = min(a.d_out - mw0, 128) * RANK / 2 - 1;     // of the A run (d_out is a multiple of 4)
#pragma unroll
            for (int k = 0; k < RANK; ++k) {
                __builtin_amdgcn_global_load_lds((egg_glb_void*)(tsrc + min(k * 64 + lane, t_last)),
                                                 (egg_lds_void*)(sty.base + LDS_T + k * 256), 4, 0, 0);
            }
#pragma unroll
            for (int k = 0; k < RANK; ++k) {
                __builtin_amdgcn_global_load_lds((egg_glb_void*)(asrc + min(k * 64 + lane, a_last)),
                                                 (egg_lds_void*)(sty.base + LDS_A + k * 256), 4, 0, 0);
            }
            if constexpr (PROJ) {
                const uint32_t* bsrc = (const uint32_t*)((const uint16_t*)a.next_B + (member_l * a.d_out + mw0) * RANK);
#pragma unroll
                for (int k = 0; k < RANK; ++k) {
                    __builtin_amdgcn_global_load_lds((egg_glb_void*)(bsrc + min(k * 64 + lane, a_last)),
                                                     (egg_lds_void*)(sty.base + LDS_NB + k * 256), 4, 0, 0);
                }
            }
        } else if constexpr (REGEN && BF16) {
            // one row per member, factors regenerated in registers: the projections of the lane's columns are all the
            // epilogue reads; fetched here (clamped, unconditional), they arrive under the last stage instead of one memory
            // round trip per column block
            static_assert(NB <= PF_NB, "prefetch storage");
            if (a.c == 0.f) return;  // unperturbed: there are no projections (t is NULL)
            fetch_t<NB>(nw0, lane, n_rows);
        } else if constexpr (!REGEN && BF16 && PREFETCH) {
            static_assert(MB <= PF_MB && NB <= PF_NB && NB * BLK <= PF_NG * CORR_COLS, "prefetch storage");
            if (!a.mma_corr) return;
            fetch_t<NB>(nw0, lane, n_rows);
#pragma unroll
            for (int g = 0; g < (NB * BLK + CORR_COLS - 1) / CORR_COLS; ++g)
#pragma unroll
                for (int i = 0; i < MB; ++i) fetch_a(pf_a[i][g], mw0 + i * BLK + (lane & (BLK - 1)), nw0 + g * CORR_COLS, n_rows);
        }
    }

    template <class MT, int MB, int NB>
    __device__ __forceinline__ void extra_mma(typename MT::acc_t (&acc)[MB][NB], int mw0, int nw0, int lane, int n_rows)
    {
        if constexpr (RESID) {
            static_assert(MB == 8 && BLK == 16, "eight row blocks of 16 per wave tile");
            res_m0 = mw0 + (lane / BLK) * 4;
            res_rows = n_rows;
            load_residual<0>(nw0 + (lane & (BLK - 1)));  // column block 0; older than the next tile's loads, so a wait for it waits for nothing else
        }
        if constexpr (!REGEN && BF16 && RANK <= 8) {
            if (!a.mma_corr) return;
            if constexpr (LEAN != 0) {
                if (nw0 >= n_rows || mw0 >= a.d_out) return;  // nothing of this wave tile is stored
                if constexpr (PROJ) {
                    // into registers now: the slice becomes the staging area of the stores
                    if constexpr (PROJ_ROWS) {
#pragma unroll
                        for (int i = 0; i < MB; ++i) {
                            const uint2 w = *(const uint2*)(sty.base + LDS_NB + (i * BLK + (lane / BLK) * 4) * 2);
                            nb[i][0] = w.x;
                            nb[i][1] = w.y;
                        }
                    } else {
                        const int cc = lane & 15;
                        const int rows_left = a.d_out - (mw0 + cc * 8);  // rows past d_out hold copies: their factors count as 0
                        const char* br = sty.base + LDS_NB + cc * 8 * RANK * 2;  // 8 rows x RANK bf16, l fastest
                        uint32_t w[4 * RANK];
#pragma unroll
                        for (int k = 0; k < RANK; ++k) {
                            const u32x4 v = *(const u32x4*)(br + 16 * k);
                            w[4 * k] = v[0]; w[4 * k + 1] = v[1]; w[4 * k + 2] = v[2]; w[4 * k + 3] = v[3];
                        }
                        constexpr int WPR = RANK / 2;  // dwords per row
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int lp = 0; lp < WPR; ++lp) {
                                const uint32_t ra = w[(2 * q) * WPR + lp], rb = w[(2 * q + 1) * WPR + lp];  // rows 2q, 2q + 1: (l, l + 1)
                                const bool in = 2 * q < rows_left;
                                bp[2 * lp][q] = in ? ((ra & 0xFFFFu) | (rb << 16)) : 0u;
                                bp[2 * lp + 1][q] = in ? ((ra >> 16) | (rb & 0xFFFF0000u)) : 0u;
                            }
                    }
                }
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int l = 0; l < RANK; ++l) pf_t[j][l] = *(const float*)(sty.base + LDS_T + ((j * BLK + (lane & (BLK - 1))) * RANK + l) * 4);
            } else if constexpr (!PREFETCH) {
                fetch_t<NB>(nw0, lane, n_rows);
            }
            // K-slots 0..7 (hi part of c*t), 8..15 (lo part); the 16x16x32 block has 16 more, left at zero
            const int half = lane / BLK;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                uint32_t tb[4] = {0u, 0u, 0u, 0u};
                float ct[RANK];
#pragma unroll
                for (int l = 0; l < RANK; ++l) {
                    const float v = a.c * pf_t[j][l];
                    const float hi = round_bf16(v);
                    ct[l] = half == 0 ? hi : (half == 1 ? v - hi : 0.f);
                }
#pragma unroll
                for (int l = 0; l < RANK; l += 2) tb[l >> 1] = pack_bf16x2(ct[l], l + 1 < RANK ? ct[l + 1] : 0.f);
                const u32x4 bfrag = {tb[0], tb[1], tb[2], tb[3]};
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    u32x4 afrag = {0u, 0u, 0u, 0u};
                    if constexpr (LEAN != 0) {
                        const char* ar = sty.base + LDS_A + (i * BLK + (lane & (BLK - 1))) * RANK * 2;
                        if constexpr (RANK == 1) afrag[0] = *(const uint16_t*)ar;
                        else
#pragma unroll
                            for (int w = 0; w < AW; ++w) afrag[w] = *(const uint32_t*)(ar + 4 * w);
                    } else if constexpr (PREFETCH) {
#pragma unroll
                        for (int w = 0; w < AW; ++w) afrag[w] = pf_a[i][j * BLK / CORR_COLS][w];
                    } else {
                        uint32_t tmp[AW];
                        fetch_a(tmp, mw0 + i * BLK + (lane & (BLK - 1)), nw0 + j * BLK, n_rows);
#pragma unroll
                        for (int w = 0; w < AW; ++w) afrag[w] = tmp[w];
                    }
                    MT::mma(afrag, bfrag, acc[i][j]);  // rows m >= d_out hold a clamped copy and are never stored
                }
            }
        }
    }

    // Materialised factors: with S rows per member a 256-column tile touches only BN/S + 1 members,
    // so their A_i[m0 .. m0+BM) slices are fetched once, cooperatively and coalesced, instead of by
    // 32 dependent global loads per lane behind live accumulators.
    template <int NT, int BM, int BN>
    __device__ __forceinline__ bool tile_begin(char* lds_tail, int m0, int n0, int tid, int n_rows)
    {
        if constexpr (REGEN || LEAN != 0) {
            return false;
        } else {
            if (!a.stage_a || a.c == 0.f || a.mma_corr) return false;
            constexpr int ESZ = BF16 ? 2 : 4;
            first_member = n0 / a.S;
            const int64_t last_member = (int64_t)(min(n0 + BN, n_rows) - 1) / a.S;
            const int nm = (int)(last_member - first_member) + 1;
            tile_m0 = m0;
            tile_rows = min(BM, a.d_out - m0);               // valid rows of this tile
            const int row_chunks = tile_rows * RANK * ESZ / 16;  // 16-byte chunks per member slice (d_out % 4 == 0)
            constexpr int SLICE_CHUNKS = BM * RANK * ESZ / 16;
            for (int idx = tid; idx < nm * row_chunks; idx += NT) {
                const int ml = idx / row_chunks, ch = idx - ml * row_chunks;
                const u32x4 v = *(const u32x4*)((const char*)a.A_buf + ((first_member + ml) * a.d_out + m0) * (int64_t)(RANK * ESZ) + (int64_t)ch * 16);
                *(u32x4*)(lds_tail + ((int64_t)ml * SLICE_CHUNKS + ch) * 16) = v;
            }
            a_tile = lds_tail;
            bm_rows = BM;
            return true;
        }
    }

    int bm_rows = 0;  // BM of the launched tile (rows per member slice in the staged A)
    __device__ __forceinline__ int tile_stride() const { return bm_rows; }

    // bf16 outputs are staged through LDS; the regenerated bf16 factors too when a cache is kept
    static constexpr __host__ __device__ int lds_per_wave(int wtm) { return (REGEN && BF16 ? 2 : 1) * stager_t::bytes(wtm); }

    __device__ __forceinline__ FwdEpi(const Args& a_, char* slice, int lane)
        : a(a_), sty{slice, lane, lane & (BLK - 1)},
          sta{slice + (LEAN != 0 ? 0 : RowStager2B::bytes((a_.wtm_pitch - 16) / 2)), lane, lane & (BLK - 1)}
    {
    }

    // the persistent kernel names the column block
    template <int J>
    __device__ __forceinline__ void column_at(int n, bool valid)
    {
        if constexpr (REGEN && BF16 && LEAN == 0) {
            static_assert(J < PF_NB, "prefetch storage");
            if (!valid || a.c == 0.f) return;
            ml_member = n / a.S;
            member = a.member_begin + (uint32_t)ml_member;
#pragma unroll
            for (int l = 0; l < RANK; ++l) tc[l] = a.c * pf_t[J][l];  // fetched by prefetch()
        } else {
            column(n, valid);
        }
        if constexpr (RESID) load_residual<(J + 1) & 1>(n + BLK);  // the next column block (past the last one: a clamped re-read that is never used)
    }

    __device__ __forceinline__ void column(int n, bool valid)
    {
        if constexpr (PROJ_ROWS) tn = 0.f;
        if constexpr (LEAN != 0) return;
        if (!valid || a.c == 0.f || (!REGEN && a.mma_corr)) return;
        ml_member = n / a.S;
        member = a.member_begin + (uint32_t)ml_member;
#pragma unroll
        for (int l = 0; l < RANK; ++l) tc[l] = a.c * a.t[(int64_t)n * RANK + l];
    }

    // the persistent kernel names the row block (a compile-time index into per-block registers)
    template <int I, int J = 0>
    __device__ __forceinline__ void store4_at(int m, int n, const float (&v)[4], bool valid, int ml)
    {
        if constexpr (PROJ) {
            float y[4] = {v[0], v[1], v[2], v[3]};
            if constexpr ((LEAN & LEAN_GELU) != 0) gelu_bf16_grade4(y);
            static_assert((LEAN & LEAN_RESID) == 0, "not combined with the residual form");
            const uint32_t p0 = pack_bf16x2(y[0], y[1]), p1 = pack_bf16x2(y[2], y[3]);
            if constexpr (PROJ_ROWS) {
                if (valid && m < a.d_out) {
                    tn = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, p0), __builtin_bit_cast(bf16x2_t, nb[I][0]), tn, false);
                    tn = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, p1), __builtin_bit_cast(bf16x2_t, nb[I][1]), tn, false);
                }
            }
            sty.put(a.wtm_pitch, ml, p0, p1);
        } else if constexpr (RESID) {
            float y[4] = {v[0], v[1], v[2], v[3]};
            if constexpr ((LEAN & LEAN_GELU) != 0) gelu_bf16_grade4(y);
            // each output element is read here and written by flush exactly once, so Y may be the residual buffer itself
            // (rows and columns past the end hold clamped copies and are never stored)
            y[0] += bf16_lo(rres[J & 1][I].x); y[1] += bf16_hi(rres[J & 1][I].x);
            y[2] += bf16_lo(rres[J & 1][I].y); y[3] += bf16_hi(rres[J & 1][I].y);
            sty.put(a.wtm_pitch, ml, pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
        } else {
            store4(m, n, v, valid, ml);
        }
    }

    __device__ __forceinline__ void store4(int m, int n, const float (&v)[4], bool valid, int ml)
    {
        const bool live = valid && m < a.d_out;  // m and d_out are multiples of 4
        float y[4] = {v[0], v[1], v[2], v[3]};
        if constexpr (LEAN != 0) {
            if constexpr ((LEAN & LEAN_GELU) != 0) gelu_bf16_grade4(y);
            if constexpr ((LEAN & LEAN_RESID) != 0) {
                if (live) {
                    const uint2 rv = *(const uint2*)((const uint16_t*)a.resid + (int64_t)n * a.d_out + m);
                    y[0] += bf16_lo(rv.x); y[1] += bf16_hi(rv.x);
                    y[2] += bf16_lo(rv.y); y[3] += bf16_hi(rv.y);
                }
            }
            sty.put(a.wtm_pitch, ml, pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
            return;
        }
        if (live && a.c != 0.f && !(!REGEN && a.mma_corr)) {
            float z[4 * RANK];
            const int64_t aoff = (ml_member * a.d_out + m) * RANK;  // element offset of A_i[m][0]
            if constexpr (REGEN) {
                static_assert(RANK == 1, "in-register regeneration is the rank-1 path");
                const uint32_t blk0 = (uint32_t)m >> 1;
                uint32_t p0 = 0, p1 = 0;  // bf16: the four factors as two packed words
                if (a.pair_share) {
                    // antithetic pairs, one row per member: lanes n and n ^ 1 hold the two rows of one pair and
                    // need the same four factors, so each generates one of the two Threefry blocks and they swap
                    const int b = sty.lane & 1;
                    uint32_t w0, w1;
                    noise_words(a.ka, member, blk0 + b, w0, w1);
                    float o0, o1;
                    normal_pair<!BF16>(w0, w1, o0, o1);
                    if constexpr (BF16) {
                        const uint32_t own = pack_bf16x2(o0, o1), oth = __shfl_xor(own, 1, 64);
                        p0 = b ? oth : own;
                        p1 = b ? own : oth;
                    } else {
                        const float x0 = __shfl_xor(o0, 1, 64), x1 = __shfl_xor(o1, 1, 64);
                        z[0] = b ? x0 : o0; z[1] = b ? x1 : o1;
                        z[2] = b ? o0 : x0; z[3] = b ? o1 : x1;
                    }
                } else {
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        uint32_t w0, w1;
                        noise_words(a.ka, member, blk0 + b, w0, w1);
                        normal_pair<!BF16>(w0, w1, z[2 * b], z[2 * b + 1]);
                    }
                    if constexpr (BF16) {
                        p0 = pack_bf16x2(z[0], z[1]);
                        p1 = pack_bf16x2(z[2], z[3]);
                    }
                }
                if constexpr (BF16) {
                    z[0] = bf16_lo(p0); z[1] = bf16_hi(p0);
                    z[2] = bf16_lo(p1); z[3] = bf16_hi(p1);
                    if (a.A_buf) sta.put(a.wtm_pitch, ml, p0, p1);
                } else {
                    if (a.A_buf) *(float4*)((float*)a.A_buf + aoff) = make_float4(z[0], z[1], z[2], z[3]);
                }
            } else {
                const char* abase = (const char*)a.A_buf + aoff * (BF16 ? 2 : 4);
                if (a_tile) abase = a_tile + (((ml_member - first_member) * (int64_t)tile_stride() + (m - tile_m0)) * RANK) * (BF16 ? 2 : 4);
                if constexpr (BF16) {
                    const uint2* src = (const uint2*)abase;
#pragma unroll
                    for (int v4 = 0; v4 < RANK; ++v4) {
                        const uint2 p = src[v4];
                        z[4 * v4] = bf16_lo(p.x); z[4 * v4 + 1] = bf16_hi(p.x);
                        z[4 * v4 + 2] = bf16_lo(p.y); z[4 * v4 + 3] = bf16_hi(p.y);
                    }
                } else {
                    const float4* src = (const float4*)abase;
#pragma unroll
                    for (int v4 = 0; v4 < RANK; ++v4) {
                        const float4 p = src[v4];
                        z[4 * v4] = p.x; z[4 * v4 + 1] = p.y; z[4 * v4 + 2] = p.z; z[4 * v4 + 3] = p.w;
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float corr = 0.f;
#pragma unroll
                for (int l = 0; l < RANK; ++l) corr = fmaf(tc[l], z[e * RANK + l], corr);
                y[e] += corr;
            }
        }
        if (a.act == EGG_ACT_GELU) {
            if (a.y_bf16) {
                gelu_bf16_grade4(y);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = 0.5f * y[e] * (1.0f + erff(y[e] * 0.70710678118654752f));
            }
        }
        if (a.resid && live) {
            // each output element is read here and written (by flush or below) exactly once, so Y may be the
            // residual buffer itself
            if (a.y_bf16) {
                const uint2 rv = *(const uint2*)((const uint16_t*)a.resid + (int64_t)n * a.d_out + m);
                y[0] += bf16_lo(rv.x); y[1] += bf16_hi(rv.x);
                y[2] += bf16_lo(rv.y); y[3] += bf16_hi(rv.y);
            } else {
                const float4 rv = *(const float4*)((const float*)a.resid + (int64_t)n * a.d_out + m);
                y[0] += rv.x; y[1] += rv.y; y[2] += rv.z; y[3] += rv.w;
            }
        }
        if (a.y_bf16) {
            sty.put(a.wtm_pitch, ml, pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));  // written out by flush
        } else if (live) {
            *(float4*)((float*)a.Y + (int64_t)n * a.d_out + m) = make_float4(y[0], y[1], y[2], y[3]);
        }
    }

    template <int WTM>
    __device__ __forceinline__ void flush(int mw0, int nb0, int n_rows)
    {
        if constexpr (PROJ_FLUSH) {
            // The stager's flush with the projections formed on the way out: the 16 lanes that read one staged row (8 outputs
            // each) multiply them with their B' and add up across the row of lanes.
            static_assert(WTM == 128 && BLK == 16, "16 chunks of 8 outputs per staged row, 4 rows per pass of the wave");
            constexpr int P = stager_t::pitch(WTM);
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes have landed
            __builtin_amdgcn_wave_barrier();
            const int cc = sty.lane & 15;
            const int m = mw0 + cc * 8;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int r = it * 4 + (sty.lane >> 4);
                const int n = nb0 + r;
                const u32x4 v = *(const u32x4*)(sty.base + r * P + (((cc ^ r) & 15) << 4));
                if (n < n_rows && m < a.d_out) {
                    uint16_t* dst = (uint16_t*)a.Y + (int64_t)n * a.d_out + m;
                    if (m + 8 <= a.d_out) *(u32x4*)dst = v;
                    else *(uint2*)dst = make_uint2(v[0], v[1]);
                }
                const uint32_t vw[4] = {v[0], v[1], v[2], v[3]};  // (bit_cast of a vector element, v[q], reads element 0 whatever q is)
                float ts[RANK];
#pragma unroll
                for (int l = 0; l < RANK; ++l) {
                    ts[l] = 0.f;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        ts[l] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, vw[q]), __builtin_bit_cast(bf16x2_t, bp[l][q]), ts[l], false);
                }
#pragma unroll
                for (int l = 0; l < RANK; ++l) ts[l] = row_sum16(ts[l]);
                if (cc == 0 && n < n_rows && mw0 < a.d_out) {
                    float* dst = a.next_part + ((int64_t)(mw0 >> 7) * n_rows + n) * RANK;
                    if constexpr (RANK == 2) *(float2*)dst = make_float2(ts[0], ts[1]);
                    else *(float4*)dst = make_float4(ts[0], ts[1], ts[2], ts[3]);
                }
            }
            __builtin_amdgcn_wave_barrier();  // the slice is reused by the next column block
        } else {
            if (LEAN != 0 || a.y_bf16) sty.template flush<WTM, BLK>((uint16_t*)a.Y, a.d_out, mw0, nb0, n_rows, a.d_out);
        }
        if constexpr (PROJ_ROWS) {
            static_assert(WTM == 128 && BLK == 16, "slabs of 128 rows, four lane groups per column");
            float tsum = tn + __shfl_xor(tn, 16, 64);
            tsum += __shfl_xor(tsum, 32, 64);
            const int n = nb0 + (sty.lane & 15);
            if (sty.lane < 16 && n < n_rows && mw0 < a.d_out) a.next_part[(int64_t)(mw0 >> 7) * n_rows + n] = tsum;
        }
        if constexpr (REGEN && BF16) {
            // REGEN means one row per member, so local member index == row index: same addressing as Y
            if (a.A_buf && a.c != 0.f) sta.template flush<WTM, BLK>((uint16_t*)a.A_buf, a.d_out, mw0, nb0, n_rows, a.d_out);
        }
    }
};

template <class MT, int BM, int BN, int WM, int WN, class Epi>
static egg_status launch_gemm(eggroll_ctx* c, const char* name, const Operand& P, const Operand& Q, int kchunks,
                              typename Epi::Args ea)
{
    ea.wtm_pitch = Epi::stager_t::pitch(BM / WM);
    auto kern = gemm_nt_kernel<MT, BM, BN, WM, WN, false, Epi>;
    const int tiles_m = (P.rows + BM - 1) / BM, tiles_n = (Q.rows + BN - 1) / BN;
    size_t lds = gemm_lds_bytes<BM, BN>();
    size_t epi_lds = (size_t)WM * WN * Epi::lds_per_wave(BM / WM);
    ea.stage_a = 0;
    // (rank <= 8: the 16 K-slots of the extra MFMA hold r factor entries beside the hi and lo halves of c t)
    ea.mma_corr = (!Epi::REGEN_MODE && Epi::IS_BF16 && Epi::RANK_ELEMS_BYTES <= 16 && ea.c != 0.f && ea.S % Epi::CORR_COLS == 0) ? 1 : 0;
    if (!Epi::REGEN_MODE && ea.c != 0.f && !ea.mma_corr) {
        const size_t need = (size_t)(BN / ea.S + 2) * BM * Epi::RANK_ELEMS_BYTES;
        // 16-byte copies: every member slice must start and end on a 16-byte boundary
        if (need <= (size_t)Epi::A_STAGE_BYTES && ((size_t)ea.d_out * Epi::RANK_ELEMS_BYTES) % 16 == 0) {
            ea.stage_a = 1;
            epi_lds += need;
        }
    }
    if (epi_lds > lds) lds = epi_lds;
    if (!operand_offsets_fit(P, BM) || !operand_offsets_fit(Q, BN)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, (size_t)lds, "gemm smem attr");
    if (st != EGG_OK) return st;
    const int64_t grid = (int64_t)tiles_m * tiles_n;
    if (grid > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "too many tiles");
    KernelScope ks(c, shaped_name(c, name, P.rows, kchunks * 16 / (Epi::IS_BF16 ? 2 : 4)));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WM * WN * 64), lds, c->stream, P, Q, kchunks, tiles_m, tiles_n, 0,
                       (const char*)c->zero_page.p, ea);
    return check_hip(c, hipGetLastError(), name);
}

// t[n] = sum over the 128-row slabs of d_out of the partial projections, in slab order (a fixed order: run-to-run identical)
__global__ __launch_bounds__(256) void sum_slabs_kernel(const float* __restrict__ part, int slabs, int64_t R, float* __restrict__ t)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= R) return;
    float acc = 0.f;
    for (int p = 0; p < slabs; ++p) acc += part[(int64_t)p * R + n];
    t[n] = acc;
}

egg_status launch_sum_slabs(eggroll_ctx* c, const float* part, int slabs, int64_t R, float* t)
{
    KernelScope ks(c, "project_sum_slabs");
    hipLaunchKernelGGL(sum_slabs_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, c->stream, part, slabs, R, t);
    return check_hip(c, hipGetLastError(), "project_sum_slabs");
}

bool forward_fuses_next_projection(const egg_shape& s, egg_dtype io, egg_dtype yd, float sigma, egg_act act, bool resid)
{
    const int64_t R = s.member_count * (int64_t)s.rows_per_member;
    const int64_t big_tiles = ((s.d_out + 255) / 256) * ((R + 255) / 256);
    return io == EGG_BF16 && yd == EGG_BF16 && sigma != 0.f && (s.rank == 1 || s.rank == 2 || s.rank == 4) && !s.antithetic && act == EGG_ACT_GELU && !resid &&
           s.rows_per_member % 64 == 0 && s.rows_per_member > 1 && big_tiles >= 192 && s.d_in % 64 == 0;
}

// The persistent kernel for store-only epilogues: one workgroup per compute unit walks the tiles.
template <class MT, int BM, int BN, int WM, int WN, class Epi>
static egg_status launch_gemm_persistent(eggroll_ctx* c, const char* name, const Operand& P, const Operand& Q, int kchunks,
                                         typename Epi::Args ea)
{
    ea.wtm_pitch = Epi::stager_t::pitch(BM / WM);
    auto kern = gemm_nt_persistent_kernel<MT, BM, BN, WM, WN, Epi>;
    const int tiles_m = (P.rows + BM - 1) / BM, tiles_n = (Q.rows + BN - 1) / BN;
    const size_t lds = gemm_lds_bytes<BM, BN>() + (size_t)WM * WN * Epi::lds_per_wave(BM / WM);
    ea.stage_a = 0;
    ea.mma_corr = (Epi::RANK_ELEMS_BYTES <= 16 && ea.c != 0.f && ea.S % Epi::CORR_COLS == 0) ? 1 : 0;
    if (ea.c != 0.f && !ea.mma_corr) return fail(c, EGG_EINVAL, "store-only epilogue launched with a correction left to apply");
    if (!operand_offsets_fit(P, BM) || !operand_offsets_fit(Q, BN)) return fail(c, EGG_EUNSUPPORTED, "operand strides too large for 32-bit tile offsets");
    egg_status st = ensure_dynamic_lds(c, (const void*)kern, lds, "gemm smem attr");
    if (st != EGG_OK) return st;
    const int64_t total = (int64_t)tiles_m * tiles_n;
    if (total > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "too many tiles");
    const unsigned grid = (unsigned)(total < c->compute_units ? total : c->compute_units);
    KernelScope ks(c, shaped_name(c, name, P.rows, kchunks * 8));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds, c->stream, P, Q, kchunks, tiles_m, tiles_n,
                       (const char*)c->zero_page.p, ea);
    return check_hip(c, hipGetLastError(), name);
}

template <bool BF16, int RANK, bool REGEN>
static egg_status launch_forward_t(eggroll_ctx* c, const StreamKey& ka, const egg_shape& s, egg_dtype yd, float sigma,
                                   egg_act act, const void* W, const void* X, void* Y, const float* t, void* A_buf,
                                   const void* resid, const NextProjection* next)
{
    typedef FwdEpi<BF16, RANK, REGEN, BF16 ? 16 : 32> Epi;
    const int esz = BF16 ? 2 : 4;
    const int64_t R = s.member_count * (int64_t)s.rows_per_member;
    // antithetic pairs: the epilogue sees pairs as members of 2S rows (noise id = row / 2S); the sign of
    // the odd member is already folded into its projections t
    const int anti = s.antithetic ? 2 : 1;
    Operand P{(const char*)W, (int64_t)s.d_in * esz, 16, s.d_out};
    Operand Q{(const char*)X, (int64_t)s.d_in * esz, 16, (int)R};
    const int kchunks = s.d_in * esz / 16;
    typename Epi::Args ea{ka, (uint32_t)(s.member_begin / anti), s.rows_per_member * anti, s.d_out, sigma / sqrtf((float)s.rank),
                          (int)act, yd == EGG_BF16 ? 1 : 0, Y, t, A_buf, 0, 0, 0, (REGEN && s.antithetic) ? 1 : 0, resid,
                          nullptr, nullptr};
    if constexpr (BF16) {
        const int64_t big_tiles = ((s.d_out + 255) / 256) * ((R + 255) / 256);
        if (big_tiles >= 192) {
            // bf16 out and nothing left to correct in the epilogue (unperturbed, or the correction folds into the
            // accumulators): the store-only epilogue with the activation and the residual fixed at compile time
            const bool folded = !REGEN && Epi::RANK_ELEMS_BYTES <= 16 && ea.c != 0.f && ea.S % Epi::CORR_COLS == 0;
            if (next) {
                // the fused next-layer projection exists in one form: rank 1, 2 or 4 (the next layer's too), folded correction,
                // GELU, no residual
                if constexpr (!REGEN && (RANK == 1 || RANK == 2 || RANK == 4)) {
                    if (forward_fuses_next_projection(s, EGG_BF16, yd, sigma, act, resid != nullptr)) {
                        const int slabs = (s.d_out + 127) / 128;
                        egg_status st = reserve(c, c->proj_part, (size_t)slabs * R * RANK * sizeof(float));
                        if (st != EGG_OK) return st;
                        ea.next_B = next->B;
                        ea.next_part = (float*)c->proj_part.p;
                        st = launch_gemm_persistent<MmaBf16Blk16, 256, 256, 2, 4, FwdEpi<true, RANK, false, 16, LEAN_ON | LEAN_GELU | LEAN_PROJ>>(
                            c, "forward_gemm_bf16", P, Q, kchunks, ea);
                        if (st != EGG_OK) return st;
                        return launch_sum_slabs(c, (const float*)c->proj_part.p, slabs, R * RANK, next->t);
                    }
                }
                return fail(c, EGG_EINVAL, "this layer cannot form the next layer's projections (ask forward_fuses_next_projection first)");
            }
            if (yd == EGG_BF16 && (ea.c == 0.f || folded) && kchunks % 8 == 0) {
                constexpr int LR = (REGEN || RANK > 8) ? 1 : RANK;
#define EGG_LEAN(L) \
    return launch_gemm_persistent<MmaBf16Blk16, 256, 256, 2, 4, FwdEpi<true, LR, false, 16, L>>(c, "forward_gemm_bf16", P, Q, kchunks, ea)
                switch ((act == EGG_ACT_GELU ? LEAN_GELU : 0) | (resid ? LEAN_RESID : 0)) {
                    case 0: EGG_LEAN(LEAN_ON);
                    case LEAN_GELU: EGG_LEAN(LEAN_ON | LEAN_GELU);
                    case LEAN_RESID: EGG_LEAN(LEAN_ON | LEAN_RESID);
                    default: EGG_LEAN(LEAN_ON | LEAN_GELU | LEAN_RESID);
                }
#undef EGG_LEAN
            }
            return launch_gemm<MmaBf16Blk16, 256, 256, 2, 4, Epi>(c, "forward_gemm_bf16", P, Q, kchunks, ea);
        }
        if (next) return fail(c, EGG_EINVAL, "this layer cannot form the next layer's projections (ask forward_fuses_next_projection first)");
        // few rows against a large layer (the paper's own benchmark shape, batch 1024 on 8192 x 8192): tall
        // tiles keep one workgroup per CU busy where 256 x 256 tiles would leave half the chip idle
        const int64_t tall_tiles = ((s.d_out + 255) / 256) * ((R + 127) / 128);
        if (tall_tiles >= 192) {
            return launch_gemm<MmaBf16Blk16, 256, 128, 4, 2, Epi>(c, "forward_gemm_bf16_tall", P, Q, kchunks, ea);
        }
        return launch_gemm<MmaBf16Blk16, 128, 128, 2, 2, Epi>(c, "forward_gemm_bf16_small", P, Q, kchunks, ea);
    } else {
        if (next) return fail(c, EGG_EINVAL, "this layer cannot form the next layer's projections (ask forward_fuses_next_projection first)");
        return launch_gemm<MmaF32, 128, 128, 2, 2, Epi>(c, "forward_gemm_f32", P, Q, kchunks, ea);
    }
}

egg_status launch_forward_gemm(eggroll_ctx* c, const StreamKey& ka, const egg_shape& s, egg_dtype io, egg_dtype yd,
                               float sigma, egg_act act, const void* W, const void* X, void* Y, const float* t,
                               void* A_cache, const void* resid, const NextProjection* next)
{
    const bool bf = io == EGG_BF16;
    // rank 1 with one row per member (or the unperturbed pass): regenerate in the epilogue
    // (with antithetic pairs a kept cache has one entry per pair, not per row: that goes the materialised way)
    if (sigma == 0.f || (s.rank == 1 && s.rows_per_member == 1 && !(s.antithetic && A_cache))) {
        return bf ? launch_forward_t<true, 1, true>(c, ka, s, yd, sigma, act, W, X, Y, t, A_cache, resid, next)
                  : launch_forward_t<false, 1, true>(c, ka, s, yd, sigma, act, W, X, Y, t, A_cache, resid, next);
    }
    // otherwise materialise A once (into the caller's cache if there is one) and read it back
    void* A_buf = A_cache;
    const int anti = s.antithetic ? 2 : 1;  // one set of factors per pair
    if (!A_buf) {
        const size_t bytes = (size_t)(s.member_count / anti) * s.d_out * s.rank * (bf ? 2 : 4);
        egg_status st = reserve(c, c->a_buf, bytes);
        if (st != EGG_OK) return st;
        A_buf = c->a_buf.p;
    }
    egg_status st = launch_noise(c, ka, (uint32_t)(s.member_begin / anti), s.member_count / anti, (int64_t)s.d_out * s.rank, io,
                                 EGG_NORMAL, 0, A_buf);
    if (st != EGG_OK) return st;
#define EGG_FWD(B, R) return launch_forward_t<B, R, false>(c, ka, s, yd, sigma, act, W, X, Y, t, A_buf, resid, next)
    if (bf) {
        switch (s.rank) {
            case 1: EGG_FWD(true, 1);
            case 2: EGG_FWD(true, 2);
            case 4: EGG_FWD(true, 4);
            case 8: EGG_FWD(true, 8);
            default: EGG_FWD(true, 16);
        }
    } else {
        switch (s.rank) {
            case 1: EGG_FWD(false, 1);
            case 2: EGG_FWD(false, 2);
            case 4: EGG_FWD(false, 4);
            case 8: EGG_FWD(false, 8);
            default: EGG_FWD(false, 16);
        }
    }
#undef EGG_FWD
}

}  // namespace egg

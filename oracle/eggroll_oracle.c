/*
 * EGGROLL CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of what the GPU hot path computes, written from
 * the paper's statement of the method ("Evolution Strategies at the Hyperscale", EGGROLL):
 *
 *   - noise:   A_i in R^{d_out x r}, B_i in R^{d_in x r} as a pure function of
 *              (seed, step, layer, which, member, flat index)   [Sec. 1 "counter-based deterministic
 *              RNG ... reconstruct noise on demand"; Alg. 1 "reconstruct E_j from seeds"]
 *   - forward: for every member i, materialise W_i = M + (sigma/sqrt(r)) A_i B_i^T as a dense fp64
 *              matrix and multiply                               [Alg. 1 line f_i <- f(W = M + sigma E_i),
 *              E_i = A_i B_i^T / sqrt(r); Sec. 4.1]
 *   - update:  G = scale * sum_i f_i A_i B_i^T as N*r explicit outer products in fp64
 *              [EGGROLL UPDATE box, Eq. (eggroll_update); the 1/(sigma N) constant of Eq. (matrix_mc)]
 *   - int8:    the integer perturbed matmul step by step        [App. "Adding EGGROLL Perturbations"]
 *
 * It deliberately does NOT use the factored form u M^T + (sigma/sqrt r)(u B)A^T or the
 * (diag(f)A)^T B contraction of Sec. 4.2: those are what the GPU path uses, and the tests check
 * that the two agree.  Nothing here is shared with the HIP sources (no common header, table or
 * helper).  Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 *
 * Pins (tests/test_oracle_*.py): the Threefry block function against rocRAND's host-callable
 * Threefry-2x32-20 engine; the normal transform against N(0,1) moments / KS and the K_0 product density of the
 * mean-field appendix; the integer map exhaustively; forward/update against brute-force numpy,
 * closed forms and the identities of Sec. 4.2.  Parity against the authors' own JAX noise stream
 * is unpinned: the paper does not publish its stream and it need not be matched.  Parity unpinned as well:
 * the rounding mode of the EXP2 / LOG2 table entries of oracle_loglik_i8 (see there).
 *
 * Build: gcc -O2 -fopenmp -fPIC -shared -o liboracle.so eggroll_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------------------------ */
/* Threefry-2x32, 20 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as  */
/* 1, 2, 3", SC'11) -- the counter-based generator the paper cites for noise reconstruction    */
/* (it is the block function of the JAX PRNG the paper's code base uses).                      */
/* ------------------------------------------------------------------------------------------ */

static uint32_t rotl32(uint32_t v, unsigned s) { return (v << s) | (v >> (32u - s)); }

/* rotation amounts of Threefry-2x32, indexed by round mod 8 */
static const unsigned TF_ROT[8] = {13, 15, 26, 6, 17, 29, 16, 24};

void oracle_threefry2x32_20(const uint32_t ctr[2], const uint32_t key[2], uint32_t out[2])
{
    uint32_t ks[3];
    ks[0] = key[0];
    ks[1] = key[1];
    ks[2] = 0x1BD11BDAu ^ key[0] ^ key[1]; /* Threefish key-schedule parity word, 32-bit form */
    uint32_t x0 = ctr[0] + ks[0];
    uint32_t x1 = ctr[1] + ks[1];
    for (int round = 0; round < 20; ++round) {
        x0 += x1;
        x1 = rotl32(x1, TF_ROT[round % 8]);
        x1 ^= x0;
        if ((round & 3) == 3) { /* key injection after every fourth round */
            const uint32_t s = (uint32_t)(round / 4 + 1);
            x0 += ks[s % 3u];
            x1 += ks[(s + 1u) % 3u] + s;
        }
    }
    out[0] = x0;
    out[1] = x1;
}

/*
 * Stream addressing (this build's contract; the paper only requires "known random seeds").
 *   stream key  = Threefry(key = (seed low 32, seed high 32), counter = (step, layer | which<<31))
 *                 which: A = 0, B = 1; layer < 2^31
 *   block b of member i = Threefry(key = stream key, counter = (b, i)),  0 <= i < 2^32
 * One block yields output words 2b and 2b+1 of that member's vector.
 */
static void stream_key(uint64_t seed, uint32_t step, uint32_t layer, int which, uint32_t out[2])
{
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const uint32_t ctr[2] = {step, (layer & 0x7FFFFFFFu) | ((uint32_t)(which & 1) << 31)};
    oracle_threefry2x32_20(ctr, key, out);
}

static void noise_block(uint64_t seed, uint32_t step, uint32_t layer, int which, int64_t member,
                        uint32_t block, uint32_t out[2])
{
    uint32_t sk[2];
    stream_key(seed, step, layer, which, sk);
    const uint32_t ctr[2] = {block, (uint32_t)((uint64_t)member)};
    oracle_threefry2x32_20(ctr, sk, out);
}

void oracle_stream_key(uint64_t seed, uint32_t step, uint32_t layer, int which, uint32_t out[2])
{
    stream_key(seed, step, layer, which, out);
}

/* raw words first_word .. first_word+n-1 of one member's stream */
void oracle_raw_words(uint64_t seed, uint32_t step, uint32_t layer, int which, int64_t member,
                      uint64_t first_word, uint64_t n, uint32_t* out)
{
    for (uint64_t w = 0; w < n; ++w) {
        const uint64_t word = first_word + w;
        uint32_t blk[2];
        noise_block(seed, step, layer, which, member, (uint32_t)(word >> 1), blk);
        out[w] = blk[word & 1u];
    }
}

/*
 * Standard normals, one 32-bit word per value.  The paper leaves the transform open (Assumption 1
 * asks only for iid, zero-mean, symmetric, unit-variance entries; the configs ask for Gaussians).
 * Reading used here: the top 23 bits of a word give u = (k + 1/2) 2^-23 in (0,1); words (2p, 2p+1)
 * form a Box-Muller pair: rho = sqrt(-2 ln u1); z_2p = rho cos(2 pi u2), z_2p+1 = rho sin(2 pi u2).
 * Value with flat index n (= d*rank + l) is z_n.  Evaluated in fp64.
 */
static double word_to_unit(uint32_t w) { return ((double)(w >> 9) + 0.5) * (1.0 / 8388608.0); }

void oracle_noise_normal(uint64_t seed, uint32_t step, uint32_t layer, int which, int64_t member,
                         uint64_t first, uint64_t n, double* out)
{
    static const double TWO_PI = 6.283185307179586476925286766559;
    for (uint64_t v = 0; v < n; ++v) {
        const uint64_t idx = first + v;
        uint32_t blk[2];
        noise_block(seed, step, layer, which, member, (uint32_t)(idx >> 1), blk);
        const double u1 = word_to_unit(blk[0]);
        const double u2 = word_to_unit(blk[1]);
        const double rho = sqrt(-2.0 * log(u1));
        out[v] = (idx & 1u) ? rho * sin(TWO_PI * u2) : rho * cos(TWO_PI * u2);
    }
}

/*
 * Bounded integers on {-b..b} from the BYTES of the same stream: value n uses word n>>2, byte n&3
 * (little end first).  With m = 2b+1 and q = floor(256/m): byte < q*m -> floor(byte/q) - b, else 0.
 * Exactly symmetric and zero-mean (Assumption 1), no floating point (App. "Adding EGGROLL
 * Perturbations" keeps float arithmetic off the accelerator).  b = 0 gives all zeros.
 */
int oracle_int_from_byte(unsigned byte, int bound)
{
    const int m = 2 * bound + 1;
    const int q = 256 / m;
    return ((int)byte < q * m) ? (int)byte / q - bound : 0;
}

/*
 * The paper's own integer noise (App. "Adding EGGROLL Perturbations": "a pre-generated table of int8 normals
 * [round(16 N(0,1))] randomly indexed", so that no floating point runs on the accelerator).  The paper does not
 * give the table; reading: 2^16 entries, entry k the value at the midpoint of the k-th of 65536 equal-probability
 * cells of N(0,1), T[k] = round(16 Phi^-1((k + 1/2)/65536)), half away from zero, clipped to 127 (never reached:
 * the largest magnitude is 69).  Phi^-1 by bisection on Phi(x) = erfc(-x / sqrt 2) / 2.  Indexed by the 16-bit
 * halves of the stream's words: value n uses half n & 1 (low half first) of word n >> 1.  Selected by bound = -16.
 */
#define ORACLE_BOUND_NORMAL16 (-16)

static double normal_cdf(double x) { return 0.5 * erfc(-x * 0.70710678118654752440); }

void oracle_normal_int_table(int8_t* out)
{
    for (int k = 0; k < 65536; ++k) {
        const double p = ((double)k + 0.5) / 65536.0;
        double lo = -10.0, hi = 10.0;
        for (int it = 0; it < 200; ++it) { /* Phi is increasing: keep Phi(lo) <= p <= Phi(hi) */
            const double mid = 0.5 * (lo + hi);
            if (normal_cdf(mid) < p) lo = mid; else hi = mid;
        }
        const double z16 = 16.0 * 0.5 * (lo + hi);
        double v = z16 >= 0.0 ? floor(z16 + 0.5) : -floor(-z16 + 0.5); /* half away from zero */
        if (v > 127.0) v = 127.0;
        if (v < -127.0) v = -127.0;
        out[k] = (int8_t)v;
    }
}

static const int8_t* normal_int_table_once(void)
{
    static int8_t table[65536];
    static int ready = 0;
#pragma omp critical(oracle_normal_table)
    {
        if (!ready) {
            oracle_normal_int_table(table);
            ready = 1;
        }
    }
    return table;
}

void oracle_noise_int(uint64_t seed, uint32_t step, uint32_t layer, int which, int64_t member,
                      uint64_t first, uint64_t n, int bound, int8_t* out)
{
    if (bound == ORACLE_BOUND_NORMAL16) {
        const int8_t* table = normal_int_table_once();
        for (uint64_t v = 0; v < n; ++v) {
            const uint64_t idx = first + v;
            uint32_t blk[2];
            noise_block(seed, step, layer, which, member, (uint32_t)(idx >> 2), blk);
            const uint32_t word = blk[(idx >> 1) & 1u];
            out[v] = table[(word >> (16u * (unsigned)(idx & 1u))) & 0xFFFFu];
        }
        return;
    }
    for (uint64_t v = 0; v < n; ++v) {
        const uint64_t idx = first + v;
        uint32_t blk[2];
        noise_block(seed, step, layer, which, member, (uint32_t)(idx >> 3), blk);
        const uint32_t word = blk[(idx >> 2) & 1u];
        out[v] = (int8_t)oracle_int_from_byte((word >> (8u * (unsigned)(idx & 3u))) & 0xFFu, bound);
    }
}

/* ------------------------------------------------------------------------------------------ */
/* storage roundings (round-to-nearest-even), so the oracle sees exactly the values the method */
/* stores: fp32 noise in fp32 mode; fp32 then bfloat16 in bf16 mode.                            */
/* ------------------------------------------------------------------------------------------ */
double oracle_round_f32(double v) { return (double)(float)v; }

double oracle_round_bf16(double v)
{
    float f = (float)v;
    uint32_t bits;
    memcpy(&bits, &f, 4);
    if ((bits & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan pass through */
    const uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7FFFu + lsb;
    bits &= 0xFFFF0000u;
    memcpy(&f, &bits, 4);
    return (double)f;
}

static double round_storage(double v, int noise_dtype) /* 0 = fp32, 1 = bf16 */
{
    return noise_dtype == 1 ? oracle_round_bf16(v) : oracle_round_f32(v);
}

/* A_i (which = 0, d = d_out) or B_i (which = 1, d = d_in) as stored: out[d*rank], index d*rank+l */
void oracle_noise_matrix(uint64_t seed, uint32_t step, uint32_t layer, int which, int64_t member,
                         int64_t d, int rank, int noise_dtype, double* out)
{
    const uint64_t n = (uint64_t)d * (uint64_t)rank;
    oracle_noise_normal(seed, step, layer, which, member, 0, n, out);
    for (uint64_t v = 0; v < n; ++v) out[v] = round_storage(out[v], noise_dtype);
}

/*
 * Random access into the factors of many members at once: out[m][q] = storage-rounded entry idx[q] of the
 * vector of member member_begin + m (which = 0: A, flat index j*rank + l; which = 1: B).  Used by sampled
 * checks of the update at sizes where no whole factor matrix can be drawn per member.
 */
void oracle_noise_gather(uint64_t seed, uint32_t step, uint32_t layer, int which, int64_t member_begin,
                         int64_t member_count, const int64_t* idx, int64_t n_idx, int noise_dtype, double* out)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < member_count; ++m) {
        for (int64_t q = 0; q < n_idx; ++q) {
            double v;
            oracle_noise_normal(seed, step, layer, which, member_begin + m, (uint64_t)idx[q], 1, &v);
            out[(size_t)m * (size_t)n_idx + (size_t)q] = round_storage(v, noise_dtype);
        }
    }
}

/* ------------------------------------------------------------------------------------------ */
/* forward: explicit W_i per member                                                            */
/* ------------------------------------------------------------------------------------------ */
static double gelu_exact(double x) { return 0.5 * x * (1.0 + erf(x * 0.70710678118654752440)); }

/*
 * Y[row, j] = act( sum_k W_i[j,k] X[row,k] ),  W_i = W + (sigma/sqrt(rank)) A_i B_i^T,
 * rows of X are member-major: member(row) = member_begin + row / S.
 * W[d_out*d_in], X[count*S*d_in], Y[count*S*d_out] all fp64 holding storage-dtype values.
 * Returns 0, or -1 if memory for the per-thread W_i could not be obtained.
 */
static int forward_worker(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                          int64_t member_count, int S, int d_out, int d_in, int rank, int noise_dtype,
                          double sigma, int act, int antithetic, const double* W, const double* X, double* Y)
{
    const double c0 = sigma / sqrt((double)rank);
    int failed = 0;
#pragma omp parallel
    {
        double* Wi = (double*)malloc(sizeof(double) * (size_t)d_out * (size_t)d_in);
        double* A = (double*)malloc(sizeof(double) * (size_t)d_out * (size_t)rank);
        double* B = (double*)malloc(sizeof(double) * (size_t)d_in * (size_t)rank);
        if (!Wi || !A || !B) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t m = 0; m < member_count; ++m) {
                const int64_t member = member_begin + m;
                /* antithetic: members 2p and 2p+1 evaluate M + sigma E_p and M - sigma E_p */
                const int64_t noise_id = antithetic ? member / 2 : member;
                const double c = (antithetic && (member & 1)) ? -c0 : c0;
                oracle_noise_matrix(seed, step, layer, 0, noise_id, d_out, rank, noise_dtype, A);
                oracle_noise_matrix(seed, step, layer, 1, noise_id, d_in, rank, noise_dtype, B);
                for (int j = 0; j < d_out; ++j) {
                    for (int k = 0; k < d_in; ++k) {
                        double e = 0.0;
                        for (int l = 0; l < rank; ++l)
                            e += A[(size_t)j * rank + l] * B[(size_t)k * rank + l];
                        Wi[(size_t)j * d_in + k] = W[(size_t)j * d_in + k] + c * e;
                    }
                }
                for (int s = 0; s < S; ++s) {
                    const double* x = X + ((size_t)m * S + s) * (size_t)d_in;
                    double* y = Y + ((size_t)m * S + s) * (size_t)d_out;
                    for (int j = 0; j < d_out; ++j) {
                        double acc = 0.0;
                        const double* w = Wi + (size_t)j * d_in;
                        for (int k = 0; k < d_in; ++k) acc += w[k] * x[k];
                        y[j] = act == 1 ? gelu_exact(acc) : acc;
                    }
                }
            }
        }
        free(Wi); free(A); free(B);
    }
    return failed ? -1 : 0;
}

int oracle_forward(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                   int64_t member_count, int S, int d_out, int d_in, int rank, int noise_dtype,
                   double sigma, int act, const double* W, const double* X, double* Y)
{
    return forward_worker(seed, step, layer, member_begin, member_count, S, d_out, d_in, rank, noise_dtype,
                          sigma, act, 0, W, X, Y);
}

/*
 * Antithetic pairs (used by the paper's integer and quantised experiments: App. "Fitness Shaping",
 * "antithetical pair"): member ids 2p and 2p+1 share the factors of pair p (noise id p) and are
 * evaluated at W = M + sigma E_p and W = M - sigma E_p.  member_begin counts members, not pairs.
 */
int oracle_forward_antithetic(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                              int64_t member_count, int S, int d_out, int d_in, int rank, int noise_dtype,
                              double sigma, int act, const double* W, const double* X, double* Y)
{
    return forward_worker(seed, step, layer, member_begin, member_count, S, d_out, d_in, rank, noise_dtype,
                          sigma, act, 1, W, X, Y);
}

/* ------------------------------------------------------------------------------------------ */
/* update: explicit sum of N*r outer products                                                  */
/* ------------------------------------------------------------------------------------------ */
/*
 * G[j,k] = scale * sum_i fitness[i] * sum_l A_i[j,l] B_i[k,l]      (members member_begin .. +count)
 * Row blocks of G are owned by threads; every thread walks the members in increasing order, so
 * the summation order of each entry is fixed.
 */
int oracle_update(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                  int64_t member_count, int d_out, int d_in, int rank, int noise_dtype,
                  const double* fitness, double scale, double* G)
{
    /* materialise all factors once (N*(d_out+d_in)*r doubles) */
    const size_t na = (size_t)d_out * rank, nb = (size_t)d_in * rank;
    double* A = (double*)malloc(sizeof(double) * na * (size_t)member_count);
    double* B = (double*)malloc(sizeof(double) * nb * (size_t)member_count);
    if (!A || !B) { free(A); free(B); return -1; }
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < member_count; ++m) {
        oracle_noise_matrix(seed, step, layer, 0, member_begin + m, d_out, rank, noise_dtype, A + na * (size_t)m);
        oracle_noise_matrix(seed, step, layer, 1, member_begin + m, d_in, rank, noise_dtype, B + nb * (size_t)m);
    }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < d_out; ++j) {
        double* g = G + (size_t)j * d_in;
        for (int k = 0; k < d_in; ++k) g[k] = 0.0;
        for (int64_t m = 0; m < member_count; ++m) {
            const double* a = A + na * (size_t)m + (size_t)j * rank;
            const double* b = B + nb * (size_t)m;
            for (int l = 0; l < rank; ++l) {
                const double fa = fitness[m] * a[l];
                for (int k = 0; k < d_in; ++k) g[k] += fa * b[(size_t)k * rank + l];
            }
        }
        for (int k = 0; k < d_in; ++k) g[k] *= scale;
    }
    free(A); free(B);
    return 0;
}

/* one entry of G, by random access into the noise stream (for sampled checks at full size) */
double oracle_update_entry(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                           int64_t member_count, int rank, int noise_dtype, const double* fitness,
                           double scale, int64_t j, int64_t k)
{
    double acc = 0.0;
    double a[8], b[8];
    for (int64_t m = 0; m < member_count; ++m) {
        oracle_noise_normal(seed, step, layer, 0, member_begin + m, (uint64_t)j * rank, (uint64_t)rank, a);
        oracle_noise_normal(seed, step, layer, 1, member_begin + m, (uint64_t)k * rank, (uint64_t)rank, b);
        double e = 0.0;
        for (int l = 0; l < rank; ++l) e += round_storage(a[l], noise_dtype) * round_storage(b[l], noise_dtype);
        acc += fitness[m] * e;
    }
    return scale * acc;
}

/* ------------------------------------------------------------------------------------------ */
/* integer perturbed matmul, repeated as a recurrence                                          */
/* ------------------------------------------------------------------------------------------ */
static int32_t shr_floor(int64_t v, int s) /* arithmetic shift: floor(v / 2^s) */
{
    if (s <= 0) return (int32_t)v;
    return (int32_t)(v >= 0 ? (v >> s) : -((-v + ((int64_t)1 << s) - 1) >> s));
}

/*
 * For each member row h (int8[d]) and `steps` times:
 *     acc_j  = sum_k h_k W[j,k]                     (int32)
 *     dot    = sum_k h_k B_i[k]                     (int32)            "u . B"
 *     corr_j = (dot * int32(A_i[j])) >> corr_shift  (arithmetic)       "(u.B) I32(A) >> (4+sigma_hat)"
 *     h'_j   = clamp((acc_j + corr_j) >> out_shift, -127, 127)         "I8(. / (16 sqrt n))"
 * rank 1, square W (d x d), noise on {-bound..bound}.  H_in/H_out: [count][d].
 */
static void forward_i8_worker(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                              int64_t member_count, int d_out, int d_in, int bound, int corr_shift, int out_shift,
                              int steps, int antithetic, const int8_t* W, const int8_t* H_in, int8_t* H_out)
{
    /* theta is d_out x d_in ("m x n"); more than one step feeds h' back in and needs d_out == d_in */
    const int dmax = d_out > d_in ? d_out : d_in;
#pragma omp parallel
    {
        int8_t* A = (int8_t*)malloc((size_t)d_out);
        int8_t* B = (int8_t*)malloc((size_t)d_in);
        int32_t* h = (int32_t*)malloc(sizeof(int32_t) * (size_t)dmax);
        int32_t* hn = (int32_t*)malloc(sizeof(int32_t) * (size_t)dmax);
#pragma omp for schedule(dynamic, 4)
        for (int64_t m = 0; m < member_count; ++m) {
            const int64_t member = member_begin + m;
            const int64_t noise_id = antithetic ? member / 2 : member;
            oracle_noise_int(seed, step, layer, 0, noise_id, 0, (uint64_t)d_out, bound, A);
            oracle_noise_int(seed, step, layer, 1, noise_id, 0, (uint64_t)d_in, bound, B);
            /* the negative member of a pair carries the perturbation A (-B)^T: one formula for both signs */
            if (antithetic && (member & 1))
                for (int k = 0; k < d_in; ++k) B[k] = (int8_t)(-B[k]);
            for (int k = 0; k < d_in; ++k) h[k] = H_in[(size_t)m * d_in + k];
            for (int t = 0; t < steps; ++t) {
                int32_t dot = 0;
                for (int k = 0; k < d_in; ++k) dot += h[k] * (int32_t)B[k];
                for (int j = 0; j < d_out; ++j) {
                    int32_t acc = 0;
                    const int8_t* w = W + (size_t)j * d_in;
                    for (int k = 0; k < d_in; ++k) acc += h[k] * (int32_t)w[k];
                    const int32_t corr = shr_floor((int64_t)dot * (int64_t)A[j], corr_shift);
                    int32_t v = shr_floor((int64_t)acc + (int64_t)corr, out_shift);
                    if (v > 127) v = 127;
                    if (v < -127) v = -127;
                    hn[j] = v;
                }
                for (int k = 0; k < d_out; ++k) h[k] = hn[k];
            }
            for (int k = 0; k < d_out; ++k) H_out[(size_t)m * d_out + k] = (int8_t)h[k];
        }
        free(A); free(B); free(h); free(hn);
    }
}

void oracle_forward_i8(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                       int64_t member_count, int d, int bound, int corr_shift, int out_shift,
                       int steps, const int8_t* W, const int8_t* H_in, int8_t* H_out)
{
    forward_i8_worker(seed, step, layer, member_begin, member_count, d, d, bound, corr_shift, out_shift, steps, 0,
                      W, H_in, H_out);
}

/* antithetic pairs in the integer model: members 2p, 2p+1 share noise id p; the odd one uses -B_p */
void oracle_forward_i8_antithetic(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                                  int64_t member_count, int d, int bound, int corr_shift, int out_shift,
                                  int steps, const int8_t* W, const int8_t* H_in, int8_t* H_out)
{
    forward_i8_worker(seed, step, layer, member_begin, member_count, d, d, bound, corr_shift, out_shift, steps, 1,
                      W, H_in, H_out);
}

/* one application of a rectangular theta (d_out x d_in), e.g. the 4D x D and D x 4D matrices of the integer MLP */
void oracle_matmul_i8(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin, int64_t member_count,
                      int d_out, int d_in, int bound, int corr_shift, int out_shift, int antithetic,
                      const int8_t* W, const int8_t* H_in, int8_t* H_out)
{
    forward_i8_worker(seed, step, layer, member_begin, member_count, d_out, d_in, bound, corr_shift, out_shift, 1,
                      antithetic, W, H_in, H_out);
}

/* ------------------------------------------------------------------------------------------ */
/* integer GRU cell (App. "GRU" of the EGG architecture), one time step for a population       */
/* ------------------------------------------------------------------------------------------ */
static int32_t sat127(int64_t v) { return (int32_t)(v > 127 ? 127 : (v < -127 ? -127 : v)); }

/*
 *   f     = I8( I32(u @ Wf^T) + I32(s @ Uf^T) + I32(bf) )                 sigma = identity
 *   f^    = I8( ((I32(f) + 127) * I32(s)) >> 8 )
 *   h^    = I8( I32(u @ Wh^T) + I32(f^ @ Uh^T) + I32(bh) )                phi = identity
 *   h     = s + I8( ((I32(f) + 127) * (I32(h^) - I32(s))) >> 8 )
 * "@" is the perturbed scaled matmul of forward_i8_worker (one application, square D x D); the four
 * matrices are perturbed independently: Wf, Uf, Wh, Uh use noise layers layer, layer+1, layer+2, layer+3.
 * I8 clips to [-127, 127]; shifts are arithmetic.  Reading: the final sum s + I8(.) is clipped to
 * [-127, 127] as well (h is the next state, an I8 vector).  U, S, H: [count][D].
 */
void oracle_gru_step_i8(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin, int64_t member_count,
                        int D, int bound, int corr_shift, int out_shift, int antithetic,
                        const int8_t* Wf, const int8_t* Uf, const int8_t* Wh, const int8_t* Uh,
                        const int8_t* bf, const int8_t* bh, const int8_t* U, const int8_t* S, int8_t* H)
{
    const size_t n = (size_t)member_count * (size_t)D;
    int8_t* a1 = (int8_t*)malloc(n); int8_t* a2 = (int8_t*)malloc(n);
    int8_t* a3 = (int8_t*)malloc(n); int8_t* a4 = (int8_t*)malloc(n);
    int8_t* f = (int8_t*)malloc(n); int8_t* fh = (int8_t*)malloc(n);
    forward_i8_worker(seed, step, layer + 0, member_begin, member_count, D, D, bound, corr_shift, out_shift, 1, antithetic, Wf, U, a1);
    forward_i8_worker(seed, step, layer + 1, member_begin, member_count, D, D, bound, corr_shift, out_shift, 1, antithetic, Uf, S, a2);
    for (size_t i = 0; i < n; ++i) {
        const int j = (int)(i % (size_t)D);
        f[i] = (int8_t)sat127((int64_t)a1[i] + a2[i] + bf[j]);
        fh[i] = (int8_t)sat127(shr_floor(((int64_t)f[i] + 127) * (int64_t)S[i], 8));
    }
    forward_i8_worker(seed, step, layer + 2, member_begin, member_count, D, D, bound, corr_shift, out_shift, 1, antithetic, Wh, U, a3);
    forward_i8_worker(seed, step, layer + 3, member_begin, member_count, D, D, bound, corr_shift, out_shift, 1, antithetic, Uh, fh, a4);
    for (size_t i = 0; i < n; ++i) {
        const int j = (int)(i % (size_t)D);
        const int32_t hh = sat127((int64_t)a3[i] + a4[i] + bh[j]);
        const int32_t delta = sat127(shr_floor(((int64_t)f[i] + 127) * ((int64_t)hh - (int64_t)S[i]), 8));
        H[i] = (int8_t)sat127((int64_t)S[i] + delta);
    }
    free(a1); free(a2); free(a3); free(a4); free(f); free(fh);
}

/* ------------------------------------------------------------------------------------------ */
/* integer parameter update (App. "Parameter Update" of the integer pretraining section)       */
/* ------------------------------------------------------------------------------------------ */
/*
 *   E[j,k]      = sum_i F_i A_i[j] B_i[k]                      int32, F_i in {-1, 0, 1}   "E = (diag(F)A)^T B"
 *   theta'[j,k] = clamp(theta[j,k] + sign(E[j,k]) * [ |E[j,k]| >= threshold ], -127, 127)
 * "when the absolute value of E is above a pre-specified threshold we move theta by one discrete
 * bin in the direction of the sign of E".  The boundary case |E| == threshold moves (a reading: the
 * paper says "above"; >= makes threshold 0 mean "every non-zero E moves").  E as explicit outer
 * products member by member.  Returns 0, -1 on allocation failure, -2 if some |E| left int32.
 * E_out may be NULL.
 */
int oracle_update_i8(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin,
                     int64_t member_count, int d_out, int d_in, int bound, const int8_t* F,
                     int64_t threshold, const int8_t* theta_in, int8_t* theta_out, int32_t* E_out)
{
    int8_t* A = (int8_t*)malloc((size_t)d_out * (size_t)member_count + 1);
    int8_t* B = (int8_t*)malloc((size_t)d_in * (size_t)member_count + 1);
    if (!A || !B) { free(A); free(B); return -1; }
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < member_count; ++m) {
        oracle_noise_int(seed, step, layer, 0, member_begin + m, 0, (uint64_t)d_out, bound, A + (size_t)d_out * (size_t)m);
        oracle_noise_int(seed, step, layer, 1, member_begin + m, 0, (uint64_t)d_in, bound, B + (size_t)d_in * (size_t)m);
    }
    int overflow = 0;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < d_out; ++j) {
        int64_t* e = (int64_t*)calloc((size_t)d_in, sizeof(int64_t));
        for (int64_t m = 0; m < member_count; ++m) {
            const int64_t fa = (int64_t)F[m] * (int64_t)A[(size_t)d_out * (size_t)m + j];
            if (fa == 0) continue;
            const int8_t* b = B + (size_t)d_in * (size_t)m;
            for (int k = 0; k < d_in; ++k) e[k] += fa * (int64_t)b[k];
        }
        for (int k = 0; k < d_in; ++k) {
            const int64_t v = e[k], mag = v < 0 ? -v : v;
            if (mag > 2147483647LL) {
#pragma omp atomic write
                overflow = 1;
            }
            if (E_out) E_out[(size_t)j * d_in + k] = (int32_t)v;
            int t = theta_in[(size_t)j * d_in + k];
            if (mag >= threshold && v != 0) t += v > 0 ? 1 : -1;
            if (t > 127) t = 127;
            if (t < -127) t = -127;
            theta_out[(size_t)j * d_in + k] = (int8_t)t;
        }
        free(e);
    }
    free(A); free(B);
    return overflow ? -2 : 0;
}

/*
 * Threshold of the integer update, precalculated on the CPU as the paper says:
 *     I32(16 * Phi^-1(.)) * 16 sqrt(N)        for noise of standard deviation 16.
 * Printed argument of Phi^-1 is (1 - alpha)/2; with it the updated fraction would be 1 - alpha, while
 * the text states that alpha "approximately equals the fraction of parameters that are updated" and
 * lets alpha decay from 1 towards 0.  Reading taken: the two-sided alpha-quantile z = Phi^-1(1 - alpha/2)
 * (so P(|Z| >= z) = alpha), I32 = truncation, and 16 generalised to the standard deviation of the noise in
 * use:  threshold = trunc(noise_std * z) * round(noise_std * sqrt(n_terms)).
 * Phi^-1 by bisection on erfc (monotone; 200 halvings of [0, 40]).
 */
int64_t oracle_int_threshold(double alpha, int64_t n_terms, double noise_std)
{
    if (!(alpha > 0.0)) return INT64_MAX;
    if (alpha >= 1.0) return 0;
    double lo = 0.0, hi = 40.0;
    for (int it = 0; it < 200; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (erfc(mid * 0.70710678118654752440) > alpha) lo = mid; /* P(|Z| >= mid) = erfc(mid / sqrt 2) */
        else hi = mid;
    }
    const double z = 0.5 * (lo + hi);
    const int64_t first = (int64_t)(noise_std * z); /* truncation */
    const int64_t second = (int64_t)llround(noise_std * sqrt((double)n_terms));
    return first * second;
}

/* ------------------------------------------------------------------------------------------ */
/* integer model around the cell (App. "EGG architecture": Embedding, Layer Normalisation,     */
/* MLP, Alg. "EGG forward pass")                                                               */
/* ------------------------------------------------------------------------------------------ */
/*
 * Layer normalisation of rows u in I8^D, D a power of two:
 *     u_mav = (sum_k |u_k|) >> log2(D)                            mean absolute value, fraction dropped
 *     out_k = I8( DIVIDE( I16(u_k) * I16(ln_k), u_mav ) )
 * Readings: DIVIDE is the integer quotient rounded toward zero (symmetric in the sign of the product,
 * like the rest of the integer model); a row whose mean absolute value truncates to 0 divides by 1;
 * the quotient is clipped to [-127, 127] (the result feeds an int8 matmul).
 */
void oracle_layernorm_i8(int64_t rows, int D, const int8_t* ln, const int8_t* U, int8_t* out)
{
    int lg = 0;
    while ((1 << lg) < D) ++lg;
    for (int64_t r = 0; r < rows; ++r) {
        const int8_t* u = U + (size_t)r * D;
        int64_t sum = 0;
        for (int k = 0; k < D; ++k) sum += u[k] < 0 ? -(int64_t)u[k] : (int64_t)u[k];
        int64_t mav = sum >> lg;
        if (mav == 0) mav = 1;
        for (int k = 0; k < D; ++k) {
            const int64_t prod = (int64_t)u[k] * (int64_t)ln[k];
            const int64_t mag = (prod < 0 ? -prod : prod) / mav;
            out[(size_t)r * D + k] = (int8_t)sat127(prod < 0 ? -mag : mag);
        }
    }
}

/*
 * Perturbed embedding: y = I8( emb[t] + ((A_i[t] * I32(B_i)) >> corr_shift) ), emb in I8^{256 x D}.
 * The lookup is one_hot(t) applied to the table, so the dot product of the input with the token-side
 * factor is that factor's entry t ("replacing u.B with B[t]").  Readings: the factor indexed by the
 * token is drawn from stream A (length 256) and the one along the width from stream B (length D), so
 * the perturbation A B^T has the table's own [256][D] layout; the output scaling 1/(16 sqrt n) of a
 * matmul does not apply to a lookup (it would erase the table entry).  tokens: [count]; Y: [count][D].
 */
void oracle_embed_i8(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin, int64_t member_count,
                     int D, int bound, int corr_shift, int antithetic, const int8_t* emb, const uint8_t* tokens,
                     int8_t* Y)
{
    int8_t A[256];
    int8_t* B = (int8_t*)malloc((size_t)D);
    for (int64_t m = 0; m < member_count; ++m) {
        const int64_t member = member_begin + m;
        const int64_t noise_id = antithetic ? member / 2 : member;
        oracle_noise_int(seed, step, layer, 0, noise_id, 0, 256, bound, A);
        oracle_noise_int(seed, step, layer, 1, noise_id, 0, (uint64_t)D, bound, B);
        const int sign = (antithetic && (member & 1)) ? -1 : 1;
        const int t = tokens[m];
        for (int j = 0; j < D; ++j) {
            const int64_t corr = shr_floor((int64_t)A[t] * (int64_t)(sign * B[j]), corr_shift);
            Y[(size_t)m * D + j] = (int8_t)sat127((int64_t)emb[(size_t)t * D + j] + corr);
        }
    }
    free(B);
}

/* 4 + log2(sqrt n): the division by 16 sqrt(n) of the scaled matmul as a shift; n must be a power of 4 */
static int scaled_shift(int n)
{
    int lg = 0;
    while ((1 << lg) < n) ++lg;
    return 4 + lg / 2;
}

/*
 * Alg. "EGG forward pass" for a population, T tokens per member, state carried from token to token:
 *     y = EMBED(emb, t)
 *     for each layer i:  y', s'_i = GRU(LN(ln1_i, y), s_i);  y = I8(y' + y)
 *                        y' = MLP(LN(ln2_i, y)) = (u @ mlp1_i^T) @ mlp2_i^T;  y = I8(y' + y)
 *     logits = LN(ln_out, y) @ head^T
 * Every "@" is the perturbed scaled matmul with out shift 4 + log2(sqrt d_in); D is a power of 4.
 * Noise layers: layer + 0 embedding; layer + 1 + 6 i + {0,1,2,3: Wf, Uf, Wh, Uh; 4: mlp1; 5: mlp2};
 * layer + 1 + 6 L the head.  Layer-norm weights and the two GRU biases are not perturbed.
 * Layouts: gru_w [L][4][D][D], gru_b [L][2][D] (bf, bh), ln1/ln2 [L][D], mlp1 [L][4D][D], mlp2 [L][D][4D],
 * tokens [T][count], S_in/S_out [L][count][D], logits [T][count][256].  Returns 0, or -1 (allocation).
 */
int oracle_egg_forward_i8(uint64_t seed, uint32_t step, uint32_t layer, int64_t member_begin, int64_t member_count,
                          int D, int L, int bound, int corr_shift, int antithetic, int T,
                          const int8_t* emb, const int8_t* ln1, const int8_t* gru_w, const int8_t* gru_b,
                          const int8_t* ln2, const int8_t* mlp1, const int8_t* mlp2, const int8_t* ln_out,
                          const int8_t* head, const uint8_t* tokens, const int8_t* S_in, int8_t* S_out,
                          int8_t* logits)
{
    const size_t n = (size_t)member_count * (size_t)D;
    const size_t DD = (size_t)D * D;
    int8_t* y = (int8_t*)malloc(n);
    int8_t* u = (int8_t*)malloc(n);
    int8_t* yp = (int8_t*)malloc(n);
    int8_t* hid = (int8_t*)malloc(4 * n);
    int8_t* state = (int8_t*)malloc((size_t)L * n);
    if (!y || !u || !yp || !hid || !state) { free(y); free(u); free(yp); free(hid); free(state); return -1; }
    memcpy(state, S_in, (size_t)L * n);
    const int os_d = scaled_shift(D), os_4d = scaled_shift(4 * D);
    for (int t = 0; t < T; ++t) {
        oracle_embed_i8(seed, step, layer, member_begin, member_count, D, bound, corr_shift, antithetic, emb,
                        tokens + (size_t)t * member_count, y);
        for (int i = 0; i < L; ++i) {
            const uint32_t base = layer + 1u + 6u * (uint32_t)i;
            const int8_t* w = gru_w + (size_t)i * 4 * DD;
            int8_t* s = state + (size_t)i * n;
            oracle_layernorm_i8(member_count, D, ln1 + (size_t)i * D, y, u);
            oracle_gru_step_i8(seed, step, base, member_begin, member_count, D, bound, corr_shift, os_d, antithetic,
                               w, w + DD, w + 2 * DD, w + 3 * DD, gru_b + (size_t)i * 2 * D,
                               gru_b + (size_t)i * 2 * D + D, u, s, yp);
            memcpy(s, yp, n);                                        /* the cell's output is the new state */
            for (size_t e = 0; e < n; ++e) y[e] = (int8_t)sat127((int64_t)yp[e] + y[e]);
            oracle_layernorm_i8(member_count, D, ln2 + (size_t)i * D, y, u);
            forward_i8_worker(seed, step, base + 4, member_begin, member_count, 4 * D, D, bound, corr_shift, os_d, 1,
                              antithetic, mlp1 + (size_t)i * 4 * DD, u, hid);
            forward_i8_worker(seed, step, base + 5, member_begin, member_count, D, 4 * D, bound, corr_shift, os_4d, 1,
                              antithetic, mlp2 + (size_t)i * 4 * DD, hid, yp);
            for (size_t e = 0; e < n; ++e) y[e] = (int8_t)sat127((int64_t)yp[e] + y[e]);
        }
        oracle_layernorm_i8(member_count, D, ln_out, y, u);
        forward_i8_worker(seed, step, layer + 1u + 6u * (uint32_t)L, member_begin, member_count, 256, D, bound,
                          corr_shift, os_d, 1, antithetic, head, u, logits + (size_t)t * member_count * 256);
    }
    memcpy(S_out, state, (size_t)L * n);
    free(y); free(u); free(yp); free(hid); free(state);
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* fitness of the integer language model (App. "Fitness Calculation in Integer Types")         */
/* ------------------------------------------------------------------------------------------ */
/*
 *   y' = I32(y) + 128;   o = y'[t'] - LOG2[ sum_j EXP2[y'_j] ]
 *   EXP2[i] = 16 * 2^(i/16),   LOG2[s] = 16 * log2(s / 16)
 * the log-likelihood of token t' in units of 1/16 bit (logits count sixteenths of a bit).  Reading: both
 * tables hold their formula rounded to the nearest integer (the paper calls them integer lookup tables and
 * does not say how the entries are rounded): for that choice parity is unpinned -- the pin holds the result to
 * the real log-softmax within 1.5/16 bit, which any rounding of the entries satisfies.  logits: int8 [rows][256], targets: uint8 [rows]; out: int32
 * [rows], added to what is there when accumulate != 0 (a member's fitness is the sum over its tokens).
 */
void oracle_loglik_i8(int64_t rows, const int8_t* logits, const uint8_t* targets, int accumulate, int32_t* out)
{
    for (int64_t r = 0; r < rows; ++r) {
        const int8_t* y = logits + (size_t)r * 256;
        int64_t sum = 0;
        for (int j = 0; j < 256; ++j) sum += (int64_t)nearbyint(16.0 * exp2(((double)y[j] + 128.0) / 16.0));
        const int32_t lg = (int32_t)nearbyint(16.0 * log2((double)sum / 16.0));
        const int32_t o = ((int32_t)y[targets[r]] + 128) - lg;
        out[r] = accumulate ? out[r] + o : o;
    }
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

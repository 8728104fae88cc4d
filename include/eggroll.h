/*
 * eggroll.h -- C ABI of the MI355X (gfx950) EGGROLL hot path.
 *
 * EGGROLL ("Evolution Strategies at the Hyperscale") evaluates a population of N members in one
 * batched pass.  Member i sees the weights  W_i = M + sigma * E_i,  E_i = A_i B_i^T / sqrt(r),
 * A_i in R^{d_out x r}, B_i in R^{d_in x r} (Sec. 4.1, Alg. 1), and the mean M is moved along
 * sum_i f_i E_i (EGGROLL UPDATE box, Eq. eggroll_update).  The library never forms W_i or E_i:
 *   forward:  u_i W_i^T = u_i M^T + (sigma/sqrt r) (u_i B_i) A_i^T      (Sec. 4.2)
 *   update :  sum_i f_i A_i B_i^T = (diag(f) A)^T B, one contraction over K = N*r   (Sec. 4.2)
 * and the factors A_i, B_i are never stored by the caller: they are a pure function of
 * (seed, step, layer, which, member, index) from a counter-based generator (Sec. 1; Alg. 1
 * "reconstruct E_j from the seeds").
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, valid on the device the
 *     context was created for, 16-byte aligned.  The library allocates only its own scratch
 *     (inside the context), never frees or keeps caller memory, never synchronises the stream:
 *     all work is enqueued on the stream given at creation and is ordered on it.
 *     One exception to "never synchronises": the first eggroll_loglik_i8 call of a context uploads its
 *     tables with a blocking copy.
 *   - Scratch only grows.  A call that needs more scratch than the context holds (the first call at a new,
 *     larger shape) allocates a larger buffer and parks the old one until eggroll_trim or eggroll_destroy, so
 *     work already enqueued, and HIP graphs captured from earlier calls, keep valid addresses.  A graph
 *     replays the scratch addresses of the calls it captured: capture after an eager call of the same shapes,
 *     and do not call eggroll_trim while such a graph is still in use.  eggroll_scratch_generation changes
 *     whenever a buffer was replaced.
 *   - A context is not thread-safe: its calls share the scratch, so calls on one context must not
 *     overlap in time on the host, and work of two contexts that share a stream is ordered by it.
 *   - Matrices are dense row-major.  M = W[d_out][d_in].  Activations X[R][d_in], Y[R][d_out] with
 *     R = member_count * rows_per_member, member-major: row q belongs to member
 *     member_begin + q / rows_per_member.  Factors are laid out [member][d][rank] (rank fastest).
 *   - Noise depends on the GLOBAL member id (member_begin + local index), so any partition of the
 *     population into calls (or devices) regenerates identical factors.  Ids must stay < 2^32.
 *   - Every call returns egg_status; nothing throws or aborts.  EGG_EINVAL: null pointer,
 *     non-positive or inconsistent size, misaligned pointer, rank not in {1,2,4,8,16}, member range
 *     outside [0, 2^32).  EGG_EUNSUPPORTED: a dtype/shape combination no kernel covers (the text
 *     from eggroll_last_error says which).  EGG_EHIP: a HIP runtime call failed.  EGG_ENOMEM:
 *     scratch could not be allocated.
 *   - Noise stream (fixed contract, bit-exact):  Threefry-2x32-20.
 *       stream key = Threefry(key=(seed lo32, seed hi32), counter=(step, layer | which<<31)),
 *                    which: A = 0, B = 1, layer < 2^31;
 *       words 2b, 2b+1 of member i's vector = Threefry(key = stream key, counter = (b, i)).
 *     Normal value n (n = d*rank + l) comes from word n: u = ((word>>9) + 1/2) 2^-23; words
 *     (2p, 2p+1) form a Box-Muller pair, z_2p = rho cos(2 pi u2), z_2p+1 = rho sin(2 pi u2),
 *     rho = sqrt(-2 ln u1); rounded to fp32, and then to bf16 (nearest even) in bf16 mode.
 *     Integer value n comes from byte n&3 (little end first) of word n>>2: with m = 2b+1,
 *     q = floor(256/m): byte < q*m ? floor(byte/q) - b : 0.
 */
#ifndef EGGROLL_H
#define EGGROLL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eggroll_ctx eggroll_ctx; /* opaque; owns scratch buffers and the stream handle */

typedef enum { EGG_OK = 0, EGG_EINVAL = -1, EGG_EUNSUPPORTED = -2, EGG_EHIP = -3, EGG_ENOMEM = -4 } egg_status;
typedef enum { EGG_F32 = 0, EGG_BF16 = 1, EGG_I8 = 2, EGG_U32 = 3 } egg_dtype;
typedef enum { EGG_NORMAL = 0, EGG_UNIFORM_INT = 1, EGG_RAW = 2, EGG_NORMAL_INT16 = 3 } egg_dist;
/* Passed as `int_bound` to any integer entry point: the factors are the paper's own integer noise instead of uniform
   integers (App. "Adding EGGROLL Perturbations": int8 values round(16 z), z ~ N(0,1), from a pre-generated table indexed
   at random).  Value n of a factor vector is T[h], h = 16-bit half n & 1 (low half first) of word n >> 1 of the stream,
   T[k] = round(16 Phi^-1((k + 1/2) / 65536)) for k = 0 .. 65535 (half away from zero; T[65535 - k] = -T[k]; |T| <= 69;
   standard deviation 16.0 to three digits).  With this noise the paper's correction shift is corr_shift = 4 + sigma_hat.
   The table is built on the host and uploaded with a blocking copy the first time a context needs it. */
#define EGG_INT_NOISE_NORMAL16 (-16)
typedef enum { EGG_ACT_NONE = 0, EGG_ACT_GELU = 1 } egg_act;

/* names one weight matrix at one ES iteration (Alg. 1: the seeds every worker knows) */
typedef struct { uint64_t seed; uint32_t step; uint32_t layer; } egg_key;

typedef struct {
    int64_t member_begin;     /* global id of the first member of this call              */
    int64_t member_count;     /* members in this call                                    */
    int32_t rows_per_member;  /* S: rows of X per member (tokens evaluated by a member)  */
    int32_t d_out, d_in;      /* M is d_out x d_in                                       */
    int32_t rank;             /* r in {1,2,4,8,16}                                       */
    int32_t antithetic;       /* forward passes only: 1 = members 2p, 2p+1 form pair p    */
} egg_shape;

/* Antithetic pairs (App. "Fitness Shaping": "antithetical pair"; used by the integer and quantised
   experiments).  With antithetic = 1 the two members of pair p = member/2 share the factors of noise
   id p and are evaluated at M + sigma E_p (even member) and M - sigma E_p (odd member); in the integer
   form the odd member uses (A_p, -B_p).  member_begin and member_count still count members and must
   be even; A_cache / B_cache then hold member_count/2 entries.  The update entry points take the pair
   view instead: member ids = pair ids, one fitness value per pair (antithetic must be 0 there). */

/* Context.  `device`: HIP device ordinal; `hip_stream`: a hipStream_t (NULL = default stream).
   Host pointers.  Destroy synchronises the stream and frees the scratch. */
egg_status eggroll_create(eggroll_ctx** out, int device, void* hip_stream);
egg_status eggroll_destroy(eggroll_ctx* ctx);
const char* eggroll_strerror(egg_status s);
/* text of the last failure on this context (host string owned by the context) */
const char* eggroll_last_error(const eggroll_ctx* ctx);

/* Number of scratch replacements so far (see "Scratch only grows" above). */
uint64_t eggroll_scratch_generation(const eggroll_ctx* ctx);
/* Waits for the stream and frees the scratch buffers that larger ones have replaced. */
egg_status eggroll_trim(eggroll_ctx* ctx);

/* 1/(N * sigma * sqrt(r)): the constant of the Monte-Carlo estimator (Eq. matrix_mc) times the
   1/sqrt(r) of E_i, so that  scale * sum_i f_i A_i B_i^T  =  (1/(sigma N)) sum_i f_i E_i.
   (Alg. 1 absorbs 1/sigma into the learning rate; pass your own `scale` for that form.) */
double eggroll_default_scale(int64_t population, double sigma, int rank);

/*
 * (1) Materialise the factors (Sec. 1 "reconstruct noise on demand"; Alg. 1 sampling lines).
 *   A_out[member_count][d_out][rank], B_out[member_count][d_in][rank]; either may be NULL.
 *   dist = EGG_NORMAL      dtype EGG_F32 or EGG_BF16      Gaussian factors
 *   dist = EGG_UNIFORM_INT dtype EGG_I8                   integers on {-int_bound..int_bound}
 *   dist = EGG_NORMAL_INT16 dtype EGG_I8                  the table noise of EGG_INT_NOISE_NORMAL16 (int_bound ignored)
 *   dist = EGG_RAW         dtype EGG_U32                  the raw 32-bit words (one per element)
 * rows_per_member is ignored.
 */
egg_status eggroll_noise_gen(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, egg_dtype dtype,
                             egg_dist dist, int int_bound, void* A_out, void* B_out);

/*
 * (2) Population forward of one linear layer (Sec. 4.2):
 *   Y[q][j] = act( sum_k X[q][k] W[j][k] + (sigma/sqrt r) sum_l t[q][l] A_i[j][l] ),
 *   t[q][l] = sum_k X[q][k] B_i[k][l],  i = member of row q.
 * io_dtype (W, X and the factors): EGG_BF16 (MFMA bf16, fp32 accumulate) or EGG_F32.
 * y_dtype: EGG_BF16 or EGG_F32 (EGG_F32 only when io_dtype is EGG_F32 or for inspection).
 * sigma == 0 runs the same kernels with the correction switched off (the unperturbed pass).
 * A_cache / B_cache: optional side outputs holding exactly what eggroll_noise_gen would write
 * for this key and shape, for reuse by eggroll_update; NULL = do not keep.
 * d_in must be a multiple of 8 (bf16) or 4 (fp32).
 */
egg_status eggroll_perturbed_forward(eggroll_ctx* ctx, egg_key key, const egg_shape* shape,
                                     egg_dtype io_dtype, egg_dtype y_dtype, float sigma, egg_act act,
                                     const void* W, const void* X, void* Y, void* A_cache, void* B_cache);

/*
 * (2b) eggroll_perturbed_forward for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as (2); the one
 * scratch buffer of that path, the projections t[R][rank] (fp32), lives in a static device array of
 * 2^20 values (4 MiB per GPU, held until the process ends) instead of the context's growable scratch, and the
 * call performs no hipMalloc / hipFree.  Limits: member_count * rows_per_member * rank <= 2^20, else
 * EGG_EUNSUPPORTED; with more than one row per member or rank > 1 the factors A_i are materialised, so A_cache
 * must be given (EGG_EINVAL otherwise); per-kernel timing must be off.  Every call on one GPU, from any
 * context, shares the array: calls that overlap in time on one GPU race; calls ordered on one stream do not.
 */
egg_status eggroll_perturbed_forward_noalloc(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                             egg_dtype y_dtype, float sigma, egg_act act, const void* W, const void* X,
                                             void* Y, void* A_cache, void* B_cache);

/*
 * (2a) The same layer inside a residual stream:  Y = R_in + act( X W_i^T )  with W_i as in (2), summed in
 * fp32 before the one rounding to y_dtype.  R_in: [R][d_out] of y_dtype; it may be Y itself (every element
 * is read once and then written once by the same wavefront).  All other arguments as in (2).
 */
egg_status eggroll_perturbed_forward_add(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                         egg_dtype y_dtype, float sigma, egg_act act, const void* W, const void* X,
                                         const void* R_in, void* Y, void* A_cache, void* B_cache);

/*
 * (2c) The same layer between other perturbed layers, without reading activations twice (App. "Arithmetic Intensity
 * Analysis": the R x r projections are the only intermediate the method adds to a layer's traffic).
 *   R_in:   optional residual as in (2a); NULL = none.
 *   t_in:   optional [R][rank] fp32 (device), the projections X B_i of THIS layer as an earlier call delivered them
 *           through its t_next; NULL = the projection pass of (2) reads X and forms them.  Read only when sigma > 0.
 *   want_next != 0: additionally t_next[row][l] = sum_j Y[row][j] * B'_{member(row)}[j][l] (fp32, device, [R][rank]),
 *           where B' are the factors B of the layer with noise id next_layer (same seed, step and rank; its d_in is this
 *           d_out), formed from the very bf16 values stored to Y -- what that layer's own projection pass would compute,
 *           summed in another order.  This form exists for io_dtype = y_dtype = EGG_BF16, rank 1, 2 or 4, act = EGG_ACT_GELU,
 *           R_in = NULL, sigma > 0, no antithetic pairs, rows_per_member and d_in multiples of 64, and at least 192
 *           output tiles of 256 x 256; anything else returns EGG_EUNSUPPORTED before any work is enqueued, and the
 *           caller uses plain calls.  The factors B' are drawn into context scratch.
 * Factor caches are not written by this entry point.
 */
egg_status eggroll_perturbed_forward_chained(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                             egg_dtype y_dtype, float sigma, egg_act act, const void* W, const void* X,
                                             const void* R_in, void* Y, const float* t_in, int want_next,
                                             uint32_t next_layer, float* t_next);

/*
 * Layout of the factor caches that eggroll_perturbed_forward writes and eggroll_update reads on this context
 * (default EGG_CACHE_ROWS: exactly what eggroll_noise_gen writes, [member][d][rank]).
 * EGG_CACHE_PANEL keeps only B, already in the form the update's contraction consumes (Sec. 4.2,
 * "(diag(f)A)^T B"): B_cache is [ceil(member_count / 8)][d_in][8] fp16 (16 bytes = one input column of 8
 * consecutive members, zero beyond the last member; bf16 factors are exact in fp16), A_cache must be NULL.
 * The forward pass then costs one more write of the panel, and the update neither regenerates nor repacks B;
 * A is regenerated from the key (its panel carries the fitness, which the forward pass cannot know).
 * Supported for bf16, rank 1, one row per member, not antithetic; other shapes return EGG_EUNSUPPORTED when
 * a B_cache is passed.  Results of both calls are bit-identical to those of the default layout.
 */
typedef enum { EGG_CACHE_ROWS = 0, EGG_CACHE_PANEL = 1 } egg_cache_layout;
egg_status eggroll_set_cache_layout(eggroll_ctx* ctx, egg_cache_layout layout);

/*
 * Diagnostic switch.  The row-streaming integer matmul (used at d_in = 256) keeps loads in flight across its loop
 * iterations and waits for them by count; with on != 0 it waits for every outstanding load instead (slower, no
 * assumption about how many loads are in flight).  Results are identical in both forms; a test holds one against the other.
 */
egg_status eggroll_set_conservative_waits(eggroll_ctx* ctx, int on);

/*
 * (2') Integer form (App. "Matrix Multiplication", "Adding EGGROLL Perturbations"), rank 1, one row per
 * member, W[d_out][d_in] int8 (both multiples of 16), applied `steps` times (steps > 1 feeds h' back in
 * and needs d_out == d_in; one step with a rectangular W is the integer MLP's matmul):
 *   acc  = h W^T (int32);  dot = h . B_i (int32)
 *   h'_j = clamp( (acc_j + ((dot * int32(A_i[j])) >> corr_shift)) >> out_shift, -127, 127 )
 * Shifts are arithmetic (floor).  H_in: int8 [member_count][d_in], H_out: int8 [member_count][d_out]; they
 * may alias when the matrix is square.  The factors are integers on {-int_bound..int_bound}, fixed over
 * the `steps` applications.  Bit-exact.
 */
egg_status eggroll_perturbed_forward_i8(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int int_bound,
                                        int corr_shift, int out_shift, int steps, const int8_t* W,
                                        const int8_t* H_in, int8_t* H_out);

/*
 * (2'') Integer GRU cell (App. "GRU" of the EGG architecture), a population of states advanced over
 * `steps` inputs; "@" is the perturbed scaled matmul of (2'), I8 clips to [-127, 127], shifts are arithmetic:
 *   f  = I8( I32(u @ Wf^T) + I32(s @ Uf^T) + I32(bf) )          f^ = I8( ((I32(f) + 127) * I32(s)) >> 8 )
 *   h^ = I8( I32(u @ Wh^T) + I32(f^ @ Uh^T) + I32(bh) )         h  = I8( s + I8( ((I32(f) + 127) * (I32(h^) - I32(s))) >> 8 ) )
 * (sigma and phi are the identity, as the paper sets them).  Wf, Uf, Wh, Uh: int8 [D][D] (D = d_out = d_in,
 * a multiple of 16), perturbed independently with the noise of layers key.layer .. key.layer + 3, fixed over
 * the steps; bf, bh: int8 [D], not perturbed.  U: int8 [steps][member_count][D] inputs, S_in / S_out:
 * int8 [member_count][D] (may alias).  One row per member; antithetic pairs as in (2').  Bit-exact.
 */
egg_status eggroll_gru_i8(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int int_bound, int corr_shift,
                          int out_shift, int steps, const int8_t* Wf, const int8_t* Uf, const int8_t* Wh,
                          const int8_t* Uh, const int8_t* bf, const int8_t* bh, const int8_t* U,
                          const int8_t* S_in, int8_t* S_out);

/*
 * (2c) The integer model around the cell (App. "EGG architecture": Embedding, Layer Normalisation, MLP;
 * Alg. "EGG forward pass").  All arrays are device pointers, 16-byte aligned, owned by the caller.
 *
 * Layer normalisation of int8 rows U[rows][D] with weight ln[D], D a power of two in [16, 1024]:
 *   mav = max((sum_k |u_k|) >> log2 D, 1);   out_k = I8( trunc( I16(u_k) * I16(ln_k) / mav ) )
 * (quotient toward zero; a row whose mean absolute value truncates to 0 divides by 1; I8 clips to
 * [-127, 127]).  Not perturbed.  out may alias U.
 */
egg_status eggroll_layernorm_i8(eggroll_ctx* ctx, int64_t rows, int D, const int8_t* ln, const int8_t* U,
                                int8_t* out);

/*
 * Perturbed embedding lookup (App. "Embedding"; "Adding EGGROLL Perturbations", last paragraph):
 *   Y[m] = I8( emb[t_m] + ((A_i[t_m] * I32(B_i)) >> corr_shift) ),   emb: int8 [256][D], tokens: uint8 [member_count]
 * A_i (length 256, indexed by the token) and B_i (length D) are the rank-1 factors of key.layer, so the
 * perturbation A_i B_i^T has the table's layout and eggroll_update_i8 with d_out = 256, d_in = D updates the
 * table.  shape: d_out = d_in = D (a power of two in [16, 1024]), rank 1, rows_per_member 1; antithetic as
 * in (2').  No output scaling (a lookup is not a sum over n terms).  Y: int8 [member_count][D].
 */
egg_status eggroll_embed_i8(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int int_bound, int corr_shift,
                            const int8_t* emb, const uint8_t* tokens, int8_t* Y);

/* Parameters of the integer model, L layers of width D (device pointers, int8).  The forward pass only
 * reads them; eggroll_egg_update_i8 rewrites emb, gru_w, mlp1, mlp2 and head in place. */
typedef struct {
    int8_t* emb;    /* [256][D] */
    int8_t* ln1;    /* [L][D]         weight of the normalisation in front of the GRU */
    int8_t* gru_w;  /* [L][4][D][D]   Wf, Uf, Wh, Uh */
    int8_t* gru_b;  /* [L][2][D]      bf, bh */
    int8_t* ln2;    /* [L][D]         weight of the normalisation in front of the MLP */
    int8_t* mlp1;   /* [L][4D][D] */
    int8_t* mlp2;   /* [L][D][4D] */
    int8_t* ln_out; /* [D] */
    int8_t* head;   /* [256][D] */
} egg_model_i8;

/*
 * Forward pass of the integer model for a population, `steps` tokens per member, state carried over:
 *   y = EMBED(emb, t);  per layer i:  y', s'_i = GRU(LN(ln1_i, y), s_i),  y = I8(y' + y),
 *                                     y' = (LN(ln2_i, y) @ mlp1_i^T) @ mlp2_i^T,  y = I8(y' + y);
 *   logits = LN(ln_out, y) @ head^T
 * Every "@" is the perturbed scaled matmul of (2') with out_shift = 4 + log2(sqrt d_in) (the division by
 * 16 sqrt n), so D must be a power of 4: 16, 64, 256 or 1024.  Noise layers: key.layer the embedding,
 * key.layer + 1 + 6 i + {0, 1, 2, 3: Wf, Uf, Wh, Uh; 4: mlp1; 5: mlp2}, key.layer + 1 + 6 L the head; the
 * factors are generated once per call.  Normalisation weights and GRU biases are not perturbed.
 * shape: d_out = d_in = D, rank 1, rows_per_member 1; antithetic as in (2').  layers >= 0.
 * tokens: uint8 [steps][member_count]; S_in, S_out: int8 [layers][member_count][D], must not overlap
 * (both may be NULL when layers == 0); logits: int8 [steps][member_count][256].  Scratch held by the
 * context: about (18 layers + 2) D + 512 bytes per noise id for the factors, 11 D + 4 (4 + 2 layers) bytes per
 * member for one step's activations and dot products and, when steps > 1, one more copy of the state.  Bit-exact.
 */
egg_status eggroll_egg_forward_i8(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int layers, int int_bound,
                                  int corr_shift, int steps, const egg_model_i8* model, const uint8_t* tokens,
                                  const int8_t* S_in, int8_t* S_out, int8_t* logits);

/*
 * Fitness of the integer language model (App. "Fitness Calculation in Integer Types"): for each row the
 * log-likelihood of its target token in units of 1/16 bit,
 *   y' = I32(y) + 128;   o = y'[t'] - LOG2[ sum_j EXP2[y'_j] ],   EXP2[i] = 16 * 2^(i/16),  LOG2[s] = 16 * log2(s/16),
 * both tables rounded to the nearest integer (LOG2 is evaluated exactly for every sum, not stored: 2^28 entries).
 * logits: int8 [rows][256] (what eggroll_egg_forward_i8 writes for one time step, or several steps as one
 * block of rows), targets: uint8 [rows], out: int32 [rows]; accumulate != 0 adds to out (a member's fitness is
 * the sum over its tokens).  Pointers 16-byte aligned (targets: any).  Not perturbed.  Bit-exact.
 */
egg_status eggroll_loglik_i8(eggroll_ctx* ctx, int64_t rows, const int8_t* logits, const uint8_t* targets,
                             int accumulate, int32_t* out);

/*
 * Integer update of every perturbed parameter of the model (App. "Parameter Update"), the counterpart of
 * eggroll_egg_forward_i8 with the same key: for the embedding table, the four GRU matrices and the two MLP
 * matrices of each layer, and the head, with that parameter's noise layer,
 *   E = sum_i F_i A_i B_i^T (int32),   theta <- clamp(theta + sign(E) [|E| >= threshold], -127, 127)
 * exactly as eggroll_update_i8 does for one matrix (one call of it per parameter, 6 layers + 2 launches of
 * its kernels).  shape: member ids are noise ids (pair ids when the forward ran antithetic pairs; antithetic
 * must be 0 here), d_out = d_in = D, rank 1.  fitness: int8 [member_count] in {-1, 0, 1}, one shaped value
 * per noise id (for pairs sign(s+ - s-), "Fitness Shaping").  Normalisation weights and biases are left as
 * they are (the paper perturbs and updates matrices and the embedding only).  Bit-exact.
 */
egg_status eggroll_egg_update_i8(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int layers, int int_bound,
                                 const int8_t* fitness, int32_t threshold, const egg_model_i8* model);

/*
 * (3) Update direction (EGGROLL UPDATE box; Sec. 4.2 "(diag(f)A)^T B"):
 *   G[j][k] = (accumulate ? G[j][k] : 0) + scale * sum_i fitness[i] sum_l A_i[j][l] B_i[k][l]
 * G: fp32 [d_out][d_in].  fitness: fp32 [member_count], used as given (centring / z-scoring /
 * ranking is the caller's shaping).  noise_dtype: EGG_BF16 or EGG_F32 -- the precision the forward
 * pass evaluated the factors in.  A_cache/B_cache: the side outputs of the forward (or of
 * eggroll_noise_gen); NULL = regenerate from the key.
 * If W != NULL:  W[j][k] += lr * G[j][k], rounded to w_dtype (EGG_BF16 or EGG_F32), after G is final.
 * rows_per_member is ignored.
 */
egg_status eggroll_update(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, egg_dtype noise_dtype,
                          const float* fitness, float scale, int accumulate, float* G, void* W,
                          egg_dtype w_dtype, float lr, const void* A_cache, const void* B_cache);

/*
 * (3') Integer parameter update (App. "Parameter Update" of the integer pretraining section), rank 1:
 *   E[j][k]     = sum_i fitness[i] * A_i[j] * B_i[k]          int32; fitness[i] in {-1, 0, 1}
 *   theta[j][k] = clamp( theta[j][k] + sign(E[j][k]) * [ |E[j][k]| >= threshold ], -127, 127 )
 * theta: int8 [d_out][d_in], updated in place.  fitness: int8 [member_count] (with antithetic
 * pairs: one shaped value sign(s+ - s-) per pair, and member ids are pair ids).  The factors are the
 * integers on {-int_bound..int_bound} that eggroll_perturbed_forward_i8 uses for the same key.
 * threshold >= 0 (0: every non-zero E moves its entry).  E_out: optional int32 [d_out][d_in].
 * d_out and d_in must be multiples of 16, member_count * int_bound^2 < 2^31.  Bit-exact; the result
 * does not depend on the order in which partial sums are combined.  rows_per_member is ignored.
 */
egg_status eggroll_update_i8(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int int_bound,
                             const int8_t* fitness, int32_t threshold, int8_t* theta, int32_t* E_out);

/* The 65536-entry table behind EGG_INT_NOISE_NORMAL16, computed on the host (out: 65536 bytes).  Host-only. */
void eggroll_normal_int_table(int8_t* out);

/* Threshold of (3'), computed on the host as the paper prescribes: I32(16 Phi^-1(.)) * 16 sqrt(N) for
   noise of standard deviation 16, read as the two-sided alpha-quantile (a fraction of about alpha of
   the entries moves) and generalised to the standard deviation of the noise in use:
       trunc(noise_std * z) * round(noise_std * sqrt(n_terms)),   P(|Z| >= z) = alpha.
   alpha >= 1 gives 0; alpha <= 0 gives INT64_MAX.  Uniform integers on {-b..b} have
   noise_std = sqrt(b(b+1)/3).  Host-only, no context needed. */
int64_t eggroll_int_threshold(double alpha, int64_t n_terms, double noise_std);

/*
 * (4) Multi-layer float workloads built on (2) and (3).  The paper perturbs every parameter matrix of a
 * model independently (Alg. 1; Sec. 4.1) and evaluates all members in one batched pass (Sec. 4.2); the two
 * model families below are the synthetic stand-ins this library is measured on.  Everything is bf16,
 * row-major, member-major rows; a population is walked in chunks of `chunk_members` members (0 = a default
 * of about 2^18 rows per chunk), which changes neither noise nor results.  Activations of one chunk live in
 * the context's scratch.
 *
 * Unperturbed glue (identical in the perturbed and the sigma = 0 pass); d a multiple of 8:
 *   embed_rows       X[q] = emb[tokens[q]]                         emb [vocab][d], tokens int32 [rows] in [0, vocab)
 *   rmsnorm          Y[q][k] = X[q][k] gain[k] / sqrt(mean_k X[q][k]^2 + eps);  Y may be X
 *   causal_attention per member and head, over the member's own rows_per_member <= 256 tokens:
 *                    O[s] = sum_{s' <= s} softmax_s'( Q[s].K[s'] / sqrt(head_dim) ) V[s'],  no positional encoding;
 *                    Q, K, V, O [members * rows_per_member][heads * head_dim], head h in columns h*head_dim..;
 *                    head_dim in {32, 64, 128}; O must not overlap Q, K or V
 *   token_loglik     out[q] = logits[q][tokens[q+1]] - log sum_j exp(logits[q][j]) for every token that has a
 *                    successor in its member, 0 for a member's last token; logits [rows][vocab], vocab a multiple of 8
 */
egg_status eggroll_embed_rows_bf16(eggroll_ctx* ctx, int64_t rows, int d, int vocab, const void* emb, const int32_t* tokens, void* X);
egg_status eggroll_rmsnorm_bf16(eggroll_ctx* ctx, int64_t rows, int d, float eps, const void* gain, const void* X, void* Y);
egg_status eggroll_causal_attention_bf16(eggroll_ctx* ctx, int64_t members, int rows_per_member, int heads, int head_dim,
                                         const void* Q, const void* K, const void* V, void* O);

/*
 * The same attention, and additionally the rank-1 projections of its output for the perturbed layer that reads it
 * (the o-projection): t_next[row] = sum_j O[row][j] * B_{member(row)}[j] (fp32, device, [members * rows_per_member]),
 * B = the factors B of the layer (key.seed, key.step, key.layer) for members member_begin .. member_begin + members - 1
 * over d_in = heads * head_dim, formed from the bf16 values stored to O (the heads' shares are added in head order).
 * Pass t_next as t_in of eggroll_perturbed_forward_chained for that layer: O is then not read by a projection pass.
 * The factors are drawn into context scratch.
 */
egg_status eggroll_causal_attention_project_bf16(eggroll_ctx* ctx, egg_key key, int64_t member_begin, int64_t members,
                                                 int rows_per_member, int heads, int head_dim, const void* Q, const void* K,
                                                 const void* V, void* O, float* t_next);
egg_status eggroll_token_loglik_bf16(eggroll_ctx* ctx, int64_t members, int rows_per_member, int vocab, const void* logits,
                                     const int32_t* tokens, float* out);

/*
 * GELU MLP stack:  per layer l  h <- W2_l' gelu( W1_l' h ),  W' the member's perturbed copy, gelu in the exact
 * erf form, activations rounded to bf16 between the linear layers, no bias, normalisation or residual.
 * shape: d_out = d_in = d (a multiple of 8), rows_per_member = S, rank, member range; antithetic 0.
 * W1: [layers][d_ff][d], W2: [layers][d][d_ff];  X, Y: [member_count * S][d] (Y may not be X).
 * Noise layer ids: key.layer + 2 l (W1_l), key.layer + 2 l + 1 (W2_l).
 * The update applies (3) to every matrix with its noise layer:  W <- bf16( W + lr * scale * sum_i f_i A_i B_i^T );
 * there shape names the whole population (rows_per_member ignored).
 */
egg_status eggroll_mlp_stack_forward(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int layers, int d_ff, float sigma,
                                     const void* W1, const void* W2, const void* X, void* Y, int64_t chunk_members);
egg_status eggroll_mlp_stack_update(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, int layers, int d_ff,
                                    const float* fitness, float scale, float lr, void* W1, void* W2);

/*
 * Pre-norm decoder:  x = emb[token];  per layer l:
 *   h = rmsnorm(x; norm1_l);  q, k, v = Wq' h, Wk' h, Wv' h;  o = causal_attention(q, k, v);  x = x + Wo' o;
 *   h = rmsnorm(x; norm2_l);  x = x + Wdown' gelu( Wup' h );
 * logits = Whead' rmsnorm(x; norm_f).  The embedding table and the normalisation gains are not perturbed; the
 * 6 layers + 1 matrices are, under the noise layer ids key.layer + 6 l + {0..5: q, k, v, o, up, down} and
 * key.layer + 6 layers (head).  Every stored tensor is bf16; the residual sums are formed in fp32 (2a).
 * shape: rows_per_member = S <= 256 tokens per member, rank, member range (d_out, d_in ignored); antithetic 0.
 * tokens: int32 [member_count][S] in [0, vocab).  logits: bf16 [member_count * S][vocab] or NULL (then only a
 * chunk's logits exist at a time, in scratch); loglik: fp32 [member_count * S] as token_loglik defines, or NULL.
 * d_model = heads * head_dim with head_dim in {32, 64, 128}; d_model, d_ff, vocab multiples of 8.
 */
typedef struct { int32_t layers, d_model, heads, d_ff, vocab; float rms_eps; } egg_decoder_cfg;
typedef struct {
    void* emb;     /* [vocab][d]      */
    void* norm1;   /* [layers][d]     */
    void* wq;      /* [layers][d][d]  */
    void* wk;      /* [layers][d][d]  */
    void* wv;      /* [layers][d][d]  */
    void* wo;      /* [layers][d][d]  */
    void* norm2;   /* [layers][d]     */
    void* w_up;    /* [layers][d_ff][d] */
    void* w_down;  /* [layers][d][d_ff] */
    void* norm_f;  /* [d]             */
    void* head;    /* [vocab][d]      */
} egg_decoder_weights;
egg_status eggroll_decoder_forward(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, const egg_decoder_cfg* cfg,
                                   const egg_decoder_weights* weights, float sigma, const int32_t* tokens, void* logits,
                                   float* loglik, int64_t chunk_members);
egg_status eggroll_decoder_update(eggroll_ctx* ctx, egg_key key, const egg_shape* shape, const egg_decoder_cfg* cfg,
                                  const float* fitness, float scale, float lr, const egg_decoder_weights* weights);

/*
 * Per-kernel timing for benchmarks.  With profiling on, every kernel the library launches is
 * bracketed by HIP events on the context's stream.  eggroll_profile_read synchronises the stream
 * and fills names[i] (pointers to static strings), launches[i], total_ms[i] for up to `cap`
 * kernels; returns the number of distinct kernels (or a negative egg_status).  Reading resets.
 */
egg_status eggroll_profile_enable(eggroll_ctx* ctx, int on);
int eggroll_profile_read(eggroll_ctx* ctx, const char** names, int64_t* launches, double* total_ms, int cap);

#ifdef __cplusplus
}
#endif
#endif /* EGGROLL_H */

/*
 * gelo.h - C ABI of the GELO obfuscated-projection library for AMD MI355X (gfx950).
 *
 * GELO (Section 3.2 "Core Algorithm" of the paper) offloads a projection H*W to
 * an untrusted accelerator without showing it H:
 *
 *   trusted side      A  <- fresh random invertible n x n matrix        (step 1.2)
 *                     U  =  A * [H ; S]                                 (eq. 1, eq. 8)
 *   accelerator       Y  =  U * W                                       (eq. 2)
 *   trusted side      Z  =  A^-1 * Y, shield rows dropped               (eq. 3)
 *
 * and Z == H*W (eq. 4).  S are k secret high-norm "shield" rows (Section 3.2.1,
 * Mitigation 2); A is orthogonal (A^-1 = A^T) or a general well-conditioned
 * matrix (Mitigation 1).  Both roles run on one GPU here; U and Y are always
 * materialised in device memory because they are the messages the accelerator
 * sees (Section 3.1, the observation set O_t).
 *
 * Conventions
 *  - Every matrix pointer is a DEVICE pointer owned by the caller, row-major,
 *    16-byte aligned, with a leading dimension (in elements) that is a multiple
 *    of 8.  d and p must be multiples of 8.  The library never frees or keeps
 *    caller memory.  gelo_ctx and gelo_mixing objects are library-owned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued asynchronously on it; argument errors are reported
 *    synchronously and enqueue nothing.
 *  - dtype GELO_F32: H, W, U, Y, Z are float.  GELO_BF16: they are bfloat16
 *    (upper 16 bits of a float), products accumulate in float, A is generated
 *    in float and rounded once to bfloat16 for the two mixing products.
 *  - All calls return a gelo_status; gelo_last_error() gives a message for the
 *    last failing call on a context.  No exceptions, no aborts.
 *  - A context is not thread-safe.  Sampling uses context-owned workspace, so
 *    two gelo_sample_mixing calls on one context must not overlap in time on
 *    different streams; sampling may overlap mix/project/unmix of other batches.
 *  - Memory: a context owns a factorisation workspace, a pool of mixing objects and
 *    (for gelo_qkv_forward without caller U / Y) a chain workspace.  gelo_reserve
 *    sizes all three ahead of time; a per-batch call allocates only when it meets a
 *    shape that was not reserved (first use), and only then may it synchronise the
 *    device to replace a smaller buffer.  The per-batch calls make no host allocation.
 *  - The kernels clamp out-of-range rows and columns of a ragged last tile to valid
 *    addresses and multiply them by the zero padding of A; operand rows beyond the
 *    contraction length are replaced by zeros, so a NaN or Inf in the data reaches
 *    only the outputs that mathematically depend on it.
 */
#ifndef GELO_H
#define GELO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gelo_ctx gelo_ctx;        /* device, Philox key (seed), workspace, record of used batch ids */
typedef struct gelo_mixing gelo_mixing;  /* the trusted side's secrets for ONE batch: A, A^-1, shield directions */

typedef enum {
    GELO_OK = 0,
    GELO_EINVAL = 1,      /* null pointer, non-positive size, bad enum value */
    GELO_ESHAPE = 2,      /* sizes outside what the kernels support (see each call) */
    GELO_EDTYPE = 3,      /* dtype of the call and of the mixing object differ */
    GELO_EALIGN = 4,      /* pointer not 16-byte aligned or leading dimension / width not a multiple of 8 */
    GELO_ENOMEM = 5,      /* device or host allocation failed */
    GELO_ECOND = 6,       /* no draw with kappa_2(A) <= cond_max within max_attempts */
    GELO_ESINGULAR = 7,   /* zero pivot met while factorising A */
    GELO_EREUSE = 8,      /* batch id already used on this context, or mixing object already consumed */
    GELO_ESTATE = 9,      /* call out of order (unmix before mix) */
    GELO_EHIP = 10        /* HIP runtime error; text in gelo_last_error() */
} gelo_status;

typedef enum { GELO_F32 = 0, GELO_BF16 = 1 } gelo_dtype;

/* How A is drawn (Section 3.2 step 1.2; Section 3.2.1).
 *  ORTHOGONAL   A = Q diag(sign r_ii) from the Householder QR of a Philox Gaussian; A^-1 = A^T.
 *  GAUSSIAN     A = G/sqrt(n); redrawn until kappa_2(A) <= cond_max; A^-1 from a pivoted LU.
 *  CONDITIONED  A = Q + 0.25 G2/sqrt(n): dense, A^T A != I, kappa of a few; A^-1 from a pivoted LU.
 *  STRUCTURED   A = P_3 (B D_2 P_2)(B D_1 P_1)(B D_0 P_0): Philox-drawn row permutations P_r and sign
 *               flips D_r around B, the normalised Walsh-Hadamard transform on the row blocks of the
 *               binary expansion of n.  Orthogonal (A^-1 = A^T), never formed: mix and unmix apply it in
 *               O(n log n) per column and drawing it costs O(n^2 / 64) comparisons.  The "structured
 *               orthogonal transforms" the paper's Conclusion proposes for cheaper fresh mixing, in a
 *               construction of this library's own.  It leaks what every orthogonal A leaks
 *               (Section 3.2.1 eqs. 5-6: U^T U = H^T H, the spectrum of H H^T) and comes from a finite
 *               family, 4 permutations and 3 n sign bits; its resistance to the attacks of Section 4 has
 *               not been measured by anyone.  gelo_mixing_export builds the dense A for inspection.
 *  BLOCK_ORTHOGONAL  the mixed rows are cut into blocks of at most GELO_BLOCK_ROWS rows and each block is
 *               mixed by a dense orthogonal matrix of its own (the ORTHOGONAL construction on the block's own
 *               Philox Gaussian): rows [r0, r0 + rows) of U = A_i [H[d0 : d0 + dn]; S[s0 : s0 + sn]], where
 *               of the rows up to a cut r floor(k_shield r / n) are shield rows, so every block gets its
 *               share of them.  A^-1 = A^T.  Mixing costs O(n GELO_BLOCK_ROWS (d + p)) instead of
 *               O(n^2 (d + p)) and drawing it O(n GELO_BLOCK_ROWS^2): the other route to the cheaper fresh
 *               mixing the paper's Conclusion asks for.  What it gives up: rows mix only inside their block
 *               (a block's U^T U is the Gram matrix of ITS rows of [H; S], so the leak of eq. 5 is per block,
 *               244 rows at a time here instead of all n_data), which the paper does not analyse.
 *               gelo_mixing_export builds the dense n x n matrix that acts on the stacked [H; S].
 *  REFLECTOR_PRODUCT  A = H_0 H_1 ... H_{n-1} diag(sign beta_k): the Householder reflectors of the ORTHOGONAL
 *               construction, but reflector k is built from the raw entries G[k:, k] of the Philox Gaussian (it
 *               maps them to beta_k e_0) instead of from column k of a partly factorised matrix.  In the QR that
 *               column, given the earlier reflectors, is again a vector of independent Gaussians, so A has
 *               exactly the law of the ORTHOGONAL kind (Haar; Stewart 1980) - a dense orthogonal A with
 *               A^-1 = A^T, the same leakage statement - at half the arithmetic (4/3 n^3: only the product is
 *               formed) and without the chain of dependent panels: the cheaper generation of A that Section
 *               4.2 finds wanting for n > 2048.  A different matrix than ORTHOGONAL gives for the same ids. */
typedef enum { GELO_ORTHOGONAL = 0, GELO_GAUSSIAN = 1, GELO_CONDITIONED = 2, GELO_STRUCTURED = 3,
               GELO_BLOCK_ORTHOGONAL = 4, GELO_REFLECTOR_PRODUCT = 5 } gelo_kind;

/* Row-norm statistic of H that the shield rows are scaled by. */
typedef enum { GELO_NORM_MEDIAN = 0, GELO_NORM_MEAN = 1 } gelo_norm_stat;

#define GELO_MAX_N 5120        /* largest n = n_data + k_shield the factorisation kernels take */
#define GELO_MAX_ATTEMPTS 255  /* the attempt number is one byte of the Philox counter */
#define GELO_BATCH_WINDOW 4096 /* how far below the highest batch id used so far an unused id is still accepted */
#define GELO_STATIC_MAX_N 128  /* largest n gelo_qkv_forward_static takes (and one-launch batched draws) */
#define GELO_MAX_BATCH_DRAW 48 /* mixing objects one gelo_sample_mixing_batch call draws */
#define GELO_BLOCK_ROWS 256    /* mixed rows per block of a GELO_BLOCK_ORTHOGONAL A */
#define GELO_STATIC_SCRATCH_BYTES (16u << 20)   /* size of its static device buffer, held per GPU until the process ends */

/* Creates a context on HIP device `device` with Philox key `seed`.  `allow_batch_reuse` != 0
 * switches off the check that a batch id is used at most once (for tests and benchmarks that
 * replay a batch; production callers pass 0: A must never be reused, Section 3.2 step 1.2).
 * The check keeps no growing set: with h = 1 + the highest id used so far, an id is refused
 * (GELO_EREUSE) if it was used, if it lies below the floor (gelo_set_batch_floor), or if it lies
 * more than GELO_BATCH_WINDOW below h; ids at or above h are always new.  Callers that number their
 * batches upwards (layer by layer, step by step) never meet the window. */
gelo_status gelo_create(gelo_ctx** out, int device, uint64_t seed, int allow_batch_reuse);
/* Checkpoint / resume of "never reused": A is a pure function of (seed, batch id), so the whole state
 * of a context is its seed and the ids it has used.  gelo_get_batch_floor returns the smallest id f
 * such that no id >= f has been used; a context created later with the same seed and
 * gelo_set_batch_floor(ctx, f) refuses every id below f and so never derives an A a second time.
 * The floor only moves up (GELO_EINVAL otherwise). */
gelo_status gelo_set_batch_floor(gelo_ctx* ctx, uint64_t first_unused);
gelo_status gelo_get_batch_floor(const gelo_ctx* ctx, uint64_t* first_unused);
/* Sizes the context's device memory for batches of this shape before the first of them arrives:
 * the factorisation workspace (and the side-by-side attempt buffers of GELO_GAUSSIAN with this
 * max_attempts), `mixings` pooled mixing objects, and, if p > 0, the U / Y workspace of
 * gelo_qkv_forward.  May synchronise the device and allocate; the per-batch calls that follow
 * then do neither.  Arguments as in gelo_sample_mixing. */
gelo_status gelo_reserve(gelo_ctx* ctx, gelo_kind kind, gelo_dtype dtype, int n_data, int k_shield, int d, int p,
                         int max_attempts, int mixings);
gelo_status gelo_destroy(gelo_ctx* ctx);
/* Message of the last failing call on `ctx` ("" if none).  Owned by the context. */
const char* gelo_last_error(const gelo_ctx* ctx);
const char* gelo_status_string(gelo_status s);

/* Trusted side, Section 3.2 step 1.2.  Draws the secrets of batch `batch_id`: A (n x n,
 * n = n_data + k_shield), its inverse, and k_shield Gaussian shield directions of width d.
 * A pure function of (seed, batch_id, kind, n, k_shield, d) (GELO_BLOCK_ORTHOGONAL: its blocks depend on how n
 * splits into n_data and k_shield).  cond_max and max_attempts
 * (1..GELO_MAX_ATTEMPTS) are used by GELO_GAUSSIAN only: it factorises up to four consecutive
 * attempts side by side on streams of its own (n <= 1024; one at a time beyond), reads their
 * condition estimates back (the only host synchronisation in the library) and returns the first
 * acceptable attempt in order, so the result does not depend on how many ran at once.  The
 * estimate (20 Lanczos steps) approaches kappa_2 from below, within 0.5 % as measured; an attempt
 * is accepted only if 1.01 x estimate <= cond_max, so an accepted A meets the bound itself
 * ("generate and verify", Section 3.2.1) and a draw within 1 % below it may be redrawn.
 * n <= GELO_MAX_N (GELO_STRUCTURED keeps 4 columns of all n rows in one workgroup's LDS at least,
 * which allows more rows than that on this chip), n_data >= 1,
 * k_shield >= 0, d a multiple of 8.  *out is owned by the library: release it with
 * gelo_mixing_free (which recycles its device memory inside the context). */
gelo_status gelo_sample_mixing(gelo_ctx* ctx, gelo_kind kind, int n_data, int k_shield, int d,
                               gelo_dtype dtype, double cond_max, int max_attempts,
                               uint64_t batch_id, gelo_mixing** out, void* stream);

/* Trusted side, Section 3.2 step 1.2, many batches at once: `count` mixing objects (1..GELO_MAX_BATCH_DRAW) for
 * batch ids first_batch_id .. first_batch_id + count - 1, all of one shape.  A does not depend on the data, so
 * a decode step's worth, or the next few prefill batches, can be drawn ahead together.  GELO_ORTHOGONAL,
 * GELO_REFLECTOR_PRODUCT (always by the launches for larger n below), and
 * GELO_BLOCK_ORTHOGONAL (all full blocks of all objects share the launches of one batched factorisation).
 *  n <= GELO_STATIC_MAX_N  ONE launch draws all of them (at this size a fresh A per layer-step costs more in
 *                          launch latency than in work);
 *  larger n                up to 32 factorisations (fewer where 32 workspaces would exceed 4 GiB) share every
 *                          launch of the Householder QR, each in a workspace of its own (the chain of panel factorisations leaves most of the chip idle when one
 *                          matrix is factorised alone; side by side the strips of all of them fill it).
 * Object i is what gelo_sample_mixing returns for its batch id, bit for bit.  out: HOST array of `count`
 * pointers; on an argument error nothing is drawn and no id is consumed. */
gelo_status gelo_sample_mixing_batch(gelo_ctx* ctx, gelo_kind kind, int n_data, int k_shield, int d, gelo_dtype dtype,
                                     uint64_t first_batch_id, int count, gelo_mixing** out, void* stream);

/* Trusted side, eq. 1 / eqs. 7-8.  Shield rows S_i = g_i * shield_scale * m(H) / ||g_i||, m the
 * median or mean row 2-norm of H; then U[n x d] = A * [H ; S].  H: n_data x d (ldh), U: n x d (ldu),
 * both of type `dtype`, which must be the one the mixing object was drawn for (GELO_EDTYPE otherwise:
 * the kernels would read and write the buffers with the wrong element size).  The row counts are the
 * mixing object's (gelo_mixing_info); the caller's buffers must hold them. */
gelo_status gelo_mix(gelo_ctx* ctx, gelo_mixing* mixing, gelo_dtype dtype, const void* H, int64_t ldh,
                     float shield_scale, gelo_norm_stat stat, void* U, int64_t ldu, void* stream);

/* Accelerator side, eq. 2.  Y[n x p] = U[n x d] * W[d x p].  Touches no secret: it takes no
 * mixing object.  Also serves as the plain baseline H*W (pass H as U, n = n_data).  A bf16 product
 * of at most 96 rows whose width leaves most of the chip idle (p < 8192) cuts d over workgroups and
 * keeps their float partial sums in a context workspace (gelo_reserve with p sizes it): two such
 * calls on one context must not overlap in time on different streams. */
gelo_status gelo_project(gelo_ctx* ctx, gelo_dtype dtype, int n, int d, int p,
                         const void* U, int64_t ldu, const void* W, int64_t ldw,
                         void* Y, int64_t ldy, void* stream);

/* Accelerator side, eq. 2 with both operands stored as 8-bit floats (OCP FP8 E4M3, the "FP8 / INT8 quantized
 * numerics" of the paper's Conclusion): twice the matrix rate of the bf16 projection.  The weight is public and
 * static, so it is prepared once: gelo_prepare_weight_fp8 writes into the caller's DEVICE buffer Wq
 * (gelo_fp8_weight_bytes(d, p) bytes, 16-byte aligned) the codes of W^T (p x d bytes: code of
 * W[k][j] * 448 / max_k |W[k][j]| at byte j d + k, round to nearest even, saturating at 448), padded to a
 * multiple of 256 bytes, then the p column scales max_k |W[k][j]| / 448 as floats.  gelo_project_fp8 quantises
 * U (bf16, n x d) per row the same way into context workspace (allocated on first use of a size), multiplies
 * on the matrix cores with float accumulation and writes Y[i][j] = acc * su[i] * sw[j] as bf16.  d a multiple
 * of 128 (GELO_ESHAPE otherwise), p a multiple of 8.  The rounding of U and W to 3 fraction bits (relative
 * error 2^-4 per element at worst) reaches Z = A^-1 Y at about 4e-2 to 7e-2 relative Frobenius error with
 * shield rows in the batch: this call does NOT meet the 2e-2 bound of the bf16 chain; mix and unmix stay bf16. */
gelo_status gelo_fp8_weight_bytes(int d, int p, size_t* bytes);
gelo_status gelo_prepare_weight_fp8(gelo_ctx* ctx, int d, int p, const void* W, int64_t ldw, void* Wq, void* stream);
gelo_status gelo_project_fp8(gelo_ctx* ctx, int n, int d, int p, const void* U, int64_t ldu, const void* Wq,
                             void* Y, int64_t ldy, void* stream);

/* Trusted side, eq. 3 + shield drop.  Z[n_data x p] = (A^-1 * Y)[0:n_data, :]; the shield rows
 * of the product are never computed.  Y: n x p (ldy), Z: n_data x p (ldz), both of type `dtype`
 * (GELO_EDTYPE if it is not the mixing object's).  Marks the mixing consumed: a second
 * gelo_mix or gelo_unmix on it returns GELO_EREUSE. */
gelo_status gelo_unmix(gelo_ctx* ctx, gelo_mixing* mixing, gelo_dtype dtype, int p, const void* Y, int64_t ldy,
                       void* Z, int64_t ldz, void* stream);

gelo_status gelo_mixing_free(gelo_ctx* ctx, gelo_mixing* mixing);
/* gelo_mix, gelo_project and gelo_unmix (eqs. 1-3) for a mixing object drawn earlier, in one call: H (n_data x d),
 * W (d x p), Z (n_data x p), U (n x d) and Y (n x p) densely packed, all of type `dtype`; U and Y are required (they
 * are the observable messages).  The latency-bound decode path spends one host call per layer-step this way. */
gelo_status gelo_chain(gelo_ctx* ctx, gelo_mixing* mixing, gelo_dtype dtype, int p, const void* H, const void* W,
                       float shield_scale, gelo_norm_stat stat, void* Z, void* U, void* Y, void* stream);
/* Shape and type a mixing object was drawn for (any out pointer may be NULL): H is n_data x d,
 * U is (n_data + k_shield) x d, Y is (n_data + k_shield) x p, Z is n_data x p. */
gelo_status gelo_mixing_info(gelo_ctx* ctx, const gelo_mixing* mixing, int* n_data, int* k_shield, int* d,
                             gelo_dtype* dtype, gelo_kind* kind);

/* The whole chain for one batch: sample, mix, project, unmix (eqs. 1-3).  H: n_data x d, W: d x p,
 * Z: n_data x p, all densely packed (leading dimension = width).  U_opt (n x d) and Y_opt (n x p)
 * receive the two observable messages; if NULL they are written to context workspace instead. */
gelo_status gelo_qkv_forward(gelo_ctx* ctx, gelo_kind kind, gelo_dtype dtype, int n_data, int k_shield,
                             int d, int p, const void* H, const void* W, float shield_scale,
                             gelo_norm_stat stat, double cond_max, int max_attempts, uint64_t batch_id,
                             void* Z, void* U_opt, void* Y_opt, void* stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): gelo_qkv_forward for one decode-shaped batch with every intermediate of the
 * trusted side (A, A^-1, the factorisation workspace, shield directions and rows) in a static device
 * buffer of GELO_STATIC_SCRATCH_BYTES that each GPU the library runs on holds until the process ends.
 * Calls no hipMalloc / hipFree and creates no stream, event or pooled object.  n = n_data + k_shield
 * <= GELO_STATIC_MAX_N, and the batch's buffers (about 0.6 MB at n = 128 plus 10 bytes (bf16) or
 * 12 bytes (float) per element of the k_shield x d shield block) must fit the static buffer:
 * GELO_ESHAPE otherwise.  kind: any but GELO_GAUSSIAN.  U (n x d) and
 * Y (n x p) are required; H, W, Z, U, Y densely packed as in gelo_qkv_forward.  All calls on one GPU
 * share the one buffer, whatever their context or stream: calls that overlap in time on a GPU race;
 * issue them on one stream or order them yourself.  Same results, bit for bit, as gelo_qkv_forward
 * (a projection that cuts K over workgroups keeps its float partial sums in the static buffer too;
 * only if they do not fit behind the batch's buffers is K left whole, and Y then differs from
 * gelo_qkv_forward's in the order of summation: never for n x p up to 68 x 12288). */
gelo_status gelo_qkv_forward_static(gelo_ctx* ctx, gelo_kind kind, gelo_dtype dtype, int n_data, int k_shield,
                                    int d, int p, const void* H, const void* W, float shield_scale,
                                    gelo_norm_stat stat, uint64_t batch_id, void* Z, void* U, void* Y, void* stream);

/* Test hook: copies the secrets of a mixing object to caller DEVICE buffers (any may be NULL):
 * A and A_inv as float n x n (dense), S as float k_shield x d (dense; valid after gelo_mix).
 * attempt / kappa are HOST pointers: the accepted attempt number and the library's estimate of
 * kappa_2(A) (1 for ORTHOGONAL and STRUCTURED).  A STRUCTURED object holds no matrix: A and A_inv
 * are built here by transforming the identity, in the context workspace that gelo_qkv_forward also
 * uses for U / Y when they are not passed in - do not run the two at the same time on one context. */
gelo_status gelo_mixing_export(gelo_ctx* ctx, const gelo_mixing* mixing, float* A, float* A_inv,
                               float* S, int* attempt, float* kappa, void* stream);

/* Test hooks for bitwise checks of the integer work.
 * gelo_debug_philox_words: words[4 i .. 4 i + 3] (DEVICE, 16-byte aligned) = the four 32-bit outputs of
 * Philox4x32-10 for counter (first_block + i, stream_id << 8 | attempt, batch id low, batch id high)
 * under the context's key; stream ids: 0 mixing Gaussian (attempt = redraw number), 1 shield
 * directions, 2 CONDITIONED perturbation, 3 sort keys of permutation r and 4 sign words of round r of
 * the structured kind (r travels in the attempt byte).
 * gelo_mixing_export_table: the (rounds + 1) x n words of a GELO_STRUCTURED object (entry j of
 * permutation r in the low 31 bits, sign flip of position j in round r in the top bit) to a DEVICE buffer. */
gelo_status gelo_debug_philox_words(gelo_ctx* ctx, uint32_t stream_id, uint32_t attempt, uint64_t batch_id,
                                    uint32_t first_block, uint32_t blocks, uint32_t* words, void* stream);
gelo_status gelo_mixing_export_table(gelo_ctx* ctx, const gelo_mixing* mixing, uint32_t* table, void* stream);
/* Measurement aid (for the caller that reports a kernel against the matrix-core peak, as Section 4.2 style
 * "fraction of peak" figures do): what the matrix cores of this device deliver when every wave issues nothing
 * but independent matrix instructions from registers - v_mfma_f32_32x32x16_bf16 (fp8 = 0) or
 * v_mfma_f32_32x32x64_f8f6f4 on E4M3 (fp8 = 1), eight accumulator tiles per wave, two waves per SIMD, as in a K
 * step of the projection kernels; no memory traffic.  Runs one warm-up launch and `launches` (1..1000) timed
 * launches of `iters` (1..2^20) loop passes each on `stream`, WAITS for them, and returns the mean time of one
 * launch (HOST double) and the floating-point operations one launch executes (HOST double).  Uses the static
 * scratch buffer of gelo_qkv_forward_static: do not overlap the two on one GPU. */
gelo_status gelo_measure_matrix_rate(gelo_ctx* ctx, int fp8, int iters, int launches, double* seconds, double* flop,
                                     void* stream);

/* Test hook: the row quantisation gelo_project_fp8 applies to U, into caller DEVICE buffers: codes n x d bytes
 * (16-byte aligned), scales n floats. */
gelo_status gelo_debug_quantize_rows_fp8(gelo_ctx* ctx, int n, int d, const void* U, int64_t ldu, uint8_t* codes,
                                         float* scales, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GELO_H */

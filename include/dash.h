/*
 * dash.h -- C ABI of the MI355X (gfx950) library for the hot path of block-diagonal
 * Shampoo as organised by DASH (arXiv 2602.02016): every Kronecker factor is a B x B
 * block of one stacked N x B x B tensor (paper Section 4.1), and the optimizer step is
 *   accumulate (Algorithm 1, EMA lines) -> inverse p-th roots of the damped factors by
 *   Newton-DB (Section 3.3) or Chebyshev/Clenshaw (Appendix A) after Frobenius scaling
 *   (Section 3.4) -> preconditioned update (Algorithm 1, last line) -> optional
 *   block-wise Adam grafting (Section 2.3).
 *
 * Conventions for every call below
 *   - "dev" pointers are DEVICE pointers to contiguous row-major fp32 stacks [N][B][B]
 *     (strides B*B, B, 1) on the context's device.  They are owned by the caller; the
 *     library never allocates or frees device memory and keeps no reference after the
 *     work it enqueued has run.  "host" pointers are ordinary host memory.
 *   - B must be a positive multiple of 64; N >= 0 (N == 0 is a no-op returning DASH_OK).
 *   - Work is enqueued on the context's HIP stream and is asynchronous with respect to
 *     the host; the caller synchronises the stream before reading results.  (dash_inverse_root
 *     may run half of a stack of small blocks on a second stream of its own, forked from and
 *     joined back into the context's stream inside the call: see dash_set_lanes.  Stream order
 *     as the caller sees it does not change.)
 *   - Inputs declared const are never written.  Outputs must not overlap inputs unless
 *     a call says so.
 *   - Errors in arguments or launches are reported through the return code (and the
 *     text of dash_last_error); nothing is thrown and nothing aborts.  Numerical
 *     failure (a non-finite root, e.g. a block that is not positive definite) is
 *     reported through the optional per-block flag array, never by a return code.
 *   - Two calls on the same context must not overlap in time (they share the workspace).
 */
#ifndef DASH_H
#define DASH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A context binds a device, a HIP stream, a workspace and statistics.  Calls on one context must not run
 * concurrently (use one context per host thread); different contexts are independent. */
typedef struct dash_ctx dash_ctx;

typedef enum {
    DASH_OK = 0,
    DASH_ERR_INVALID_ARG = 1, /* null pointer, bad size, bad enum, aliasing that is not allowed */
    DASH_ERR_UNSUPPORTED = 2, /* valid request this build does not implement */
    DASH_ERR_WORKSPACE = 3,   /* workspace missing or too small for even one block */
    DASH_ERR_HIP = 4          /* a HIP runtime call failed (no device, launch error, ...) */
} dash_status;

typedef enum { DASH_NEWTON_DB = 0, DASH_CHEBYSHEV = 1, DASH_COUPLED_NEWTON = 2 } dash_method;
/* DASH_SCALE_POWER_ITERATION: s = 2 * lambda_PI, the multi-Power-Iteration estimate of
 * Sections 3.4 and 3.5 (configure it with dash_set_power_iteration first). */
typedef enum { DASH_SCALE_FROBENIUS = 0, DASH_SCALE_TRACE = 1, DASH_SCALE_NONE = 2,
               DASH_SCALE_POWER_ITERATION = 3 } dash_scaling;
/* DASH_FP32: fp32 MFMA operands.  DASH_FP16_ACC32 / DASH_BF16_ACC32: the recipe of
 * Appendix A.3 -- iterates kept in fp32, every matmul operand rounded to fp16 / bf16 (round to
 * nearest even), fp32 accumulation -- applied to Clenshaw (as in the paper) and to Newton-DB
 * (which the paper reports unstable in half precision).  DASH_BF16X3: every
 * operand is carried as two bf16 planes, x ~ hi + lo with hi = bf16(x), lo = bf16(x - hi), and a
 * product is A_lo B_hi + A_hi B_lo + A_hi B_hi accumulated in fp32 -- about 16 significand bits
 * per operand at three bf16 MFMA products, which keeps Newton-DB stable where plain bf16 is not.
 * DASH_BF16X6: three planes, x ~ hi + mid + lo (24 significand bits: a float is
 * represented exactly), and the six plane products of weight 2^-16 and above,
 * A_lo B_hi + A_hi B_lo + A_mid B_mid + A_mid B_hi + A_hi B_mid + A_hi B_hi -- fp32 accuracy from six
 * bf16 MFMA products, which cost less matrix-core time than one fp32 MFMA product.
 * DASH_FP16X3: two fp16 planes, hi = fp16(x), lo = fp16((x - hi) 2^11) kept scaled (unscaled it would be
 * subnormal), the same three products as DASH_BF16X3 with the two low-plane terms scaled back by 2^-11 in the
 * accumulator: 22 significand bits per operand -- close to fp32 accuracy from three fp16 MFMA products; fp16's
 * exponent range applies to the iterates (entries above 65504 overflow and are flagged).
 * The split modes serve every method. */
typedef enum { DASH_FP32 = 0, DASH_BF16_ACC32 = 1, DASH_FP16_ACC32 = 2, DASH_BF16X3 = 3, DASH_BF16X6 = 4,
               DASH_FP16X3 = 5 } dash_precision;

/* ---- context ------------------------------------------------------------------- */

/* Creates a context bound to HIP device `device` and to `hip_stream` (a hipStream_t
 * passed as void*; NULL = the device's default stream).  The stream stays owned by the
 * caller and must outlive the context.  Fails with DASH_ERR_HIP when no such device. */
dash_status dash_create(dash_ctx** out, int device, void* hip_stream);
dash_status dash_destroy(dash_ctx* ctx);
/* Later calls enqueue on hip_stream (e.g. a stream under hipStreamBeginCapture: every entry point only
 * launches kernels -- no allocation, no memset or copy nodes, no synchronisation unless dash_set_timing is
 * on; the one thing besides kernels is the event pair with which dash_inverse_root forks and joins its
 * second stream on stacks of small blocks, see dash_set_lanes -- so a call sequence can be captured into a
 * HIP graph and replayed). */
dash_status dash_set_stream(dash_ctx* ctx, void* hip_stream);

/* Device scratch the iterative calls need.  dash_workspace_bytes(n, ...) is the size
 * that lets n blocks be processed in one chunk; with a smaller workspace the library
 * walks the stack in chunks of as many blocks as fit (at least one must fit, otherwise
 * DASH_ERR_WORKSPACE).  The workspace is caller-owned device memory, 256-byte aligned,
 * and may be replaced between calls. */
size_t dash_workspace_bytes(int64_t n_blocks, int B, dash_method method, int p,
                            dash_precision precision);
dash_status dash_set_workspace(dash_ctx* ctx, void* dev_ptr, size_t bytes);

/* Text of the last error on this context (valid until the next failing call). */
const char* dash_last_error(const dash_ctx* ctx);
const char* dash_status_string(dash_status s);

/* Launch statistics since the last reset: number of batched B x B x B matmul launches
 * (one launch computing two products counts two) and, if timing was switched on with
 * dash_set_timing(ctx, 1), the summed device time of those launches measured with HIP
 * events on the context's stream (dash_get_stats synchronises the stream then).  Used
 * to check the paper's matmul counts (Section 3.3: 3 per Newton-DB iteration, first
 * iteration 1; Appendix A.2: degree d costs d-1) and for the roofline figure. */
typedef struct {
    int64_t matmul_products;   /* B x B x B products per block, summed over launches   */
    int64_t matmul_launches;   /* kernel launches of the batched matmul kernel          */
    double  matmul_block_products; /* sum over launches of products * blocks in launch  */
    double  matmul_ms;         /* summed event time of those launches (0 if timing off) */
    /* the same three figures per kernel variant v = 2*transA + transB (0: A B, 1: A B^T,
       2: A^T B, 3: A^T B^T) */
    int64_t variant_launches[4];
    double  variant_block_products[4];
    double  variant_ms[4];
    /* flops of the output tiles actually computed (in symmetric mode a launch computes only
       the tiles on or above the diagonal), in total and per variant */
    double  matmul_flops;
    double  variant_flops[4];
} dash_stats;
dash_status dash_reset_stats(dash_ctx* ctx);
dash_status dash_set_timing(dash_ctx* ctx, int on);
dash_status dash_get_stats(dash_ctx* ctx, dash_stats* out /* host */);

/* Symmetric mode (default on).  The residual product Z Y of Newton-DB (E = 3/2 I - 1/2 Z Y)
 * and every product of the Clenshaw recurrence are polynomials in the input block and
 * therefore symmetric in exact arithmetic, and G G^T, G^T G are symmetric bit for bit.  With
 * the mode on, those products compute only the output tiles on or above the diagonal (in the
 * operand order the paper prints) and write every off-diagonal tile a second time transposed.
 * The Newton-DB updates Y E and E Z are always computed in full: symmetrising them breaks the
 * coupling between Y and Z and the iteration diverges on ill-conditioned blocks.  Off: every
 * product is computed in full.  The preconditioned update and dash_gemm_batched always
 * compute full products. */
dash_status dash_set_symmetric(dash_ctx* ctx, int on);

/* Lanes (default on).  Blocks are independent through the whole path (Section 4.1).  On stacks of small blocks
 * (B <= 512, and a chunk of at least 1024 output tiles of 128 x 128 per product in fp32, 256 with 16-bit operands)
 * the launches of the iterative methods are so short that the fixed costs of a round of workgroups weigh a tenth
 * and more; dash_inverse_root then sends the two halves of a chunk through the
 * same launch sequence on two streams -- the context's and one the library creates in dash_create (default priority)
 * -- so that the two overlap.  The second stream waits for an event recorded on the context's stream when the
 * iterative part begins, and the context's stream waits for the second one when it ends: to the caller everything
 * still happens in the order of the context's stream, also under stream capture (the second stream joins the capture
 * and leaves it inside the call).  With every product computed in full the results are bit for bit the same with
 * lanes on and off; in symmetric mode the tile edge, which follows the launch size, decides which entries of a
 * mirrored product are computed and which are copies, so the two agree to rounding.  Off: one stream only. */
dash_status dash_set_lanes(dash_ctx* ctx, int on);

/* Multi-Power-Iteration scaling (Sections 3.4, 3.5).  For every block, with A_d = A + eps I:
 *   V_0 = start vectors, columns scaled to unit length; for t = 1..sweeps: W = A_d V_{t-1},
 *   q_j = v_j . w_j (Rayleigh quotient of the unit vector v_j), V_t = W with unit columns;
 *   lambda_PI = max_j q_j of the last sweep; the block is scaled by s = 2 * lambda_PI.
 * pool: number of start vectors, 1..32 (the paper uses 16 or 32).  sweeps >= 1: passes over
 * the block.  start_vectors: DEVICE pointer, row-major [rows][pool] fp32, rows >= the B of
 * later calls (their first B rows are used), shared by all blocks; drawn by the caller
 * (e.g. seeded N(0,1)); must stay valid while the setting is in use.  The blocks are taken to be
 * symmetric: the product is evaluated as (V^T A)^T, which for an input that is not exactly
 * symmetric is the power iteration of A^T (same spectrum).  Since R_A(v) <= lambda_max, s can be below lambda_max
 * when the pool has not converged: Newton-DB still converges as long as lambda_max < 2 s
 * (its scalar map converges on (0, 3)), otherwise it diverges and the block is flagged. */
dash_status dash_set_power_iteration(dash_ctx* ctx, int pool, int sweeps, const float* start_vectors, int rows);

/* ---- the batched matmul primitive (the paper's `bmm`, Sections 3.1 and 4.1) ------ */

/* C_i <- alpha * op(A_i) * op(B_i) + beta * D_i + gamma * I   for i in [0, N).
 * op(X) = X or X^T per trans flag (0/1).  A, Bm, D, C: dev [N][B][B].  D may be NULL
 * when beta == 0 and may be the same pointer as C (in-place accumulate); C must not
 * overlap A or Bm. */
dash_status dash_gemm_batched(dash_ctx* ctx, int transA, int transB,
                              const float* A, const float* Bm, const float* D, float* C,
                              int64_t N, int B, float alpha, float beta, float gamma,
                              dash_precision precision);

/* ---- Algorithm 1, EMA lines ------------------------------------------------------ */

/* L_i <- beta * L_i + alpha * G_i G_i^T,  R_i <- beta * R_i + alpha * G_i^T G_i.
 * The paper uses alpha = 1 - beta.  G: dev const [N][B][B]; L, R: dev in/out [N][B][B]
 * (they may be the two halves of one [2N][B][B] stack, Section 4.1 "stack"). */
dash_status dash_accumulate_factors(dash_ctx* ctx, const float* G, float* L, float* R,
                                    int64_t N, int B, float beta, float alpha);

/* ---- ragged blocks and 1-D parameters (Section 4.1) ----------------------------------- */

/* block() of Section 4.1 for one row-major layer W [m][n] with block size B: with Nm = m / B,
 * Nn = n / B (integer division), rm = m mod B, rn = n mod B the layer splits into
 *   full     [Nm*Nn][B][B]   block (i, j) at index i*Nn + j, W rows i*B.., columns j*B..
 *   row_rest [Nn][rm][B]     the last rm rows            (the paper's G_rest for the embedding)
 *   col_rest [Nm][B][rn]     the last rn columns         (the classification head's case)
 *   corner   [1][rm][rn]
 * A pointer may be null when its group is empty.  Bit-exact copies; any m, n, B (16-byte
 * accesses when n, B, rn are multiples of 4).  dash_unblock_layer is the inverse (stack -> W).
 * All pointers: device. */
dash_status dash_block_layer(dash_ctx* ctx, const float* W, int64_t m, int64_t n, int B,
                             float* full, float* row_rest, float* col_rest, float* corner);
dash_status dash_unblock_layer(dash_ctx* ctx, float* W, int64_t m, int64_t n, int B,
                               const float* full, const float* row_rest, const float* col_rest,
                               const float* corner);
/* The same with the rest extents rounded up inside the stacks: with pm = rm rounded up to a multiple of pad_m
 * and pn = rn rounded up to a multiple of pad_n the groups are row_rest [Nn][pm][B], col_rest [Nm][B][pn],
 * corner [1][pm][pn]; blocking fills the padding with zeros, unblocking ignores it.  pad_m, pad_n >= 1 must
 * divide B.  Zero rows and columns of a gradient block change nothing in the part of its factors, roots and
 * update that belongs to the real entries (the factors stay block diagonal, the padded diagonal block is
 * eps I), which is how layers of any shape go through the product kernels (block edges multiples of 64). */
dash_status dash_block_layer_padded(dash_ctx* ctx, const float* W, int64_t m, int64_t n, int B, int pad_m, int pad_n,
                                    float* full, float* row_rest, float* col_rest, float* corner);
dash_status dash_unblock_layer_padded(dash_ctx* ctx, float* W, int64_t m, int64_t n, int B, int pad_m, int pad_n,
                                      const float* full, const float* row_rest, const float* col_rest,
                                      const float* corner);

/* A layer whose dimensions are not multiples of B leaves "rest" gradient blocks of shape Bm x Bn
 * (the paper's example: (2, 256, 1024) with L_rest (2, 256, 256) and R_rest (2, 1024, 1024)).
 *   L_i <- beta L_i + alpha G_i G_i^T,  R_i <- beta R_i + alpha G_i^T G_i
 * G: dev const [N][Bm][Bn]; L: dev in/out [N][Bm][Bm]; R: dev in/out [N][Bn][Bn]; Bm, Bn multiples
 * of 64.  The roots of L and R are ordinary square stacks for dash_inverse_root. */
dash_status dash_accumulate_factors_rect(dash_ctx* ctx, const float* G, float* L, float* R,
                                         int64_t N, int Bm, int Bn, float beta, float alpha);
/* U_i <- Linv_i G_i Rinv_i with Linv [N][Bm][Bm], G and U [N][Bm][Bn], Rinv [N][Bn][Bn].
 * Needs workspace for one [N][Bm][Bn] temporary (or chunks of it). */
dash_status dash_precondition_rect(dash_ctx* ctx, const float* Linv, const float* G, const float* Rinv,
                                   float* U, int64_t N, int Bm, int Bn);

/* Normalisation layers: N vectors of B entries each (a layer of size E gives E/B of them); only
 * the left factor exists.  L_i <- beta L_i + alpha g_i g_i^T;  u_i <- Linv_i g_i (the paper uses
 * the inverse square root, p = 2, here).  g, u: dev [N][B]; L, Linv: dev [N][B][B]. */
dash_status dash_accumulate_vector(dash_ctx* ctx, const float* g, float* L, int64_t N, int B,
                                   float beta, float alpha);
dash_status dash_precondition_vector(dash_ctx* ctx, const float* Linv, const float* g, float* u,
                                     int64_t N, int B);

/* ---- Section 3.4 scaling --------------------------------------------------------- */

/* s_i = ||A_i + eps I||_F (Frobenius), tr(A_i + eps I) (trace), 1 (none) or 2 lambda_PI
 * (power iteration).  A: dev const [N][B][B]; s_out: dev [N].  Needs a workspace. */
dash_status dash_block_norms(dash_ctx* ctx, const float* A, int64_t N, int B, float eps,
                             dash_scaling scaling, float* s_out);

/* dash_block_norms for callers that cannot allocate and have no workspace to hand over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit for bit
 * the same s_out as dash_block_norms, but the slab partial sums go to a 2 MiB array that is part of the
 * library's device image (one copy per GPU, held until the process ends) instead of the context's workspace:
 * no workspace is needed and the call allocates nothing.  Limits: N <= 16384 blocks (DASH_ERR_INVALID_ARG
 * beyond that); scaling Frobenius, trace or none (DASH_ERR_UNSUPPORTED for power iteration, whose pool
 * vectors need a workspace).  Every call on one GPU, from any context, uses that GPU's one array: calls that
 * overlap in time on one GPU (different streams or contexts) race; calls on one stream are ordered.  Nothing
 * has to be cleared between calls (each call writes every partial sum before it reads it). */
dash_status dash_block_norms_static(dash_ctx* ctx, const float* A, int64_t N, int B, float eps,
                                    dash_scaling scaling, float* s_out);

/* ---- inverse roots (Section 3.3 Newton-DB; Appendix A Chebyshev) ----------------- */

/* X_i <- approximately (A_i + eps I)^(-1/p), p in {2, 4}.
 *   Steps: A_d = A + eps I; s = norm(A_d) per `scaling`; A_s = A_d / s;
 *          X = s^(-1/p) * root(A_s).
 *   DASH_NEWTON_DB: `iters` >= 1 updates of (Y, Z) per call, the first in closed form
 *          (E_1 = 3/2 I - 1/2 A_s, Y_1 = A_s E_1, Z_1 = E_1); p = 4 chains two calls
 *          (first keeps Y, second keeps Z) with `iters` updates each and no rescaling
 *          in between.  cheb_* arguments are ignored.
 *   DASH_CHEBYSHEV: `iters` is the degree d >= 2; cheb_coeffs is a HOST array of d+1
 *          doubles (c_0..c_d, e.g. from dash_chebyshev_fit); the scaled block is mapped
 *          with S = (2 A_s - (a+b) I) / (b-a) for [a,b] = [cheb_a, cheb_b], then the
 *          reduced Clenshaw recurrence (d-1 matmuls) is evaluated.
 *   DASH_COUPLED_NEWTON (Section 3.2): X_0 = I/c, M_0 = A_s/c^p, C_k = (1+1/p) I - M_k/p,
 *          X_{k+1} = X_k C_k, M_{k+1} = C_k^p M_k with c = (1+p)^(-1/p); `iters` >= 1
 *          iterations; fp32, fp16 or bf16 operands (the paper runs it in fp32 and fp16 and
 *          reports that bf16 diverges).  The scale must
 *          be strictly above lambda_max (at a scaled eigenvalue of exactly 1 the iteration
 *          is stuck at 0); Frobenius, trace and 2 lambda_PI are.
 *   A: dev const [N][B][B]; X: dev out [N][B][B], must not overlap A.
 *   scale_out: dev [N] receiving s_i, or NULL.  nonfinite_out: dev int32 [N], set to 1
 *   for every block whose result holds a NaN/Inf and to 0 otherwise, or NULL.
 *   Needs a workspace (dash_set_workspace). */
dash_status dash_inverse_root(dash_ctx* ctx, const float* A, float* X, int64_t N, int B,
                              dash_method method, int p, int iters, float eps,
                              dash_scaling scaling, dash_precision precision,
                              const double* cheb_coeffs, double cheb_a, double cheb_b,
                              float* scale_out, int32_t* nonfinite_out);

/* Host-only: coefficients c_0..c_d of the Chebyshev series of x^(-1/p) on [a, b], fitted
 * at n_points Chebyshev nodes as in Appendix A.1 (cosine sums, c_0 halved), in double.
 * coeffs_out: host array of degree+1 doubles.  Needs no context and no GPU. */
dash_status dash_chebyshev_fit(int p, int degree, double a, double b, int n_points,
                               double* coeffs_out);

/* ---- Algorithm 1, update direction ------------------------------------------------ */

/* U_i <- Linv_i * G_i * Rinv_i.  All dev [N][B][B]; U must not overlap the inputs.
 * Needs workspace for one [N][B][B] temporary (or chunks of it). */
dash_status dash_precondition(dash_ctx* ctx, const float* Linv, const float* G,
                              const float* Rinv, float* U, int64_t N, int B);

/* ---- Section 2.3 block-wise Adam grafting ------------------------------------------ */

/* Acc <- beta_g Acc + (1-beta_g) G.G ; P = G / (eps_g + sqrt(Acc)) ;
 * s_i = ||P_i||_F / ||U_i||_F ; theta_i <- theta_i - lr * s_i * U_i.
 * G, U: dev const [N][B][B]; Acc, theta: dev in/out [N][B][B]; s_out: dev [N] or NULL.
 * theta may be NULL (then only Acc and s_out are produced). */
dash_status dash_graft_update(dash_ctx* ctx, const float* G, const float* U, float* Acc,
                              float* theta, int64_t N, int B, float beta_g, float eps_g,
                              float lr, float* s_out);
/* The same grafting on blocks of any shape, given as `elems` contiguous floats per block (a multiple of 4;
 * of 32 from 4096 on, of 128 from 65536 on): Acc is updated, s_i computed, and U_scaled_i <- s_i U_i written
 * (U_scaled may equal U, or be NULL).  Used for ragged blocks and vectors (Section 4.1). */
dash_status dash_graft_scale(dash_ctx* ctx, const float* G, const float* U, float* Acc, int64_t N,
                             int64_t elems, float beta_g, float eps_g, float* U_scaled, float* s_out);
/* theta <- theta - lr * update over n floats (Algorithm 1, parameter update); any n >= 0,
 * both pointers dev, 16-byte aligned. */
dash_status dash_apply_update(dash_ctx* ctx, float* theta, const float* update, int64_t n, float lr);

/* ---- one optimizer step (Algorithm 1 on a stack) ----------------------------------- */

typedef struct {
    const float* G;      /* dev const [N][B][B] gradient blocks                         */
    float* S;            /* dev in/out [2N][B][B]: L blocks then R blocks               */
    float* X;            /* dev [2N][B][B]: roots of the damped factors; written when
                            refresh != 0, read (cached roots, Section 4.1) otherwise    */
    float* U;            /* dev out [N][B][B] preconditioned update                     */
    int64_t N;           /* gradient blocks                                             */
    int32_t B;
    float beta, alpha;   /* EMA weights (paper: alpha = 1 - beta)                       */
    float eps;           /* damping                                                     */
    int32_t method;      /* dash_method                                                 */
    int32_t p;           /* 2 or 4                                                      */
    int32_t iters;       /* Newton-DB updates per call, or Chebyshev degree             */
    int32_t scaling;     /* dash_scaling                                                */
    int32_t precision;   /* dash_precision                                              */
    int32_t refresh;     /* 0: skip the inverse roots and use X as given                */
    const double* cheb_coeffs; /* host, degree+1 doubles (Chebyshev only)               */
    double cheb_a, cheb_b;
    int32_t* nonfinite_out;    /* dev int32 [2N] or NULL                                */
    /* grafting (all optional: graft != 0 switches it on) */
    int32_t graft;
    float* graft_acc;    /* dev in/out [N][B][B]                                        */
    float* theta;        /* dev in/out [N][B][B] or NULL                                */
    float beta_g, eps_g, lr;
} dash_step_args;

/* accumulate into S -> (if refresh) inverse roots of all 2N blocks of S into X ->
 * U = X_L G X_R -> (if graft) grafted update.  args: host pointer. */
dash_status dash_step(dash_ctx* ctx, const dash_step_args* args);

/* ---- all layers of a GPU in shared stacks (Section 4.1, the variant the paper calls DashGpu) ---- */

/* The blocks of every layer are bucketed by shape and every factor of one size, whatever layer or side
 * it belongs to, sits in one stack: a step is one block() per layer, one accumulate and one precondition
 * per bucket, and ONE inverse-root call per factor size (for the paper's embedding example:
 * stack(L_full, R_full, R_rest) of 126 blocks of 1024 and L_rest of 2 blocks of 256).  Between refreshes
 * (the paper's recomputation frequency f > 1) the stored roots are reused.
 * A layer is m x n row-major; n = 0 marks a 1-D parameter (normalisation layer) of m entries, which is cut
 * into vectors of B entries with a left factor only and root p_vec (the paper uses 2).  Layers of any
 * shape are accepted: rest extents (m mod B, n mod B) that are not multiples of 64 are rounded up to the next
 * one inside the model's stacks, zero filled (see dash_block_layer_padded); dash_model_get_bucket reports the
 * padded block shapes. */
typedef struct { int64_t m, n; } dash_layer_shape;
typedef struct dash_model dash_model;
typedef struct {
    int32_t n_layers, n_buckets, n_stacks, B;
    int64_t n_gradient_blocks, n_factor_blocks;
    int64_t arena_bytes;        /* device memory the model needs: factors, roots, staging of G and U,
                                   and the grafting accumulators */
} dash_model_info;

/* Host-side planning only; the model keeps ctx (which must outlive it).  ctx may be NULL for a model that
 * is only described (dash_model_get_*), never stepped.  p, p_vec in {2, 4}. */
dash_status dash_model_create(dash_ctx* ctx, const dash_layer_shape* layers, int n_layers, int B,
                              int p, int p_vec, dash_model** out);
dash_status dash_model_destroy(dash_model* model);
const char* dash_model_last_error(const dash_model* model);
dash_status dash_model_get_info(const dash_model* model, dash_model_info* info);
/* bucket i: block shape (bn = 0: vectors of bm entries) and number of blocks; any output may be null */
dash_status dash_model_get_bucket(const dash_model* model, int i, int32_t* bm, int32_t* bn, int64_t* count);
/* factor stack i: block edge, root, number of blocks, and (once the arena is set, else null) the device
 * addresses of its factors S [count][size][size] and roots X; any output may be null */
dash_status dash_model_get_stack(const dash_model* model, int i, int32_t* size, int32_t* p, int64_t* count,
                                 float** S, float** X);
/* workspace the context needs for dash_model_step with this method / precision (a smaller one makes the
 * inverse root and the rectangular precondition run in chunks) */
size_t dash_model_workspace_bytes(const dash_model* model, dash_method method, dash_precision precision);
/* Caller-owned device memory of at least arena_bytes, 256-byte aligned; the caller zeroes it once
 * (factors start at zero) and keeps it for the life of the model: it is the optimizer state. */
dash_status dash_model_set_arena(dash_model* model, void* dev_ptr, size_t bytes);

typedef struct {
    const float* const* grads;  /* host array [n_layers] of device pointers, layer l: [m][n] (or [m]) */
    float* const* updates;      /* host array [n_layers] of device pointers, same shapes: U per layer */
    float beta, alpha, eps;
    int32_t method, iters, scaling, precision;
    int32_t refresh;            /* 0: skip the inverse roots and precondition with the stored ones */
    const double* cheb_coeffs;  /* as in dash_inverse_root */
    double cheb_a, cheb_b;
    int32_t* nonfinite_out;     /* dev [n_factor_blocks] in stack order, or NULL */
    int32_t graft;              /* 1: block-wise Adam grafting (Section 2.3): updates become s_b U_b */
    float beta_g, eps_g;
    float* const* thetas;       /* host array [n_layers] of device pointers or NULL: theta_l -= lr * update_l */
    float lr;
} dash_model_step_args;

dash_status dash_model_step(dash_model* model, const dash_model_step_args* args);

#ifdef __cplusplus
}
#endif
#endif /* DASH_H */

/*
 * strp.h -- C ABI of libstrp.so: the per-module ADMM subproblem of STRUPRUNE on one MI355X.
 *
 * One transformer module is resident at a time.  For an FFN module of decoder layer l, with T
 * calibration tokens (all matrices row-major, tokens are the contiguous axis of every activation):
 *     X     [d x T]  input of fc1  (a^pre_{l-1})        W1hat [f x d]  pre-trained fc1
 *     Z, Z0 [f x T]  auxiliary / dense pre-activation    W2hat [d x f]  pre-trained fc2
 *     A     [f x T]  auxiliary post-activation (the "p" variable of the problem statement)
 *     Y     [d x T]  dense module output (z^pre_{l+1})
 * A structured unit j is hidden neuron j (row j of W1 and column j of W2); for attention the unit
 * is a head, i.e. `group` consecutive channels.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name ends in _host.  The caller owns all
 *     buffers, including the workspace; the library never allocates or frees device memory.
 *   - Calls enqueue work on the stream given to strp_create and return; argument errors are
 *     reported synchronously (nothing is enqueued), numeric failures (non-positive Cholesky
 *     pivot; NaN, Inf or a magnitude above 65504 in an activation that a scoring reduction or an
 *     operand-plane writer reads: such a value is clamped and the results are meaningless) are
 *     recorded in a device status word read by strp_poll and by strp_admm_step when it fills its report.
 *   - Leading dimensions are in elements; activation leading dimensions must be multiples of 8
 *     and base pointers 16-byte aligned.  Padding columns (index >= T) are never read as data
 *     and never written.
 *   - Inputs may be bf16 or fp32; auxiliaries, Gram matrices and refitted weights are fp32;
 *     reductions that feed scores, factors and solves run in fp64.
 */
#ifndef STRP_H
#define STRP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  STRP_OK = 0,
  STRP_EINVAL = 1,     /* bad argument (null pointer, k > n, n % group != 0, ld < T, misalignment) */
  STRP_ENOMEM = 2,     /* workspace missing or too small                                        */
  STRP_ENOTPD = 3,     /* Cholesky met a non-positive pivot                                      */
  STRP_ENONFINITE = 4, /* NaN/Inf, or a magnitude above 65504 (the fp16 operand range), in an input       */
  STRP_EHIP = 5,       /* a HIP runtime call failed                                               */
  STRP_ESTATE = 6      /* call sequence error (e.g. admm_step before module_init)                 */
} strp_status;

typedef enum { STRP_BF16 = 0, STRP_F32 = 1 } strp_dtype;
typedef enum { STRP_SCORE_WANDA = 0, STRP_SCORE_LEMMA = 1, STRP_SCORE_GAIN = 2 } strp_score_mode;
typedef enum { STRP_SIDE_FC1 = 0, STRP_SIDE_FC2 = 1 } strp_side;
/* How fp32 operands enter the fp16 matrix cores: rounded once to fp16 (FAST, 2^-12 relative) or as a two-term
 * fp16 split hi + lo with the three leading cross products hi*hi + hi*lo + lo*hi (SPLIT, ~2^-22 relative).
 * The setting is captured by strp_module_init together with the operand planes it writes; strp_admm_step on that
 * module returns STRP_ESTATE if the context's precision has been changed since (initialise the module again). */
typedef enum { STRP_PREC_FAST = 0, STRP_PREC_SPLIT = 1 } strp_precision;

/* The six token-sized products of one strp_admm_step iteration (C = P Q over the named contraction):
 *   GRAM  G  = A_S A_S^T          RHS2  R2 = Y A_S^T            RHS1  R1 = Z_S X^T        (over the tokens)
 *   RESID E  = Y - W2_S relu(Z_S) AUPD  A_S = relu(Z_S) + B E   ZUPD  Z1 = W1_S X         (over channels)
 * P is the first factor named, Q the second. */
typedef enum { STRP_PROD_GRAM = 0, STRP_PROD_RHS2 = 1, STRP_PROD_RHS1 = 2, STRP_PROD_RESID = 3, STRP_PROD_AUPD = 4,
               STRP_PROD_ZUPD = 5, STRP_PROD_COUNT = 6 } strp_product;

typedef struct strp_ctx strp_ctx;

/* Context: host object holding the device id, the caller's stream and the workspace. */
strp_status strp_create(strp_ctx** out, int device, void* hip_stream);
strp_status strp_destroy(strp_ctx* ctx);
const char* strp_last_error(const strp_ctx* ctx);
strp_status strp_set_precision(strp_ctx* ctx, strp_precision prec);
/* Under STRP_PREC_SPLIT: how many fp16 planes (1 = hi only, 2 = hi + lo) of its P and of its Q operand one product
 * of strp_admm_step multiplies; an operand that exists as one plane only (a bf16 input) is not affected.  2 x 2 runs
 * three matrix-core passes per product, 2 x 1 and 1 x 2 two, 1 x 1 one.  Defaults: see the table in the library's
 * design notes (the cheapest setting whose free-running error stays below a quarter of the 2e-3 tolerance).
 * Errors: STRP_EINVAL. */
strp_status strp_set_product_planes(strp_ctx* ctx, strp_product product, int32_t planes_p, int32_t planes_q);
/* Caller-owned scratch used by every entry point below (256-byte aligned). */
strp_status strp_set_workspace(strp_ctx* ctx, void* dev_ptr, size_t bytes);
/* Synchronise the stream and return the device status word (STRP_OK, STRP_ENOTPD, ...). */
strp_status strp_poll(strp_ctx* ctx);

/* Optional per-kernel timing (HIP events on the context's stream), for benchmarks and profiles.
 * strp_profile_enable(ctx, on) clears the records and switches recording on or off;
 * strp_profile_read synchronises the stream and returns one aggregated entry per kernel class:
 * launches, total milliseconds, algorithmic flops and algorithmic bytes.  out_host is HOST memory. */
typedef struct {
  char name[48];
  int32_t launches;
  double ms;
  double flops;
  double bytes;
} strp_profile_entry;
strp_status strp_profile_enable(strp_ctx* ctx, int on);
strp_status strp_profile_read(strp_ctx* ctx, strp_profile_entry* out_host, int32_t max_entries, int32_t* n_out);
/* The same records one by one, in the order the work was enqueued (launches = 1 in every entry; at most
 * max_entries of them): lets an external kernel trace be matched to the library's kernel classes. */
strp_status strp_profile_launches(strp_ctx* ctx, strp_profile_entry* out_host, int32_t max_entries, int32_t* n_out);

/* ---- module description shared by the stateful entry points ------------------------- */
typedef struct {
  int32_t d, f;        /* widths                                                            */
  int64_t T;           /* calibration tokens                                                */
  int64_t ldx;         /* leading dimension of X                                            */
  int64_t lda;         /* leading dimension of Z, A, Z0, Y (fp32)                           */
  int32_t x_dtype;     /* strp_dtype of X                                                   */
  int32_t w_dtype;     /* strp_dtype of W1hat, W2hat                                        */
  int32_t k_max;       /* largest number of kept units any call will use (0: f)            */
} strp_module_desc;

/* Bytes of workspace sufficient for every entry point on this module (pure function). */
size_t strp_workspace_bytes(const strp_module_desc* desc);
/* Bytes of the per-module plane cache (strp_module_state::cache); pure function. */
size_t strp_module_cache_bytes(const strp_module_desc* desc);

/*
 * strp_gram -- calibration Gram matrix over the tokens (the X X^T / a a^T that W = z a^+ needs;
 * Appendix A.1 "Reversely recovering the weight matrix", Alg. 4 first step).
 *   G[i, j] (+)= sum_{t<T} A[r_i, t] * A[r_j, t],   r_i = idx ? idx[i] : i,   i, j < s.
 * A: [C x ldA] of dtype dt (row-major).  idx: s ascending row indices (device) or NULL (s == C).
 * G: [s x ldG] fp32, full symmetric matrix written.  diag (optional): [s] fp64 diagonal of G.
 * accumulate != 0 adds to the existing G (token-chunk accumulation).
 * Errors: STRP_EINVAL (null A/G, s <= 0, s > C, ldA < T, ldG < s, misaligned), STRP_ENOMEM.
 */
strp_status strp_gram(strp_ctx* ctx, const void* A, strp_dtype dt, int32_t C, int64_t T, int64_t ldA,
                      const int32_t* idx, int32_t s, float* G, int32_t ldG, double* diag, int accumulate);

/*
 * strp_score_alloc -- structural unit scores of one module and (optionally) the softmax sparsity
 * allocation over all modules (Lemma 1 and eq. (wanda) for the scores; Lemma 2 and Alg. 1
 * steps 1-2 for the allocation).
 *
 * Part 1 (always): per channel j < n_channels the token sums
 *     g = sum A^2, e = sum A*relu(Z0), u = sum Z0*Z, v = sum Z0^2   (e, u, v only for LEMMA/GAIN)
 * and n2_j = sum_i What[i, j]^2 give P = u + n2*e, Q = v + n2*g and
 *     WANDA: n2*g     LEMMA: sum_group P / sum_group Q     GAIN: sum_group (2P - Q)
 * summed over `group` consecutive channels per unit.  unit_score[n_channels/group] (fp32) and
 * energies[layer_idx] = mean unit score (fp64) are written.
 *
 * Part 2 (iff r_out != NULL): for each softmax group (group_id, or one group if NULL)
 *     w = softmax(-(I/mean|I|)/temperature), r = rbar*L_g*w, clip [0, rmax], rescale by rbar/mean(r)
 *     if nothing sits at rmax, clip again; prune counts by largest-remainder rounding of r*n_units
 *     (total = round(sum r*n), each layer keeps >= 1 unit).
 * r_out[L] fp64 = pruned fractions, nprune_out[L] int32.
 */
typedef struct {
  const void* A;       /* [n_channels x ld] post-activation auxiliary (or head outputs)      */
  int32_t a_dtype;     /* strp_dtype of A                                                    */
  const float* Z;      /* [n_channels x ld] or NULL (WANDA)                                  */
  const float* Z0;     /* [n_channels x ld] or NULL (WANDA)                                  */
  int64_t ld;
  int64_t T;
  int32_t n_channels;
  int32_t group;       /* channels per unit (1: neurons, d_head: heads)                      */
  int32_t mode;        /* strp_score_mode                                                    */
  const double* n2;    /* [n_channels] squared column norms of What, or NULL to compute them */
  const void* What;    /* [w_rows x ldw] next linear layer (used iff n2 == NULL)             */
  int32_t w_dtype;
  int32_t w_rows;
  int64_t ldw;
} strp_score_in;

strp_status strp_score_alloc(strp_ctx* ctx, const strp_score_in* in, float* unit_score, double* energies,
                             int32_t layer_idx, int32_t L, const int32_t* n_units, const int32_t* group_id,
                             double rbar, double temperature, double rmax, double* r_out,
                             int32_t* nprune_out);

/*
 * strp_weight_energy -- weight-only layer importance (Alg. 2, step 1), one parameter group per call:
 *   *energy += scale * ( |W|_1 + var_coef * Var(W) + l2_coef * |W|_2 )
 * over every entry of the n_mats matrices listed (a head's slices of the attention matrices, or one fc
 * matrix): |W|_1 = sum of absolute values, Var = population variance, |W|_2 = Euclidean norm of the entries.
 * The listing's attention term is (var_coef, l2_coef) = (0.1, 0.01) per head with scale = gamma^l * rho, its
 * MLP term (0.05, 0) per fc matrix with scale = gamma^l; a layer's importance is the sum of its groups' calls.
 *   mats: HOST array of descriptors; each W is a DEVICE pointer, row-major [rows x ld], ld >= cols.
 *   energy: DEVICE double, accumulated (zero it first).  Needs 6 KiB of the context's workspace.
 * Errors: STRP_EINVAL, STRP_ENOMEM (no workspace).
 */
typedef struct strp_weight_ref {
  const void* W;
  int32_t dtype;     /* strp_dtype */
  int32_t rows, cols;
  int64_t ld;
} strp_weight_ref;
strp_status strp_weight_energy(strp_ctx* ctx, const strp_weight_ref* mats, int32_t n_mats, double var_coef,
                               double l2_coef, double scale, double* energy);

/*
 * strp_alloc_inverse -- temperature-guided inverse weighting (Alg. 2, step 2) over energies[L] (device):
 * per softmax group (group_id, NULL = one group) w = softmax(-I / T) with the energies divided by the group's
 * mean |I| (the same scale-free temperature as strp_score_alloc), r_l = clip(rbar * L_g * (1 - w_l) /
 * sum_j (1 - w_j), 0, rmax); a group of one layer gets rbar.  nprune_out: largest-remainder integer counts of
 * r_l * n_units[l] per group, every layer keeping at least one unit.  All arrays are device arrays of length L.
 * Errors: STRP_EINVAL.
 */
strp_status strp_alloc_inverse(strp_ctx* ctx, const double* energies, int32_t L, const int32_t* n_units,
                               const int32_t* group_id, double rbar, double temperature, double rmax,
                               double* r_out, int32_t* nprune_out);

/*
 * strp_alloc_softmax -- the softmax sparsity allocation of Lemma 2 / Alg. 1 step 2 on its own, over energies[L]
 * (device) that earlier strp_score_alloc calls have filled: exactly what strp_score_alloc runs when it is given
 * n_units (r_l = clip(rbar * L_g * softmax(-I / T)_l, 0, rmax) per softmax group with the energies divided by the
 * group's mean |I|, the rescale branch when nothing was clipped, largest-remainder integer counts, every layer
 * keeping at least one unit).  For a driver that scores the modules once and then walks a temperature grid.
 * All arrays are device arrays of length L.  Errors: STRP_EINVAL.
 */
strp_status strp_alloc_softmax(strp_ctx* ctx, const double* energies, int32_t L, const int32_t* n_units,
                               const int32_t* group_id, double rbar, double temperature, double rmax,
                               double* r_out, int32_t* nprune_out);

/*
 * strp_mask_topk -- structured mask by score threshold (rule below Lemma 1; Alg. 4 threshold step).
 * Keeps exactly the k highest of the n unit scores; equal scores keep the lower index.
 *   mask[n] uint8 in {0,1};  idx[k*group] int32 ascending kept CHANNEL indices (unit*group + c);
 *   tau (optional) = lowest kept score.
 * One module's scores (n up to 65536) are selected by one block; a longer vector -- the scores of every layer
 * at once for the single global threshold of Alg. 4 (K = floor(r n L) kept over all L n units) -- is selected
 * by a multi-block path that needs strp_topk_workspace_bytes(n) bytes of the context's workspace (group must
 * be 1 there).
 * Errors: STRP_EINVAL (k < 0, k > n, n <= 0, group <= 0, null pointers), STRP_ENOMEM (workspace).
 */
strp_status strp_mask_topk(strp_ctx* ctx, const float* score, int32_t n, int32_t k, int32_t group,
                           uint8_t* mask, int32_t* idx, float* tau);
/* Workspace (bytes, device) that strp_mask_topk needs for n scores; 0 when one block handles them. */
size_t strp_topk_workspace_bytes(int32_t n);

/*
 * strp_mask_topk_static -- strp_mask_topk (group = 1) for callers that cannot allocate or hand over device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results
 * (mask, ascending idx, tau) and the same argument meaning; the select's scratch (per-block histograms, candidate
 * lists, counters) is a fixed array inside the library instead of the context's workspace, so the call needs no
 * workspace and allocates nothing on the host or the device (it also records no profile entry).  The array takes
 * 16 * STRP_TOPK_STATIC_MAX_N + 8 MiB = 32 MiB of device memory on every GPU the library is used on, from the moment
 * the library is loaded until the process ends.
 * Limits: n <= STRP_TOPK_STATIC_MAX_N (enough for the 48 x 28672 unit scores of the largest configuration at once);
 * more returns STRP_EINVAL and nothing is enqueued.  All calls on one GPU share the one array, which keeps the last
 * call's contents (each call clears the counters it needs): calls that overlap in time on one GPU -- two contexts on
 * different streams -- race; serialise them.  Other errors as strp_mask_topk.
 */
#define STRP_TOPK_STATIC_MAX_N 1572864
strp_status strp_mask_topk_static(strp_ctx* ctx, const float* score, int32_t n, int32_t k, uint8_t* mask, int32_t* idx,
                                  float* tau);

/*
 * strp_refit -- closed-form ridge least-squares recovery of the surviving weights
 * (W = z a^+ restricted to the kept support; Appendix A.1, Alg. 3 prune+recover lines).
 *   R = Lhs_rows * Rhs_rows^T over the T tokens,  Wsub = R (Gram + lambda I)^-1.
 * side == STRP_SIDE_FC2:  Lhs [out x ld_lhs] (all rows), Rhs rows idx[0..s) of an [in x ld_rhs]
 *   matrix, Gram [s x s] = their Gram;  W[:, idx] = Wsub, every other column of W zero.
 * side == STRP_SIDE_FC1:  Lhs rows idx[0..s) of an [out x ld_lhs] matrix, Rhs [in x ld_rhs] (all
 *   rows), Gram [in x in];  W[idx, :] = Wsub, every other row of W zero.
 * Gram: fp32 symmetric, unregularised, leading dimension ldg.  W: [out x in] fp32, dense row-major.
 * chol (optional, fp64 [n x n], n = order of Gram): factorisation cache.  It holds L^-1, the inverse
 * of the lower Cholesky factor of Gram + lambda I (lower triangular, upper part zero).  If
 * chol_valid != 0 it comes from an earlier call and Gram is not read; otherwise it is computed and,
 * if chol != NULL, stored there for reuse.
 * Numeric failure (pivot <= 0) sets STRP_ENOTPD in the status word.
 */
strp_status strp_refit(strp_ctx* ctx, strp_side side, const float* Gram, int32_t ldg, double lambda,
                       double* chol, int chol_valid, const void* Lhs, strp_dtype lhs_dtype, int64_t ld_lhs,
                       const void* Rhs, strp_dtype rhs_dtype, int64_t ld_rhs, int64_t T, const int32_t* idx,
                       int32_t s, float* W, int32_t out, int32_t in);

/* ---- stateful per-module path ---------------------------------------------------------- */
typedef struct {
  const void* X;       /* [d x ldx]   x_dtype                                               */
  const void* W1hat;   /* [f x d]     w_dtype                                               */
  const void* W2hat;   /* [d x f]     w_dtype                                               */
  float* Z;            /* [f x lda]   auxiliary pre-activation                              */
  float* A;            /* [f x lda]   auxiliary post-activation                             */
  float* Z0;           /* [f x lda]   dense pre-activation (fixed)                          */
  float* Y;            /* [d x lda]   dense module output (fixed)                           */
  float* W1;           /* [f x d]     refitted fc1 (rows of pruned units zero)              */
  float* W2;           /* [d x f]     refitted fc2 (columns of pruned units zero)           */
  float* H;            /* [d x d]     X X^T                                                 */
  double* cholH;       /* [d x d]     inverse of the lower Cholesky factor of H + lam1 I    */
  double* n2;          /* [f]         squared column norms of W2hat                         */
  float* score;        /* [f]         unit scores of the last selection                     */
  uint8_t* mask;       /* [f]         1 = kept                                              */
  int32_t* idx;        /* [f]         kept indices ascending (first s valid)                */
  double* scalars;     /* [32]        device scalars: lam1, lam2, objective sums, tau       */
  void* cache;         /* strp_module_cache_bytes(desc) bytes, 256-byte aligned: fp16 operand planes of
                          X and Y written by strp_module_init and read by every later step, and the
                          cached scoring sums (see sums_cached)                                  */
  int32_t s;           /* kept units of the current mask (host field, set by the library)   */
  int32_t iter;        /* inner iterations done (host field)                                */
  int32_t sums_cached; /* host field, set by the library: which of the four token sums of the scores `cache` holds for
                          EVERY row of the current Z and A (bit 0: sum A^2; bit 1: sum A relu(Z0) and sum Z0 Z; bit 2:
                          sum Z0^2).  A full iteration leaves them there (the pruned rows' from the pass that writes those
                          rows, the kept rows' from the epilogues of the a- and z-update products), so the next selection
                          streams no row; strp_module_init clears it.  A caller that changes Z or A between iterations
                          must set this field to 0.                                                              */
  int32_t precision;   /* host field: 0 until strp_module_init has run on this state, then 1 + the strp_precision its
                          operand planes were written with; strp_admm_step refuses (STRP_ESTATE) to run on an
                          uninitialised state or under a different precision                                        */
} strp_module_state;

typedef struct {
  double alpha, beta;  /* weights of the objective                                          */
  double delta;        /* ridge damping: lam = delta * mean(diag Gram), fixed at init        */
  int32_t mode;        /* strp_score_mode used when selecting                               */
  int32_t reselect;    /* 0: select only when no mask exists yet; 1: every iteration        */
  int32_t k;           /* units to keep                                                     */
  int32_t stages;      /* bit mask of STRP_STAGE_*; 0 means all                              */
} strp_params;

enum {
  STRP_STAGE_SELECT = 1, /* scores + top-k                                                  */
  STRP_STAGE_REFIT2 = 2, /* Gram of kept A rows, fc2 refit                                  */
  STRP_STAGE_REFIT1 = 4, /* fc1 refit with the cached factor of H                           */
  STRP_STAGE_AUPD = 8,   /* a-update                                                        */
  STRP_STAGE_ZUPD = 16,  /* z-update                                                        */
  STRP_STAGE_OBJ = 32    /* objective                                                       */
};

typedef struct {
  double terms[5];     /* (1/T)[a|Y-W2A|^2, b|A-relu Z|^2, a|Z-W1X|^2, a lam2|W2|^2, a lam1|W1|^2] */
  double J;            /* first three terms                                                 */
  double J_ridge;      /* all five                                                          */
  double lam1, lam2;
  float tau;           /* lowest kept score of the last selection                           */
  int32_t s;
  int32_t status;      /* strp_status from the device status word                           */
} strp_report;

/*
 * strp_module_init -- Alg. 3 initialisation: Z0 = W1hat X, Z = Z0, A = relu(Z0), Y = W2hat A,
 * H = X X^T, lam1 = delta tr(H)/d, lam2 = delta |A|_F^2 / f, inverse Cholesky factor of H + lam1 I (the
 * cached pseudo-inverse of the listing), n2 = column norms of W2hat, W1 = W2 = 0, no mask.
 */
strp_status strp_module_init(strp_ctx* ctx, const strp_module_desc* desc, strp_module_state* st,
                             const strp_params* params);

/*
 * strp_admm_step -- one inner iteration of Alg. 3 (FFN function) / Alg. 4 step body on the resident
 * module: score + top-k (if due), fc2 refit, fc1 refit, a-update
 *     A = (alpha W2^T W2 + beta I)^-1 (alpha W2^T Y + beta relu(Z)),
 * z-update (exact per-element minimiser of beta(a - relu z)^2 + alpha(z - W1 x)^2) and the
 * objective.  report_host (optional) is filled after synchronising the stream.  The first objective term,
 * (alpha/T)|Y - W2 A|^2, is formed from Y - W2 A itself when the call does not include the a-update stage; when
 * it does, A is that update's exact minimiser and the same number is obtained as
 * (alpha/T)(beta/alpha)^2 <M^-2, E E^T>, E = Y - W2[:,S] relu(Z_S), M = (beta/alpha) I + W2[:,S] W2[:,S]^T
 * (Appendix A.1, "Updating activation": the normal equations of that step).
 */
strp_status strp_admm_step(strp_ctx* ctx, const strp_module_desc* desc, strp_module_state* st,
                           const strp_params* params, strp_report* report_host);

#ifdef __cplusplus
}
#endif
#endif /* STRP_H */

/*
 * libthanos -- Thanos block-wise post-training pruning of one linear layer on AMD MI355X
 * (gfx950).  C ABI; every kernel behind it is hand-written HIP.
 *
 * Notation follows the paper ("Formulation of the problem" and its notation table):
 *   W  in R^{c x b}   weight matrix, c output rows, b input columns, row-major, ld = b
 *   X                 calibration input.  The paper writes X in R^{b x a}; here it is held
 *                     token-major, Xc[t, j], t = token, j = input channel (ld = ldx >= b)
 *   H  in R^{b x b}   Hessian of the row-wise objective, H ~ X X^T (any positive scale)
 *   M  in {0,1}^{c x b}, M_ij = 1  <=>  W_ij is removed
 *   B  block size, p sparsity ratio, n:m = n zeros in every m consecutive weights of a row
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless it says "host".  The caller owns all
 *     buffers; the library allocates no device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All kernels are
 *     enqueued asynchronously and the call returns without waiting for the device; results are
 *     ordered after the call on `stream`.  thanos_factor and thanos_prune_layer run part of
 *     their work on helper streams (default priority; two for the factorisation, one for the
 *     sweep, one for the part of the sweep's preparation that can run beside the
 *     factorisation), forked from and joined back into `stream` with events.  These host-side HIP
 *     objects are the only state the library keeps: a call borrows them from a per-process pool
 *     (created on first use per device, one set per concurrently running call, never destroyed,
 *     because destroying a stream waits for it to drain).  On an error return every helper
 *     stream is joined into `stream` first, so work already enqueued is ordered before anything
 *     the caller enqueues on `stream` afterwards.  Calls may be issued from several host
 *     threads; the device current at the call must be the one `stream` belongs to.
 *   - The return value covers argument checks and launch errors only.  Numerical failure
 *     (a non-positive pivot) is reported through the device word `info_dev`, which the
 *     caller reads after synchronising the stream.
 *   - Matrices are dense row-major.  Pointers should be 16-byte aligned and b a multiple of
 *     8 for the vectorised paths; other shapes take slower scalar paths, not an error.
 */
#ifndef THANOS_H_
#define THANOS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  THANOS_OK = 0,
  THANOS_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, m does not divide B or b, ... */
  THANOS_ERR_UNSUPPORTED = 2, /* valid request outside what the kernels cover (see each call)  */
  THANOS_ERR_WORKSPACE = 3,   /* ws_bytes smaller than the matching *_workspace_bytes()         */
  THANOS_ERR_NOT_SPD = 4,     /* reserved for host-side callers that inspect info_dev           */
  THANOS_ERR_HIP = 5,         /* a HIP launch or runtime call failed                            */
  THANOS_ERR_TOO_LARGE = 6    /* thanos_prune_layer_noalloc: the problem needs more workspace
                                 than THANOS_NOALLOC_SCRATCH_BYTES                              */
} thanos_status;

typedef enum { THANOS_F32 = 0, THANOS_F16 = 1, THANOS_BF16 = 2 } thanos_dtype;
typedef enum { THANOS_UNSTRUCTURED = 0, THANOS_NM = 1, THANOS_STRUCTURED = 2 } thanos_mode;

/* Phases of thanos_prune_layer as reported through thanos_prune_opts.phase_ms_out. */
enum {
  THANOS_PHASE_PREP = 0,     /* weights to fp32, sqrt(xnorm2), outlier rows, block rows P_k of
                                the residual inverses                                          */
  THANOS_PHASE_FACTOR = 1,   /* damped factorisation (0 when factor_in is given)               */
  THANOS_PHASE_MASK = 2,     /* unstructured: the selection chain (threshold of the global
                                residual mask); n:m and given masks: 0, the choice is made
                                inside the solve kernels                                       */
  THANOS_PHASE_SOLVE = 3,    /* per-row systems lambda R_hat = u (with the block mask)         */
  THANOS_PHASE_UPDATE = 4,   /* trailing update W[:, j1:] -= Lambda P_k                        */
  THANOS_PHASE_FINALISE = 5, /* cast copy                                                      */
  THANOS_N_PHASES = 6
};

/* Options of the block sweep (host struct, read during the call only). */
typedef struct {
  int32_t mode;       /* THANOS_UNSTRUCTURED (Alg. 1), THANOS_NM (n:m algorithm, App. G.4.4) or
                         THANOS_STRUCTURED (Alg. 2: ceil(p*b/(1-alpha)) whole columns, those
                         of smallest loss v_j = (sum_i W_ij^2) H_jj over the non-outlier rows,
                         are removed from the non-outlier rows in one shot with the full
                         inverse Hessian; block_size, mask_in unused, factor_in rejected)       */
  double sparsity;    /* p in [0,1): r = floor(p*c*b) weights are removed (Alg. 1, problem
                         statement eq. (2)); p is read as the decimal it prints as, so 0.6
                         means 6/10.  Ignored for THANOS_NM.                                  */
  int32_t n, m;       /* THANOS_NM: n of every m consecutive weights of a row are removed;
                         0 < n < m <= 16, m divides block_size and b                          */
  int32_t block_size; /* B: columns pruned per sweep step, 1 <= B <= 4096.  A row's system of
                         one block must not exceed 2048 unknowns: B <= 2048 in general;
                         THANOS_NM without mask_in takes B <= 4096 with B*n/m <= 2048 (the whole
                         range of the block-size ablation in the Experiments section).  Systems
                         of up to 256 unknowns in blocks of up to 512 columns are solved out of
                         LDS; larger ones out of the workspace and markedly slower per unknown.
                         The last block may be narrower.                                       */
  float damping;      /* H_d = H + damping * mean(diag H) * I (relative damping, >= 0)        */
  const uint8_t* mask_in;  /* optional c*b device mask that replaces the selection step
                              (1 = remove); NULL = select as the paper does                   */
  const float* factor_in;  /* optional U (b*b) from thanos_factor for this H and damping;
                              NULL = factor inside the call                                   */
  const float* xnorm2_in;  /* required with factor_in: xnorm2 (b) from the same call          */
  double outlier_fraction; /* alpha in [0,1) of the n:m algorithm (App. G.4.4, Sec. 4.7 "Outlier
                              rows"): the ceil(alpha*c) rows with the largest loss
                              h_i = ||W_i X||^2 = W_i H W_i^T are left untouched (dense, mask 0);
                              ties by row index.  0 = prune every row.  THANOS_NM and
                              THANOS_STRUCTURED; needs H (undamped) even when factor_in is
                              given.                                                            */
  float* threshold_out;    /* optional, THANOS_UNSTRUCTURED without mask_in: ceil(b/B) floats
                              (device); entry j receives tau_j, the largest metric
                              |W_ik| * sqrt(xnorm2_k) that the global residual mask of block j
                              (psi_X over W[:, jB:b], Sec. 4.4) selects: entries below tau_j are
                              removed, entries equal to it in (row, column) order while the
                              budget r lasts.  -1 where nothing was left to remove.  NULL = not
                              reported.                                                         */
  float* phase_ms_out;     /* optional HOST pointer to THANOS_N_PHASES floats.  Diagnostic mode
                              (not THANOS_STRUCTURED): the kernels of the call run one after the
                              other on `stream` (no helper streams, hence no overlap), timing
                              events are recorded between the phases, the call WAITS for the
                              stream and writes the milliseconds of each phase.  Same results
                              as a normal call.  NULL = normal asynchronous call.               */
} thanos_prune_opts;

/*
 * Hessian accumulation, Alg. 1 step "H <- 2 X X^T" in its d-sample form (App. F.2): a sum of
 * Gram matrices over chunks of calibration tokens.
 *
 *   H[i, j] += alpha * sum_{t < n_tok} Xc[t, i] * Xc[t, j]      for i >= j
 *
 * H: b*b fp32, ld = b.  Only the lower triangle including the diagonal is defined on return;
 *    the strict upper triangle may or may not have been written.  The caller zeroes H before
 *    the first chunk.  Xc: [n_tok, b] of type xdt, row stride ldx elements, never modified.
 *    Products are exact (fp16/bf16 inputs) and accumulated in fp32 on the matrix cores.
 *    To keep every compute unit busy the token range of a tile may be split over several
 *    workgroups, whose partial sums are then added to H with fp32 atomics: the summation order,
 *    hence the last bits of H, can differ from run to run.
 * Errors: INVALID_ARG for NULL pointers, b <= 0, n_tok < 0, ldx < b, unknown xdt.
 *         n_tok == 0 is a no-op.
 */
thanos_status thanos_hessian_accumulate(float* H, int64_t b, const void* Xc, thanos_dtype xdt,
                                        int64_t n_tok, int64_t ldx, float alpha, void* stream);

/*
 * Damped factorisation.  Replaces the per-block re-inversion of the residual Hessian of
 * Alg. 1 ("H <- 2(XX^T)_{j2:b, j2:b}" followed by its inverse, cost O(b^4/B) in App. G.6) by
 * one factor that contains every one of those inverses:
 *
 *   xnorm2[j] = H[j, j]                              (undamped, ~ ||X_j:||^2 of the metric, Sec. 4.2)
 *   H_d       = H + damping * mean_j(H[j, j]) * I
 *   U upper triangular with  H_d^{-1} = U^T U, hence
 *   inv(H_d[j:, j:]) = U[j:, j:]^T U[j:, j:]   for every j.
 *
 * Reads the lower triangle of H (b*b, ld = b).  Writes U (b*b fp32, ld = b; strict lower
 * triangle set to 0) and xnorm2 (b).  U must not alias H.  ws: thanos_factor_workspace_bytes(b)
 * bytes of scratch.  info_dev: device int32; set to 0, or to k > 0 if the pivot of column k
 * (1-based; columns are eliminated from the last to the first) was not positive, in which
 * case U is meaningless.  Arithmetic: fp32 storage; matrix products are computed on the bf16
 * matrix cores from operands split into three bf16 terms each (six partial products summed in
 * fp32, error of the order of one fp32 rounding per product), everything else in plain fp32.
 */
thanos_status thanos_factor(const float* H, int64_t b, float damping, float* U, float* xnorm2,
                            void* ws, size_t ws_bytes, int32_t* info_dev, void* stream);
size_t thanos_factor_workspace_bytes(int64_t b);

/*
 * Column-block sweep: Alg. 1 (unstructured, global residual mask psi_X, Sec. 4.4) or the n:m
 * algorithm of App. G.4.4 (with its outlier rows when opts->outlier_fraction > 0); structured
 * pruning (Alg. 2) is reached through the same call.  For every block of B columns,
 * left to right: choose the block mask M from the metric |W_ij| * sqrt(xnorm2_j) of the
 * CURRENT weights, then for every row with q = phi(M_i:) (Sec. 4.5) solve lambda R_hat = u and
 * apply Delta = -u R_hat^{-1} R to all columns from the block start to b (Sec. 4.1, eqs. (R),
 * (R_hat), (u), (Delta)), with R the rows q of the inverse of the damped residual Hessian.
 * Removed weights are written as exact zeros.
 *
 * W_in: c*b of type wdt, ld = b, never modified.  H: b*b fp32 lower triangle (ignored when
 * opts->factor_in is given).  W_out: c*b fp32.  W_out_cast: NULL, or c*b of type wdt receiving
 * W_out rounded to nearest-even.  mask_out: c*b uint8, 1 = removed.  ws:
 * thanos_prune_workspace_bytes(c, b, opts) bytes.  info_dev: as in thanos_factor; in addition
 * it is set to -(i+1) if the system of row i met a non-positive pivot (that row's update is
 * then meaningless; other rows are unaffected).
 * Ties in the metric are broken by ascending (row, column).
 * Errors: INVALID_ARG (NULL, sizes, n/m/B constraints, p or alpha outside [0,1), alpha > 0
 * without H), UNSUPPORTED (block_size beyond the limits above, m > 16, alpha > 0 with
 * THANOS_UNSTRUCTURED or with mask_in, b > 65535, c > 2^24, THANOS_STRUCTURED with c > 65535),
 * WORKSPACE, HIP.
 */
thanos_status thanos_prune_layer(const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                                 const float* H, const thanos_prune_opts* opts /* host */,
                                 float* W_out, void* W_out_cast, uint8_t* mask_out, void* ws,
                                 size_t ws_bytes, int32_t* info_dev, void* stream);
size_t thanos_prune_workspace_bytes(int64_t c, int64_t b, const thanos_prune_opts* opts /* host */);

/*
 * thanos_prune_layer for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * thanos_prune_layer, without ws / ws_bytes: the workspace is a static device array of
 * THANOS_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.
 * The call allocates nothing on the device or through HIP: no hipMalloc / hipFree, and no helper
 * streams or events either (all kernels go to `stream` in one order; the overlap of
 * thanos_prune_layer's helper streams is given up, the results are the same).  The first call on
 * a device looks up that device's copy of the array (hipGetSymbolAddress, which may load the
 * library's code on the device); the device current at the call must be the one `stream` and
 * the buffers belong to.
 * opts->phase_ms_out must be NULL (the diagnostic mode creates events): UNSUPPORTED otherwise.
 * Limit: thanos_prune_workspace_bytes(c, b, opts) <= THANOS_NOALLOC_SCRATCH_BYTES, else
 * THANOS_ERR_TOO_LARGE and nothing is enqueued (e.g. c = b = 1536 at B = 128 fits, with
 * opts->factor_in c = b = 2048 does).
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents (the
 * kernels initialise what they read): calls that overlap on one GPU -- from two threads, or on
 * two streams without an ordering between them -- race.  Not re-entrant per device.
 */
#define THANOS_NOALLOC_SCRATCH_BYTES (64u << 20)
thanos_status thanos_prune_layer_noalloc(const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                                         const float* H, const thanos_prune_opts* opts /* host */,
                                         float* W_out, void* W_out_cast, uint8_t* mask_out,
                                         int32_t* info_dev, void* stream);

/* Static, NUL-terminated description of a status code (host pointer, never freed). */
const char* thanos_status_string(thanos_status s);

#ifdef __cplusplus
}
#endif
#endif /* THANOS_H_ */

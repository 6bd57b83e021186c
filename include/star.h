/*
 * libstar -- group-synchronous parameter update of STAR (arXiv 2512.09685) on
 * one MI355X (gfx950).
 *
 * A parameter server holds one shard of the parameters.  Each parameter
 * update is fed by a *worker group*: all workers (SSGD), any one worker
 * (ASGD), x workers (static x-order mode) or one cluster of workers with
 * similar iteration times (dynamic x-order mode) -- Section 1 items (2) and
 * (4), Section 4.2.  The server aggregates the group's gradient copies and
 * updates its parameter copy (Section 2, parameter-server description).  This
 * library runs a stream of U such updates over one shard of P parameters in a
 * single pass over HBM.
 *
 * One update u with group G_u (y_u distinct worker ids), on every element j:
 *     gbar_u[j] = sum_{w in G_u} c_{u,w} * g_w[j]
 *     d         = gbar_u[j] + weight_decay * p[j]
 *     v[j]      = momentum * v[j] + d
 *     p[j]      = p[j] - lr_u * v[j]
 * (the SGD of PyTorch, the framework the paper names in Section 5.1:
 * dampening 0, no Nesterov, decay coupled into the gradient), and optionally
 *     norms_out[u] = || gbar_u ||_2        (before weight decay)
 * the per-group gradient norm (gradient-norm progress signal, Sections 4.3.1
 * and 7).  c_{u,w} = 1/y_u (STAR_W_MEAN), 1/(y_u (1+s_{u,w})) with staleness
 * s (STAR_W_STALE, not renormalised) or a caller-given value (STAR_W_EXPLICIT).
 * With scale_lr_by_group the rate of update u is lr_u * y_u / W: the learning
 * rate scaled in proportion to the number of gradient reports (Section 4.3.1,
 * "Scaling learning rate after switching").
 *
 * Arithmetic on the device is fp32 with fused multiply-add, members summed in
 * ascending worker id; gradients may be fp32 or bf16 (widened exactly to
 * fp32).  Results do not depend on the order in which a group lists its
 * members.  Params and momentum are bitwise reproducible from run to run.
 * The norms are accumulated in fp32 within a tile of 1024 elements, in a
 * fixed order, and in double from there on; on long shards the tiles reach
 * the workgroups in a different order on every run, which moves the double
 * sums at the 1e-16 level; the fp32 results change only if a sum lies that
 * close to a rounding boundary of fp32 (about once in 1e9 values).
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory of the current device, "host"
 *     pointers ordinary host memory.  The caller owns every buffer; the
 *     library neither frees nor keeps them.  Host arrays and structs are
 *     consumed before the call returns.
 *   - Work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream);
 *     the call does not wait for that work.  Outputs are valid after the
 *     stream has been synchronised.  Two things can make the host wait inside
 *     a call all the same: (1) the internal workspace is a ring of 8 slots,
 *     one per call that needs tables, partial sums or the tile queue, each
 *     guarded by an event; the ninth such call blocks (hipEventSynchronize)
 *     until the work of the call that used its slot eight calls earlier has
 *     finished; (2) the first call that needs a larger workspace than any
 *     before it allocates device and pinned memory (hipMalloc, hipHostMalloc),
 *     which synchronises the device.  star_group_update_noalloc does neither.
 *   - The return value is a star_status.  Nothing is thrown, nothing aborts.
 *     All argument checks precede the first enqueue: on a status other than
 *     STAR_OK and STAR_ERR_DEVICE no device memory has been modified.
 *   - P == 0 or U == 0 is a valid no-op (norms of an empty shard are 0).
 *   - Gradient rows may alias each other; they must not alias params,
 *     momentum or norms_out.  Rows are read-only during the call.
 *   - Any alignment is accepted; when params, momentum and all rows are
 *     16-byte aligned the vector path is used, otherwise an element-wise path
 *     with the same arithmetic (identical results).
 *   - The library keeps a small internal workspace (coefficient tables,
 *     per-block norm partials, a 16-byte work queue per slot), created on
 *     first use, released by star_shutdown().  Calls may come from several
 *     host threads.
 */
#ifndef STAR_H
#define STAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STAR_MAX_WORKERS 32

typedef enum {
    STAR_OK = 0,
    STAR_ERR_NULL = 1,   /* a required pointer is NULL                                        */
    STAR_ERR_SHAPE = 2,  /* P < 0, W < 1, W > STAR_MAX_WORKERS, U < 0                          */
    STAR_ERR_GROUP = 3,  /* empty group, id outside [0,W), duplicate id, offsets not monotone  */
    STAR_ERR_HPARAM = 4, /* non-finite lr / momentum / weight decay / coefficient, negative
                            staleness, unknown weighting mode                                   */
    STAR_ERR_DTYPE = 5,  /* unknown gradient dtype                                             */
    STAR_ERR_KERNEL = 6, /* unknown kernel choice in star_options                              */
    STAR_ERR_DEVICE = 7  /* a HIP call failed; text via star_last_error()                      */
} star_status;

typedef enum { STAR_F32 = 0, STAR_BF16 = 1 } star_dtype;

typedef enum {
    STAR_W_MEAN = 0,    /* c = 1/y                    */
    STAR_W_STALE = 1,   /* c = 1/(y (1+s))            */
    STAR_W_EXPLICIT = 2 /* c = coeff[] as given       */
} star_wmode;

/* How the U updates are evaluated on the device (both give the same result up
 * to fp32 rounding; see star_plan_affine). */
typedef enum {
    STAR_KERNEL_AUTO = 0,  /* the library chooses (star_plan_choice tells what): a single update on fp32
                              rows SEQ, and with norms any stream of up to 48 multiply-adds per element
                              on a short shard (4 Mi elements, bf16 rows 16 Mi; 17 to 32 fp32 rows: 112,
                              any length); otherwise the collapsed map; with norms the Gram matrix on the
                              matrix cores (vector registers instead: up to 6 rows, and 7 or 8 rows below
                              16 Mi elements; but 3 to 8 bf16 rows up to 8 Mi elements, and most shards of 4 to
                              6 bf16 rows below 48 Mi: matrix cores),
                              except that coefficients of both signs and short streams on 17 to 32 fp32
                              rows get direct norm sums                                                  */
    STAR_KERNEL_SEQ = 1,   /* update by update, gradients held in registers; norms from direct sums of
                              gbar_u^2                                                                   */
    STAR_KERNEL_AFFINE = 2, /* the U updates collapsed into one affine map of (p, v, g_0..g_W-1); the Gram
                               matrix behind the norms in vector registers up to 16 rows             */
    STAR_KERNEL_AFFINE_MFMA = 3 /* the same map, the Gram matrix formed on the matrix cores for any number
                                   of rows                                                            */
} star_kernel;

/* star_options.flags.  STAR_OPT_DIRECT_NORMS: where the library would take the norms from the Gram
 * matrix of the rows (relative error up to 2e-8 kappa_u, see star_group_update), take them from direct
 * sums of gbar_u^2 instead, to fp32-product accuracy whatever the rows: in a pass of its own over the
 * rows beside the collapsed update (W more row reads per element), as the library does by itself for
 * coefficients of both signs.  For rows that may be anti-correlated.  Ignored when `kernel` forces an
 * evaluation (STAR_KERNEL_SEQ always sums directly) and by calls that return no norms. */
#define STAR_OPT_DIRECT_NORMS 1

/*
 * Per-call options of the *_opt entry points (host struct, read before the
 * call returns).  All zero = the defaults; a NULL pointer means the same.
 * Nothing here changes what is computed, only how (both evaluations and both
 * tile orders give the same params and momentum up to fp32 rounding, see
 * star_plan_affine), so these are tuning and test switches.  There is no
 * process-wide setting: two callers in one process may use different options
 * at the same time.  The environment variable STAR_KERNEL=seq|affine|
 * affine_mfma, read once at load time, replaces STAR_KERNEL_AUTO for calls
 * that do not choose themselves.
 */
typedef struct {
    int32_t kernel;          /* star_kernel; STAR_KERNEL_AUTO = the library chooses                    */
    int32_t flags;           /* 0 or STAR_OPT_DIRECT_NORMS; any other bit: STAR_ERR_SHAPE              */
    int64_t queue_threshold; /* shards of at least this many elements are processed by long-lived
                                workgroups that claim tiles (1024 consecutive elements of every
                                buffer) in address order from a work queue; shorter ones get a fixed
                                assignment, which starts faster.  0 = default (updates: 16 Mi elements
                                with fp32 rows, 64 Mi with up to 4 of them; with bf16 rows 64 Mi, 96 Mi
                                with up to 12 of them, 128 Mi with up to 4; updates with norms on up to
                                6 rows: 16 Mi with bf16 rows, 32 / 64 / 128 Mi with 1 / 2 / 3-6 fp32 rows; norms
                                and Gram matrix alone 16 Mi; the aggregation 64 Mi, and never with up
                                to 8 bf16 or 4 fp32 rows or with several groups of bf16 rows); 1 = always
                                the queue; negative:
                                STAR_ERR_SHAPE                                                          */
} star_options;

/* The stream of updates of one call (all arrays on the host).  Group u is
 * members[offsets[u] .. offsets[u+1]).  (Worker group: Section 1 item (4).) */
typedef struct {
    int32_t U;
    const int32_t *offsets;   /* [U+1], offsets[0] == 0, strictly increasing            */
    const int32_t *members;   /* [offsets[U]] worker ids in [0, W)                      */
    const int32_t *staleness; /* [offsets[U]] or NULL (= all 0); used by STAR_W_STALE   */
    const float *coeff;       /* [offsets[U]]; required by, and only used by, STAR_W_EXPLICIT */
    const float *lr;          /* [U] learning rate of each update, or NULL -> hp.lr     */
} star_updates;

typedef struct {
    float lr;                  /* used when star_updates.lr is NULL                      */
    float momentum;
    float weight_decay;
    int32_t wmode;             /* star_wmode                                             */
    int32_t scale_lr_by_group; /* nonzero: lr_u *= y_u / W  (Section 4.3.1)              */
} star_hparams;

/*
 * Run U group updates on one shard (Sections 1, 2, 4.2; formulas above).
 *   params, momentum : device, float[P], updated in place.
 *   grad_rows        : host array of W device pointers; row w holds worker w's
 *                      gradient for this shard, P elements of grad_dtype.
 *                      Rows no group references are never read (may be NULL).
 *   norms_out        : device float[U], or NULL when norms are not wanted.
 * Precision of the norms.  For a stream of two or more updates they are derived
 * from the Gram matrix of the rows, n_u^2 = c_u^T Gamma c_u (one pass whatever
 * U is).  That form is as accurate as its terms are free of cancellation: the
 * relative error of n_u is at most 2e-8 * kappa_u,
 *     kappa_u = (sum_w |c_{u,w}| ||g_w||)^2 / n_u^2,
 * which lies between 1 and y_u <= 32 for non-negative weights on rows that are
 * not anti-correlated (every weighting of the paper: at most 6.4e-7, observed
 * 1e-7 and less) and grows without bound when a group's weighted sum nearly
 * cancels (measured at kappa = 4e4: 2.6e-6 with the vector-register Gram
 * matrix, 1.8e-5 with the matrix-core one).  With coefficients of both signs (STAR_W_EXPLICIT) the library
 * therefore takes the norms from direct sums of gbar_u^2 in a pass of its
 * own (error 1e-6 or less, one more read of the rows), and so it does on
 * shards of fewer than 4096 elements, where a group's sum over so few
 * elements cancels as a matter of course; star_options.flags =
 * STAR_OPT_DIRECT_NORMS asks for the same on any stream (the update stays the
 * collapsed one), and star_options.kernel = STAR_KERNEL_SEQ evaluates update
 * and norms step by step.
 * Non-finite gradient values propagate: params and momentum of an element turn
 * non-finite when a member of any group holds inf or NaN there (inf may come
 * out as NaN), and norms_out[u] is non-finite exactly for the groups with such
 * a member.
 */
star_status star_group_update(float *params, float *momentum, const void *const *grad_rows,
                              star_dtype grad_dtype, int64_t P, int32_t W, const star_updates *upd,
                              const star_hparams *hp, float *norms_out, void *hip_stream);

/*
 * star_group_update for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels, same results.  Where star_group_update keeps
 * its tables, per-workgroup partial sums and tile queue in a workspace it
 * allocates on first use, this entry point keeps them in a fixed array of
 * STAR_NOALLOC_SCRATCH_BYTES that is part of the library's device code (every
 * GPU the library runs on holds one copy until the process ends), and carries
 * the group tables to it in kernel arguments.  It calls no hipMalloc, hipFree,
 * hipHostMalloc, event or copy routine, and enqueues kernels only (no memset,
 * no copy), so a call can be captured into a HIP graph and replayed; make one
 * ordinary call on the device first (the array's address is resolved on first
 * use).
 *   - at most STAR_NOALLOC_MAX_UPDATES updates per call; a longer stream is
 *     rejected with STAR_ERR_SHAPE before anything is enqueued (split it over
 *     several calls, the state carries over).
 *   - all calls on one GPU share that GPU's array: two calls of this entry
 *     point whose work overlaps in time on one GPU (different streams, or
 *     different host threads) race on it.  Calls on one stream are ordered and
 *     safe; so are calls on different GPUs.  It never conflicts with the other
 *     entry points, which do not touch the array.
 */
#define STAR_NOALLOC_MAX_UPDATES 256
#define STAR_NOALLOC_SCRATCH_BYTES (4608 * 1024)
star_status star_group_update_noalloc(float *params, float *momentum, const void *const *grad_rows,
                                      star_dtype grad_dtype, int64_t P, int32_t W, const star_updates *upd,
                                      const star_hparams *hp, float *norms_out, void *hip_stream);

/*
 * star_group_update that also writes a copy of the updated parameters for the
 * "send the updated parameters to the workers" leg (Section 2): after the U
 * updates, publish[j] = params[j] converted to publish_dtype (fp32: the same
 * bits; bf16: round to nearest even), written in the same pass, so the send
 * buffer costs no extra read of params.
 *   publish : device, P elements of publish_dtype; must not alias any other
 *             buffer of the call.  With U == 0 nothing is written.
 */
star_status star_group_update_publish(float *params, float *momentum, const void *const *grad_rows,
                                      star_dtype grad_dtype, int64_t P, int32_t W, const star_updates *upd,
                                      const star_hparams *hp, float *norms_out, void *publish,
                                      star_dtype publish_dtype, void *hip_stream);

/*
 * Per-group gradient norms only: norms_out[u] = || sum_w c_{u,w} g_w ||_2
 * (gradient-norm signal, Sections 4.3.1 and 7).  Arguments as above; wmode is
 * a star_wmode.  No parameter state is read or written.
 */
star_status star_group_norms(const void *const *grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                             const star_updates *upd, int32_t wmode, float *norms_out, void *hip_stream);

/*
 * Aggregation without the optimizer step: for every group u,
 *     out_rows[u][j] = sum_{w in G_u} c_{u,w} g_w[j]            (j = 0 .. P-1)
 * This is what a parent computes from its children's gradients and its own
 * before broadcasting in the all-reduce architecture (Section 4.2, "All-reduce
 * architecture"), and what a node of the communication tree forwards upward
 * (Section 4.4.2, tree-based communication).  One pass: every referenced row is
 * read once, every output written once.
 *   out_rows  : host array of U device pointers, each P elements of out_dtype
 *               (fp32, or bf16 rounded to nearest even).  Outputs must not
 *               alias the gradient rows or each other.
 *   norms_out : device float[U] (|| out_u ||_2 computed from the fp32 sums,
 *               before any rounding to bf16), or NULL.
 * Other arguments and all conventions as for star_group_update.
 */
star_status star_group_reduce(void *const *out_rows, star_dtype out_dtype, const void *const *grad_rows,
                              star_dtype grad_dtype, int64_t P, int32_t W, const star_updates *upd, int32_t wmode,
                              float *norms_out, void *hip_stream);

/*
 * Host-only: the U updates of a stream written as one affine map,
 *     (p_U, v_U)^T = M (p_0, v_0)^T + B (g_0 .. g_{W-1})^T,
 * composed in double precision.  M is row-major 2x2, B row-major 2xW.  Touches
 * no device.  This is what STAR_KERNEL_AFFINE evaluates (after rounding the
 * entries to fp32, M[0] as M[0]-1).  Same validation and status codes as
 * star_group_update.
 */
star_status star_plan_affine(int32_t W, const star_updates *upd, const star_hparams *hp, double M[4], double *B);

/*
 * Host-only: what star_group_update (update = 1) or star_group_norms
 * (update = 0) would launch for this call, decided by the same code that
 * launches it; buffers are taken to be 16-byte aligned.
 */
typedef struct {
    int32_t kernel;       /* star_kernel of the main kernel: STAR_KERNEL_SEQ (step-by-step), STAR_KERNEL_AFFINE
                             (collapsed map; Gram matrix behind the norms, if any, in vector registers) or
                             STAR_KERNEL_AFFINE_MFMA (collapsed map, Gram matrix on the matrix cores)       */
    int32_t grad_dtype;   /* the star_dtype asked about                                                     */
    int32_t rows_used;    /* gradient rows referenced by at least one group (only these are read)           */
    int32_t rows_padded;  /* row count the kernel is instantiated for (extra rows carry zero coefficients)  */
    int32_t queue_order;  /* 1: tiles claimed from the work queue, 0: fixed assignment                       */
    int32_t launches;     /* launches of the main kernel the stream is split into (1 unless step-by-step)   */
    int32_t finishing_launches; /* small kernels after the main one (norm reduction, norms from the Gram matrix) */
    int32_t tables_inline;      /* 1: group tables travel in the kernel arguments, 0: staged through the workspace
                                   (the collapsed map without norms needs no tables at all and reports 1)   */
    int32_t collapsed_update;   /* 1: params and momentum come from the one affine map of the stream.  Always so
                                   with AFFINE and AFFINE_MFMA; with SEQ only for 17 to 32 fp32 rows, update
                                   with norms and a short stream (direct norm sums of at most 4 W + 48
                                   multiply-adds per element), where the step-by-step kernel walks the updates
                                   for the norms alone (direct sums are cheaper there than the Gram matrix)   */
    int32_t reserved;
    double fma_seq;       /* fused multiply-adds per element of the step-by-step evaluation                 */
    double fma_affine;    /* ... and of the collapsed one (vector-register Gram counted as FMAs)            */
} star_plan_info;

star_status star_plan_choice(int64_t P, int32_t W, star_dtype grad_dtype, const star_updates *upd,
                             const star_hparams *hp, int32_t update, int32_t want_norms,
                             const star_options *opt, star_plan_info *info);

/*
 * Gram matrix of the gradient rows, Gamma[a][b] = sum_j g_a[j] g_b[j], the
 * quantity the per-group norms are derived from (|| sum_w c_w g_w ||^2 =
 * c^T Gamma c) and the input of the noise-scale estimate below.
 *   grad_rows : host array of W device pointers, all used; 1 <= W <= 32
 *   gram_out  : device double[W*W], row-major, symmetric
 * One pass over the rows; products and per-thread sums in fp32, across
 * workgroups in fp64.
 */
star_status star_group_gram(const void *const *grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                            double *gram_out, void *hip_stream);

/*
 * The entry points above with per-call options (star_options; NULL = defaults).
 * star_group_update_opt covers star_group_update (publish == NULL) and
 * star_group_update_publish.  Everything else as documented above.
 */
star_status star_group_update_opt(float *params, float *momentum, const void *const *grad_rows,
                                  star_dtype grad_dtype, int64_t P, int32_t W, const star_updates *upd,
                                  const star_hparams *hp, float *norms_out, void *publish,
                                  star_dtype publish_dtype, const star_options *opt, void *hip_stream);
star_status star_group_norms_opt(const void *const *grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                                 const star_updates *upd, int32_t wmode, float *norms_out,
                                 const star_options *opt, void *hip_stream);
star_status star_group_reduce_opt(void *const *out_rows, star_dtype out_dtype, const void *const *grad_rows,
                                  star_dtype grad_dtype, int64_t P, int32_t W, const star_updates *upd,
                                  int32_t wmode, float *norms_out, const star_options *opt, void *hip_stream);
star_status star_group_gram_opt(const void *const *grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                                double *gram_out, const star_options *opt, void *hip_stream);

/*
 * Host-only: gradient noise scale from the Gram matrix of W workers' gradients
 * of one step (the gradient-norm progress signal the paper lists as future
 * work, Section 7; the simple noise scale tr(Sigma)/|G|^2, i.e. the PGNS of
 * Section 4.3.1 with the identity as pre-conditioner).  Model: g_w = G + e_w,
 * e_w independent, zero mean, covariance Sigma / batch_per_worker.  Then
 *   E mean_w |g_w|^2 = |G|^2 + tr(Sigma)/b,   E |mean_w g_w|^2 = |G|^2 + tr(Sigma)/(W b),
 * and solving the two for the unknowns gives the unbiased estimates
 *   trace_cov = b (S - n2) W/(W-1),  grad_sq = (W n2 - S)/(W-1),  noise_scale = trace_cov / grad_sq,
 * S = mean of the diagonal of Gamma, n2 = sum of all entries of Gamma / W^2.
 *   gram : host double[W*W] (copy of star_group_gram's output); 2 <= W <= 32.
 * Any of the three outputs may be NULL.  grad_sq can come out negative when
 * the noise dominates; noise_scale is then negative or huge and means "unknown".
 */
star_status star_noise_scale(int32_t W, const double *gram, double batch_per_worker, double *grad_sq,
                             double *trace_cov, double *noise_scale);

/* ---- STAR-H: heuristic choice of the synchronization mode (host only) ---- */

typedef enum {
    STAR_MODE_SSGD = 0,      /* every update uses all N workers                    */
    STAR_MODE_ASGD = 1,      /* every update uses one worker                       */
    STAR_MODE_STATIC_X = 2,  /* every update uses x workers, 1 < x < N             */
    STAR_MODE_DYNAMIC_X = 3  /* one update per cluster of workers of similar speed */
} star_mode;

typedef struct {
    int32_t mode;            /* star_mode                                                    */
    int32_t x;               /* workers per update of the static modes (N: SSGD, 1: ASGD); 0 for dynamic */
    int32_t n_groups;        /* groups written to group_offsets / group_members              */
    int32_t n_stragglers;    /* workers with d_i above the straggler threshold               */
    int32_t n_clusters;      /* clusters the dynamic mode would use                          */
    double time_to_progress; /* T of the chosen mode                                         */
} star_mode_choice;

/*
 * Parameter-server architecture (Section 4.3.1).  From the predicted iteration
 * times of the N workers, the noise scale phi of the current step and the
 * total batch size M:  T_x = (1 + phi/(x M/N)) t_x for x = 1..N (Eq. 1),
 * T_d = 1 / sum_i 1/((1 + phi/(n_ci M/N)) t_ci) over the clusters of workers
 * with similar times (Eq. 2), and the mode with the least time.  A worker is a
 * straggler when (T_i - min T)/min T > straggler_threshold (Section 2; the
 * paper uses 0.2); without any straggler the choice is SSGD.
 * t_x is taken as the x-th smallest iteration time (the time by which x
 * gradient reports have arrived); clusters come from
 * complete-linkage agglomerative clustering that merges while the merged
 * range relative to its fastest member is within cluster_threshold.
 *   iter_time     : host double[N], predicted iteration times (> 0)
 *   choice        : host, result
 *   time_static   : host double[N] or NULL, receives T_x at [x-1]
 *   time_dynamic  : host double* or NULL, receives T_d
 *   group_offsets : host int32[N+1], group_members : host int32[N]: the groups
 *                   of the chosen mode, fastest group first, in the format of
 *                   star_updates (use scale_lr_by_group for the rate rule).
 *   is_straggler  : host int32[N] or NULL.
 * Errors: STAR_ERR_NULL, STAR_ERR_SHAPE (N outside [1, STAR_MAX_WORKERS]),
 * STAR_ERR_HPARAM (non-positive or non-finite times, batch, thresholds, phi < 0).
 */
star_status star_select_mode_ps(int32_t N, const double *iter_time, double phi, double batch_total,
                                double straggler_threshold, double cluster_threshold, star_mode_choice *choice,
                                double *time_static, double *time_dynamic, int32_t *group_offsets,
                                int32_t *group_members, int32_t *is_straggler);

/*
 * All-reduce architecture (Section 4.3.1, Eq. 3): remove the x slowest
 * workers (x at most the number of stragglers) from the ring, let parents wait
 * t_w, and minimise T_a = (1 + phi/((N-x+q) M/N)) (t_ring + t_w) over x and the
 * candidate waits; t_ring is the slowest remaining ring worker, q the removed
 * workers whose new iteration time child_time[k] is no higher than t_w.
 * x = 0 (the plain ring, no wait) is always a candidate.
 *   child_time      : host double[N], iteration time of worker k if removed
 *   wait_candidates : host double[n_wait]
 *   removed_out, wait_out, time_out : chosen x, t_w and T_a
 *   time_table      : host double[1 + X*n_wait] or NULL: T_a of the plain ring,
 *                     then of (x, wait index) row by row, X = stragglers.
 */
star_status star_select_mode_ar(int32_t N, const double *iter_time, const double *child_time, double phi,
                                double batch_total, double straggler_threshold, int32_t n_wait,
                                const double *wait_candidates, int32_t *removed_out, double *wait_out,
                                double *time_out, double *time_table);

/*
 * Host-only: the fixed first round of the work queue for a launch of
 * `workgroups` workgroups that claim `tiles_per_claim` tiles at a time (the
 * kernels use 3; 5 when a thread moves less than 96 bytes per tile; 4 with the
 * half-size workgroups of the collapsed update on 24 and more bf16 rows).
 * Workgroup b starts on tiles first_tile[b] .. first_tile[b] + count[b] - 1
 * (counts cycle 1, 2, .., tiles_per_claim: unequal on purpose, so that the
 * workgroups do not run in step); the tiles from *base on are handed out by
 * the queue's counter.  first_tile and count hold `workgroups` entries.
 * STAR_ERR_SHAPE for workgroups < 1 or tiles_per_claim < 1, STAR_ERR_NULL for
 * a NULL output.
 */
star_status star_plan_claims(int32_t workgroups, int32_t tiles_per_claim, int64_t *first_tile, int32_t *count,
                             int64_t *base);

/*
 * Host-only: the tiles of a short shard under a launch in queue order (the
 * matrix-core kernel runs in that order at every length).  Up to 8 tiles per
 * workgroup (16 with light tiles; 48 or 128 for launches that only read: norms
 * or Gram matrix alone) the queue's counter is not used at all: workgroup b of
 * `workgroups` handles the consecutive tiles first_tile[b] .. first_tile[b] +
 * count[b] - 1 = [b tiles / workgroups, (b+1) tiles / workgroups), an even
 * split (counts differ by at most one) that covers every tile once.  With so
 * few tiles the unequal first claims above would give some workgroups twice
 * the work of others, and the counter's round trips would show in a kernel of
 * a few microseconds.  first_tile and count hold `workgroups` entries.
 * STAR_ERR_SHAPE for workgroups < 1 or tiles < 0, STAR_ERR_NULL for a NULL
 * output.
 */
star_status star_plan_even_split(int32_t workgroups, int64_t tiles, int64_t *first_tile, int32_t *count);

/* Bytes of internal device workspace one call of this shape uses. */
size_t star_workspace_bytes(int64_t P, int32_t W, int32_t U);

/* Text of the last error on the calling thread ("" if none). Never NULL. */
const char *star_last_error(void);

const char *star_version(void);

/* Waits for the library's own pending work and frees its workspace. */
void star_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* STAR_H */

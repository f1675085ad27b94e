/*
 * cdgrab.h -- C ABI of the MI355X (gfx950) CD-GraB pair-balancing library.
 *
 * The library implements the order-server hot path of CD-GraB (arXiv 2302.00845):
 * per-example gradients of m data-parallel workers -> pair differences ->
 * coordinated greedy sign balancing on one running sum -> next-epoch
 * permutations.  The m workers are a batch axis on one GPU.
 *
 * Conventions for every entry point
 *   - Pointers marked "dev" are device (HBM) addresses on the handle's device;
 *     pointers marked "host" are ordinary host addresses.  The caller owns every
 *     input and output buffer; inputs are never modified.  The handle owns its
 *     workspace (running sum, partial results, staging block).
 *   - Work is enqueued on the handle's HIP stream; a call returns once the work
 *     is enqueued unless stated otherwise.  The caller synchronises the stream
 *     before reading outputs.  Calls on one handle must not overlap.  The first
 *     call with a given shape allocates workspace (and may synchronise the stream
 *     to free a smaller one); later calls of cdgrab_pergrad and the balancing
 *     entry points with dense input enqueue kernels and device-to-device copies
 *     only, so they may be captured in a HIP graph.
 *   - Return value: CDGRAB_OK (0) or a negative error code.  After an error the
 *     contents of the outputs are undefined; cdgrab_last_error() gives a text.
 *   - Sizes are int64_t counts of elements, never bytes.
 */
#ifndef CDGRAB_H
#define CDGRAB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CDGRAB_OK 0
#define CDGRAB_EINVAL (-1) /* bad size, null required pointer, odd n, bad option   */
#define CDGRAB_ENOMEM (-2) /* workspace allocation failed                           */
#define CDGRAB_EHIP (-3)   /* a HIP runtime call failed (text in last_error)        */
#define CDGRAB_EGEN (-4)   /* the generator callback returned non-zero              */

typedef struct cdgrab_handle cdgrab_handle;

typedef struct cdgrab_options {
    int32_t device;      /* HIP device ordinal                                        */
    int32_t block_pairs; /* Bb: pairs resolved per HBM pass; 0 = choose, else 16, 32 or 64 */
    void *stream;        /* hipStream_t to enqueue on; NULL = the null stream         */
    int32_t timing;      /* 0 off; 1 record events around generator / balancer work;
                            2 additionally around every balancer kernel               */
    int32_t pass1_groups; /* workgroups of the dot/Gram pass; 0 = choose              */
    int32_t apply_mode;  /* how r += sum eps_k d_k of a block is launched: 1 = its own
                            apply launch after the block is resolved; 2 = inside the next
                            block's dot/Gram launch (one streaming launch per block, the
                            running sum read once per block); 0 = choose by row length.
                            3 / 4 = as 1 with the choice of the apply kernel taken away:
                            3 = always the kernel for long rows (a resident grid that updates
                            the running sum in one burst at the end of the launch), 4 = always
                            the flat kernel (one thread per four elements)                 */
    int32_t gram_mode;   /* dense input (and the staged rows of cdgrab_train_epoch_softmax).
                            1 = every block computes its Gram matrix in
                            its own dot/Gram launch; 2 = the Gram matrices of up to 512
                            blocks are computed ahead in one launch (they depend on the
                            rows only) and a block then costs one launch (the previous
                            block's resolver and apply, this block's dots); refused
                            (EINVAL) for d > 131 072; 0 = choose (2 for rows up to 16 384
                            elements when apply_mode is 0 as well)                        */
    int32_t apply_groups; /* cap on the workgroups of the resident apply kernel; 0 = two per CU */
} cdgrab_options;

/* Event-timed durations of the last cdgrab_balance_epoch call (timing >= 1);
 * the per-kernel fields are filled only with timing == 2.  Milliseconds. */
typedef struct cdgrab_timing {
    double generator_ms; /* time inside the generator callback's enqueued work */
    double balance_ms;   /* dot/Gram pass + reduce + resolve + apply pass, all blocks */
    double pass1_ms;     /* dot/Gram launches (including the fused apply of the previous block) */
    double reduce_ms;    /* partial reduction                                  */
    double resolve_ms;   /* sequential sign resolution                         */
    double pass2_ms;     /* stand-alone apply launches (only the last block's when fused) */
    double finish_ms;    /* permutation build + running-sum export             */
    int64_t blocks;      /* number of blocks processed                         */
    int32_t block_pairs; /* Bb used                                            */
    int32_t pass1_groups;/* workgroups used by the dot/Gram pass               */
} cdgrab_timing;

/* How one epoch is cut into blocks and launched (pure host arithmetic; needs no GPU). */
typedef struct cdgrab_plan {
    int64_t pairs;           /* m*n/2 flattened pair differences                      */
    int64_t blocks;          /* ceil(pairs / block_pairs)                             */
    int32_t block_pairs;     /* Bb                                                    */
    int32_t vector_width;    /* fp32 elements per global load: 4, 2 or 1              */
    int32_t tile_elems;      /* elements of d per LDS tile of the dot/Gram pass        */
    int32_t fused_apply;     /* 1: apply fused into the next block's dot/Gram launch (0 when
                                gram_ahead is 1: that form applies inside its own launch)  */
    int32_t pass1_groups;    /* workgroups of the dot/Gram pass                       */
    int32_t pass2_groups;    /* workgroups of the apply pass                          */
    int32_t gram_ahead;      /* 1: Gram matrices of many blocks computed ahead in one launch */
    int32_t reserved;
    int64_t workspace_bytes; /* everything the handle allocates for this epoch: running sum,
                                partials, slice sums, block signs, the buffers of the
                                Grams-ahead form when gram_ahead is 1, and staging          */
    int64_t staging_bytes;   /* staging blocks [Bb][2][d] fp32 (two when fused), 0 for dense input */
    double bytes_per_example;/* algorithmic HBM bytes per example: each row twice, plus the
                                double running sum per block: 8d + 12 d / Bb (read twice,
                                written once) or 8d + 8 d / Bb when fused; 12d + 8 d / Bb
                                with the Gram matrices computed ahead (rows read three times) */
} cdgrab_plan;

/* Generator callback for streamed input ("grads-or-generator").  It must enqueue,
 * on `stream`, work that fills staging[count][2][d] (fp32, dev) with the rows of
 * the flattened pairs first_pair .. first_pair+count-1: staging[q][0] is the
 * first row the worker visited of pair first_pair+q, staging[q][1] the second.
 * Flattened pair p belongs to worker p % m and is that worker's pair p / m
 * (step-major, worker-minor: the order in which the server algorithm of
 * Sec. 3.3 / App. C.1 visits pairs).  Return 0 on success. */
typedef int (*cdgrab_gen_fn)(void *ctx, int64_t first_pair, int64_t count,
                             float *staging /*dev*/, void *stream);

/* Create / destroy a handle.  `opt` may be NULL (device 0, null stream, automatic
 * block size, no timing).  Allocates nothing until the first call that needs
 * workspace.  Errors: EINVAL (bad option), EHIP (no such device). */
int cdgrab_create(cdgrab_handle **out, const cdgrab_options *opt);
int cdgrab_destroy(cdgrab_handle *h);

/* Text of the last error on this handle (owned by the handle, valid until the
 * next call on it).  With h == NULL: the text of the last failed cdgrab_create. */
const char *cdgrab_last_error(const cdgrab_handle *h);

/* The plan a handle with default options (apply_mode 0, gram_mode 0, pass1_groups 0)
 * follows on a 256-CU device for an epoch of m workers x n rows x d parameters;
 * a handle on another device, or with those options set, may choose differently.
 * `streamed` non-zero means rows come from a generator, one block per callback.
 * block_pairs 0 = automatic.  `base_align` is the byte alignment of the gradient base
 * pointer (16 for hipMalloc'ed memory).  Host only.  Errors: EINVAL. */
int cdgrab_plan_epoch(int64_t m, int64_t n, int64_t d, int32_t block_pairs,
                      int32_t streamed, int64_t base_align, cdgrab_plan *plan /*host*/);

/* Per-example gradients of softmax cross-entropy for a linear model: the vector a
 * worker sends for each example ("CD-GraB Workers", line 4; per-example gradients
 * as in footnote 2 of Sec. 2).
 *   X [N][in_dim] fp32 dev, y [N] int32 dev (0 <= y < classes, not checked),
 *   W [(in_dim+1)][classes] fp32 dev, last row is the bias,
 *   G_out [N][(in_dim+1)*classes] fp32 dev:
 *     delta = softmax(W^T [x;1]) - onehot(y);
 *     G_out[e][r*classes + c] = x_r * delta_c,  G_out[e][in_dim*classes + c] = delta_c.
 * fp32 arithmetic.  Errors: EINVAL (N<0, in_dim<1, classes<1 or >1024, null,
 * in_dim + 1 + classes > 16384: one example's staging must fit 64 KB of LDS). */
int cdgrab_pergrad(cdgrab_handle *h, int64_t N, int64_t in_dim, int64_t classes,
                   const float *X, const int32_t *y, const float *W, float *G_out);

/* One epoch of coordinated pair balancing (server algorithm of Sec. 3.3, lines
 * 3-14; one-step form App. C.1) with the deterministic greedy rule of App. B.2
 * ("Balancing without normalization").
 *
 *   running sum r = 0
 *   for pair k = 0 .. n/2-1, worker i = 0 .. m-1 (in this order):
 *       dvec = row(i, 2k+1) - row(i, 2k)          (second minus first)
 *       t    = <r, dvec>
 *       eps  = +1 if t <= 0 else -1               (the paper's sign for the first
 *                                                  row is -eps; a zero dot gives +1)
 *       r   += eps * dvec
 *   per worker: the row with sign +1 of each pair goes to the front list in pair
 *   order, the other to the back list, which is reversed:
 *       pi'[k] = 2k+1 if eps==+1 else 2k;  pi'[n-1-k] = the other;
 *       perm_out[i][p] = perm_in[i][pi'[p]]       (pi' itself if perm_in is NULL)
 *
 * Inputs: either `grads` [m][n][d] fp32 dev (row (i,j) = the j-th gradient worker i
 * produced this epoch) or, with grads == NULL, a generator callback that fills a
 * staging block owned by the handle.  Exactly one of the two must be given.
 *   perm_in   [m][n] int32 dev or NULL : example id at each visiting position
 *   signs_out [m][n/2] int8 dev        : eps per (worker, pair)
 *   perm_out  [m][n] int32 dev         : next epoch's order; must not overlap perm_in
 *                                        (to carry an order over, alternate two buffers)
 *   r_out     [d] fp32 dev or NULL     : final running sum, rounded from double
 *   r64_out   [d] fp64 dev or NULL     : final running sum in double
 *   dots_out  [m][n/2] fp64 dev or NULL: t seen when each pair was decided
 * Arithmetic: differences, dots, Gram entries and the running sum are IEEE double
 * (fp32 inputs); sums over d are taken in a fixed order, so results are
 * reproducible run to run.
 * Errors: EINVAL (m<1, n<2, n odd, d<1, null required pointer, both or neither of
 * grads / gen, perm_out overlapping perm_in), ENOMEM, EHIP, EGEN. */
int cdgrab_balance_epoch(cdgrab_handle *h, int64_t m, int64_t n, int64_t d,
                         const float *grads, cdgrab_gen_fn gen, void *gen_ctx,
                         const int32_t *perm_in, int8_t *signs_out,
                         int32_t *perm_out, float *r_out, double *r64_out,
                         double *dots_out);

/* cdgrab_balance_epoch for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same epoch
 * on dense input, with the workspace (running sum, per-workgroup partials, slice sums,
 * block signs) in a static device array of about 3.9 MB that each GPU the library runs
 * on holds until the process ends.  It calls no hipMalloc / hipFree and records no timing
 * events.  Rows of at most CDGRAB_STATIC_MAX_D elements; longer rows are refused (EINVAL).
 * It runs the per-block launch form with at most 128 workgroups in the dot/Gram pass, so
 * sums over d may be taken in another order than cdgrab_balance_epoch's (same result on
 * exactly representable input, otherwise equal to double rounding).
 * Arguments and outputs as cdgrab_balance_epoch with grads given (no generator).
 * All calls on one GPU share that GPU's array, whatever their handle: calls that overlap
 * in time on one GPU (two streams, two threads) race.  A call clears what it needs cleared.
 * Errors: EINVAL (as cdgrab_balance_epoch; grads NULL; d > CDGRAB_STATIC_MAX_D), EHIP. */
#define CDGRAB_STATIC_MAX_D 131072
int cdgrab_balance_epoch_static(cdgrab_handle *h, int64_t m, int64_t n, int64_t d,
                                const float *grads, const int32_t *perm_in, int8_t *signs_out,
                                int32_t *perm_out, float *r_out, double *r64_out,
                                double *dots_out);

/* The epoch of cdgrab_balance_epoch with the randomized sign rule of the analysis
 * (PairBalance with its RandomizedBalance subroutine, Sec. 3.2; the paper's
 * experiments use the greedy rule instead): for c = z1 - z2 the first row gets +1
 * with probability p = (1 - <r,c>)/2, so the exported sign is
 *     eps = -1 if u < (1 + t)/2 else +1,     t = <r, z2 - z1>,
 * with u the caller's draw for that pair (a p outside [0,1] decides by itself; the
 * rule is meant for vectors of norm <= 1).  Dense input only.
 *   uniforms [m][n/2] fp32 dev, each in [0,1); other arguments as cdgrab_balance_epoch.
 * Errors: as cdgrab_balance_epoch, EINVAL for a null uniforms. */
int cdgrab_balance_epoch_randomized(cdgrab_handle *h, int64_t m, int64_t n, int64_t d,
                                    const float *grads, const float *uniforms,
                                    const int32_t *perm_in, int8_t *signs_out, int32_t *perm_out,
                                    double *r64_out, double *dots_out);

/* Centralized GraB balancing with a stale mean (Sec. 2.1: the prior method this
 * paper builds on; run per worker it is the ablation's "ID-GraB (Bal)" with the
 * deterministic rule).  One worker, n vectors (n may be odd):
 *     z_j = g_j - stale_mean;   s_j = +1 if ||r + z_j|| < ||r - z_j|| else -1;   r += s_j z_j
 *     perm_out = concat(L_pos, reverse(L_neg)) of perm_in under the signs s (Sec. 2.1)
 *   grads [n][d] fp32 dev in visiting order, stale_mean [d] fp32 dev or NULL (zero),
 *   perm_in [n] int32 dev or NULL, signs_out [n] int8 dev (s_j), perm_out [n] int32 dev,
 *   mean_out [d] fp32 dev or NULL: mean of this epoch's vectors (next epoch's stale
 *   mean; must not overlap stale_mean), r64_out [d] fp64 dev or NULL: final running sum.
 *   perm_out must not overlap perm_in.
 * Same arithmetic as cdgrab_balance_epoch.  Errors: EINVAL (sizes, null, overlapping
 * buffers), ENOMEM, EHIP. */
int cdgrab_balance_epoch_stale_mean(cdgrab_handle *h, int64_t n, int64_t d, const float *grads,
                                    const float *stale_mean, const int32_t *perm_in,
                                    int8_t *signs_out, int32_t *perm_out, float *mean_out,
                                    double *r64_out);

/* The uncoordinated ablation baseline "ID-GraB (PairBal)" (Sec. 5, ablation study):
 * every worker balances its own pairs on its own running sum, with no shared state,
 * i.e. m separate runs of cdgrab_balance_epoch with m = 1.  For short rows (where such a
 * run is a chain of small dependent launches) the m walks run side by side, the worker as
 * a grid coordinate of every launch; for long rows one after the other.  Either way a
 * worker's result is that of its own one-worker epoch.  Same layouts as there:
 *   grads [m][n][d] fp32 dev, perm_in [m][n] or NULL, signs_out [m][n/2], perm_out [m][n].
 * Errors: as cdgrab_balance_epoch. */
int cdgrab_balance_epoch_independent(cdgrab_handle *h, int64_t m, int64_t n, int64_t d,
                                     const float *grads, const int32_t *perm_in,
                                     int8_t *signs_out, int32_t *perm_out);

/* One training epoch of the softmax-regression model under CD-GraB ("CD-GraB
 * Workers" + "CD-GraB Parameter Server", Sec. 3.3), the m workers simulated on one
 * GPU.  For step j = 0 .. n-1: worker i computes the gradient of example
 * perm_in[i][j] at the current weights, the server averages the m gradients and
 * every worker applies  v <- momentum v + gbar;  W <- W - lr v.  After every second
 * step the m new pairs are balanced in worker order exactly as in
 * cdgrab_balance_epoch, whose outputs signs_out / perm_out have the same meaning.
 *   X [m][n][in_dim] fp32 dev (example j of worker i is row (i, j)), y [m][n] int32 dev,
 *   perm_in [m][n] int32 dev or NULL, W [(in_dim+1)][classes] fp32 dev (in/out),
 *   velocity [(in_dim+1)*classes] fp32 dev (in/out) or NULL when momentum == 0,
 *   grads_out [m][n][(in_dim+1)*classes] fp32 dev or NULL: the gradient rows in
 *     visiting order (for verification; the epoch itself keeps only a few steps' rows),
 *   loss_out [m][n] fp32 dev or NULL: loss of each example when it was visited.
 *   perm_out must not overlap perm_in.
 * fp32 model arithmetic, double balancing arithmetic.
 * Errors: EINVAL (sizes, n odd, null, momentum without velocity, overlapping orders),
 * ENOMEM, EHIP. */
int cdgrab_train_epoch_softmax(cdgrab_handle *h, int64_t m, int64_t n, int64_t in_dim,
                               int64_t classes, const float *X, const int32_t *y,
                               const int32_t *perm_in, float *W, float *velocity, float lr,
                               float momentum, int8_t *signs_out, int32_t *perm_out,
                               float *grads_out, float *loss_out);

/* T training epochs with the permutations carried over (the outer loop of "CD-GraB
 * Workers" / "CD-GraB Parameter Server", Sec. 3.3: the order built while epoch t is
 * balanced is the order epoch t+1 visits).  Equivalent to `epochs` calls of
 * cdgrab_train_epoch_softmax, each taking the previous call's perm_out as perm_in.
 *   perm [m][n] int32 dev, in/out: the first epoch's order on entry, the order the
 *     next epoch would visit on return,
 *   signs_out [m][n/2] int8 dev or NULL: the last epoch's pair signs,
 *   loss_out [epochs][m][n] fp32 dev or NULL: loss of each example when it was visited.
 * Other arguments as in cdgrab_train_epoch_softmax.  The handle keeps one spare
 * permutation and one sign buffer.
 * Errors: EINVAL (as above, epochs < 1, perm NULL), ENOMEM, EHIP. */
int cdgrab_train_softmax(cdgrab_handle *h, int64_t m, int64_t n, int64_t in_dim, int64_t classes,
                         const float *X, const int32_t *y, int32_t *perm, float *W,
                         float *velocity, float lr, float momentum, int64_t epochs,
                         int8_t *signs_out, float *loss_out);

/* Reorder from arbitrary per-example signs ("Reordering Vectors based on Balanced
 * Signs", Sec. 2.1), one independent problem per worker:
 *   perm_out[i] = concat(L_pos, reverse(L_neg)), L_pos / L_neg the entries of
 *   perm_in[i] (identity if NULL) whose sign is +1 / -1, in visiting order.
 *   signs [m][n] int8 dev, perm_in [m][n] int32 dev or NULL, perm_out [m][n] int32 dev
 *   (must not overlap perm_in).
 * This call synchronises the stream to report a sign that is not +1 or -1.
 * Errors: EINVAL (m<1, n<1, null pointer, bad sign value, overlapping orders), EHIP. */
int cdgrab_reorder(cdgrab_handle *h, int64_t m, int64_t n, const int8_t *signs,
                   const int32_t *perm_in, int32_t *perm_out);

/* Parallel herding objective of a set of vectors under given per-worker orders
 * (Sec. 3.2, the quantity PairBalance + Reorder drive down; Lemma 1):
 *     max_{k<=n} || sum_{j<=k} sum_{i<m} ( z[i][perm[i][j]] - zbar ) ||_inf,
 *     zbar = mean of all m*n vectors.
 *   z [m][n][d] fp32 dev, indexed by example id (NOT by visiting position),
 *   perm [m][n] int32 dev or NULL (identity), bound_out: one double, dev.
 * Sums in double.  Errors: EINVAL (sizes, null), ENOMEM, EHIP. */
int cdgrab_herding_bound(cdgrab_handle *h, int64_t m, int64_t n, int64_t d, const float *z,
                         const int32_t *perm, double *bound_out);

/* Timings of the last cdgrab_balance_epoch on this handle (options.timing >= 1).
 * Synchronises the stream.  Errors: EINVAL (timing was off), EHIP. */
int cdgrab_get_timing(cdgrab_handle *h, cdgrab_timing *out /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* CDGRAB_H */

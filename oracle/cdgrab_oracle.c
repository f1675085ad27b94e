/*
 * CD-GraB CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded reference for the coordinated pair-balancing
 * path of CD-GraB (arXiv 2302.00845), written from the paper's algorithm
 * statements so that it can be checked against them by eye.  Only tests, the
 * smoke check and the CPU-baseline leg of the benchmark may call it; it shares
 * no code with the HIP library and the HIP library never calls it.
 *
 * Arithmetic: inputs are fp32 values; every difference, product and sum below
 * is IEEE double.  There is no blocking, vectorisation or reordering: each
 * function walks the loops in the order the paper states them.
 *
 * What follows which passage
 *   oracle_greedy_balance     "Balancing without normalization" (App. B.2): the
 *                             deterministic rule the authors actually use
 *                             instead of RandomizedBalance.
 *   oracle_pair_balance       Algorithm "PairBalance" (Sec. 3.2) with that rule
 *                             as its subroutine: balance c = z1 - z2, z1 gets
 *                             the sign, z2 the opposite sign.
 *   oracle_server_epoch       "Server-side PairBalance over a set of vectors
 *                             (one step)" (App. C.1): j = 1..n outer, worker
 *                             i = 1..m inner, a pair is examined at even j,
 *                             front/back pointer form of the reorder.
 *   oracle_reorder            "Reordering Vectors based on Balanced Signs"
 *                             (Sec. 2.1): L_pos, L_neg, concat(L_pos,
 *                             reverse(L_neg)).
 *   oracle_stream_pairs       the same walk fed block by block (for inputs too
 *                             large to hold at once) with an optional replay of
 *                             externally supplied signs.
 *   oracle_softmax_pergrad    textbook softmax cross-entropy gradient of a
 *                             linear model (the per-example gradient a worker
 *                             computes in "CD-GraB Workers", line 4).
 *   oracle_parallel_herding   the parallel herding objective (Sec. 3.2).
 *   oracle_randomized_epoch   the server walk with PairBalance's RandomizedBalance
 *                             subroutine (Sec. 3.2) and caller-supplied uniform draws.
 *   oracle_grab_stale_mean    centralized GraB balancing (Sec. 2.1): vectors centred
 *                             by a stale mean, greedy sign per vector, reorder.
 *   oracle_train_epoch_softmax  "CD-GraB Workers" + "CD-GraB Parameter Server"
 *                             (Sec. 3.3) for the softmax-regression model: per
 *                             step, m per-example gradients at the current
 *                             weights, their average, one SGD(+momentum) update.
 *
 * Readings of the paper taken here (each is also pinned by a test):
 *   - Sign exported per pair.  The paper balances c = z1 - z2 and calls the
 *     result s "the sign for z1"; z2 gets -s.  The exported value is
 *     eps = -s, i.e. the sign of the SECOND example of the pair, which is the
 *     same as balancing d = z2 - z1 with "eps = +1 iff <r,d> <= 0".  The
 *     running sum is identical: r + s*c = r + eps*d.
 *   - Tie.  The greedy rule uses a strict "<": ||r+c|| < ||r-c|| gives s=+1,
 *     anything else s=-1.  ||r+c||^2 - ||r-c||^2 = 4<r,c>, so s=+1 iff
 *     <r,c> < 0 and a zero inner product gives s=-1 (eps=+1).  The norm is the
 *     Euclidean one (the text speaks of the inner product of r and g1-g2).
 *   - Flattened order.  Pairs are visited step-major, worker-minor: pair k of
 *     workers 1..m, then pair k+1 (the loop nest of the server algorithm; the
 *     printed flat index n(k-1)+i cannot address m*n/2 items and is read as
 *     m(k-1)+i).
 *   - Back pointer.  The one-step algorithm prints the back pointer's start
 *     value as 1 although it is decremented; it is read as n, which is what
 *     "reverse(L_neg)" and the sequence x+_1..x+_{n/2}, x-_{n/2}..x-_1 in the
 *     proof of Lemma 1 require.
 *   - pi' holds visiting positions; the next absolute order is the old order
 *     composed with it: perm_out[p] = perm_in[pi'[p]].
 *   - The running sum starts at zero in every epoch and is not normalised or
 *     centred.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* "Balancing without normalization": given running sum r and a vector c,
 * s = +1 if ||r + c|| < ||r - c|| else -1; r <- r + s c.
 * The comparison is done through the inner product (see header); t = <r,c> is
 * returned through *t_out, with ||r|| (before the update) and ||c||. */
int oracle_greedy_balance(int64_t d, double *r, const double *c,
                          double *t_out, double *norm_r_out, double *norm_c_out)
{
    double t = 0.0, rr = 0.0, cc = 0.0;
    for (int64_t e = 0; e < d; ++e) {
        t += r[e] * c[e];
        rr += r[e] * r[e];
        cc += c[e] * c[e];
    }
    int s = (t < 0.0) ? +1 : -1;
    for (int64_t e = 0; e < d; ++e)
        r[e] += (double)s * c[e];
    if (t_out) *t_out = t;
    if (norm_r_out) *norm_r_out = sqrt(rr);
    if (norm_c_out) *norm_c_out = sqrt(cc);
    return s;
}

/* The same update with the sign imposed from outside (replay): r <- r + s c.
 * t, ||r||, ||c|| are still reported so the caller can judge the imposed sign. */
static void forced_balance(int64_t d, double *r, const double *c, int s,
                           double *t_out, double *norm_r_out, double *norm_c_out)
{
    double t = 0.0, rr = 0.0, cc = 0.0;
    for (int64_t e = 0; e < d; ++e) {
        t += r[e] * c[e];
        rr += r[e] * r[e];
        cc += c[e] * c[e];
    }
    for (int64_t e = 0; e < d; ++e)
        r[e] += (double)s * c[e];
    if (t_out) *t_out = t;
    if (norm_r_out) *norm_r_out = sqrt(rr);
    if (norm_c_out) *norm_c_out = sqrt(cc);
}

/* "PairBalance": c = z1 - z2; s, r <- Balance(r, c); return s for z1 (and -s
 * for z2).  scratch holds d doubles.  If force_s is +1/-1 that sign is used
 * instead of the greedy one (replay); 0 means decide greedily. */
int oracle_pair_balance(int64_t d, double *r, const float *z1, const float *z2,
                        double *scratch, int force_s,
                        double *t_out, double *norm_r_out, double *norm_c_out)
{
    for (int64_t e = 0; e < d; ++e)
        scratch[e] = (double)z1[e] - (double)z2[e];
    if (force_s == 0)
        return oracle_greedy_balance(d, r, scratch, t_out, norm_r_out, norm_c_out);
    forced_balance(d, r, scratch, force_s, t_out, norm_r_out, norm_c_out);
    return force_s;
}

/* ------------------------------------------------------------------------- */
/* One epoch of server-side PairBalance over m*n vectors (one-step algorithm,
 * App. C.1).
 *   z        [m][n][d] fp32, row (i,j) = the j-th vector worker i visits
 *   perm_in  [m][n] or NULL: example id at each visiting position
 *   eps_out  [m][n/2]  exported sign per pair (= sign of the pair's second row)
 *   r_out    [d]       final running sum
 *   perm_out [m][n]    next order (old order composed with pi')
 *   t_out    [m][n/2]  or NULL: <r,c> seen when the pair was decided
 *   nr_out, nc_out [m][n/2] or NULL: ||r|| before the update, ||c||
 * Returns 0, or -1 on bad sizes / allocation failure. */
int oracle_server_epoch(int64_t m, int64_t n, int64_t d, const float *z,
                        const int32_t *perm_in, int8_t *eps_out, double *r_out,
                        int32_t *perm_out, double *t_out, double *nr_out,
                        double *nc_out)
{
    if (m < 1 || n < 2 || (n & 1) || d < 1) return -1;
    double *h = (double *)calloc((size_t)d, sizeof(double));      /* running sum = 0 */
    double *scratch = (double *)malloc((size_t)d * sizeof(double));
    int64_t *l = (int64_t *)malloc((size_t)m * sizeof(int64_t)); /* front pointers */
    int64_t *rp = (int64_t *)malloc((size_t)m * sizeof(int64_t)); /* back pointers */
    int64_t *pi_new = (int64_t *)malloc((size_t)(m * n) * sizeof(int64_t));
    if (!h || !scratch || !l || !rp || !pi_new) {
        free(h); free(scratch); free(l); free(rp); free(pi_new);
        return -1;
    }
    for (int64_t i = 0; i < m; ++i) { l[i] = 1; rp[i] = n; }

    for (int64_t j = 1; j <= n; ++j) {            /* example index, 1-based */
        for (int64_t i = 1; i <= m; ++i) {        /* worker index, 1-based  */
            if (j % 2 != 0) continue;             /* a full pair needs an even j */
            const float *z_prev = z + ((i - 1) * n + (j - 2)) * d;  /* z^i_{j-1} */
            const float *z_cur  = z + ((i - 1) * n + (j - 1)) * d;  /* z^i_j     */
            int64_t k = j / 2 - 1;                                  /* pair, 0-based */
            double t, nr, nc;
            int s_prev = oracle_pair_balance(d, h, z_prev, z_cur, scratch, 0,
                                             &t, &nr, &nc);
            int64_t *pi = pi_new + (i - 1) * n;   /* 1-based positions below */
            if (s_prev == +1) {
                pi[l[i - 1] - 1] = j - 1;  l[i - 1] += 1;   /* first to the front */
                pi[rp[i - 1] - 1] = j;     rp[i - 1] -= 1;  /* second to the back */
            } else {
                pi[l[i - 1] - 1] = j;      l[i - 1] += 1;   /* second to the front */
                pi[rp[i - 1] - 1] = j - 1; rp[i - 1] -= 1;  /* first to the back  */
            }
            int64_t o = (i - 1) * (n / 2) + k;
            eps_out[o] = (int8_t)(-s_prev);       /* sign of the second row */
            /* t is <r, z1-z2>; the exported dot is <r, z2-z1> = -t. */
            if (t_out) t_out[o] = -t;
            if (nr_out) nr_out[o] = nr;
            if (nc_out) nc_out[o] = nc;
        }
    }
    for (int64_t i = 0; i < m; ++i)
        for (int64_t p = 0; p < n; ++p) {
            int64_t pos = pi_new[i * n + p] - 1;  /* 0-based visiting position */
            perm_out[i * n + p] = perm_in ? perm_in[i * n + pos] : (int32_t)pos;
        }
    memcpy(r_out, h, (size_t)d * sizeof(double));
    free(h); free(scratch); free(l); free(rp); free(pi_new);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The same walk, fed a block of consecutive flattened pairs at a time.
 *   r      [d]            running sum, carried by the caller (zero at epoch start)
 *   rows   [count][2][d]  (first row, second row) of each pair, in flattened order
 *   eps_in [count] or NULL: if given, these exported signs are imposed (replay)
 *   eps_out[count]        exported sign used for each pair
 *   t_out, nr_out, nc_out [count] or NULL: <r, z2-z1>, ||r|| before, ||z2-z1||
 * Returns 0 or -1. */
int oracle_stream_pairs(int64_t d, double *r, int64_t count, const float *rows,
                        const int8_t *eps_in, int8_t *eps_out, double *t_out,
                        double *nr_out, double *nc_out)
{
    if (d < 1 || count < 0) return -1;
    double *scratch = (double *)malloc((size_t)d * sizeof(double));
    if (!scratch) return -1;
    for (int64_t p = 0; p < count; ++p) {
        const float *z1 = rows + (2 * p) * d;
        const float *z2 = rows + (2 * p + 1) * d;
        int force = 0;
        if (eps_in) force = -(int)eps_in[p];      /* s = -eps */
        double t, nr, nc;
        int s = oracle_pair_balance(d, r, z1, z2, scratch, force, &t, &nr, &nc);
        eps_out[p] = (int8_t)(-s);
        if (t_out) t_out[p] = -t;
        if (nr_out) nr_out[p] = nr;
        if (nc_out) nc_out[p] = nc;
    }
    free(scratch);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* "Reordering Vectors based on Balanced Signs": one worker.
 *   signs   [n]  +1 / -1 per visiting position
 *   perm_in [n]  or NULL (identity): example id at each visiting position
 *   perm_out[n]  concat(L_pos, reverse(L_neg))
 * Returns 0, or -1 if a sign is not +-1 or allocation fails. */
int oracle_reorder(int64_t n, const int8_t *signs, const int32_t *perm_in,
                   int32_t *perm_out)
{
    if (n < 0) return -1;
    int32_t *L_pos = (int32_t *)malloc((size_t)(n ? n : 1) * sizeof(int32_t));
    int32_t *L_neg = (int32_t *)malloc((size_t)(n ? n : 1) * sizeof(int32_t));
    if (!L_pos || !L_neg) { free(L_pos); free(L_neg); return -1; }
    int64_t n_pos = 0, n_neg = 0;
    for (int64_t j = 0; j < n; ++j) {
        int32_t id = perm_in ? perm_in[j] : (int32_t)j;
        if (signs[j] == +1) L_pos[n_pos++] = id;
        else if (signs[j] == -1) L_neg[n_neg++] = id;
        else { free(L_pos); free(L_neg); return -1; }
    }
    int64_t p = 0;
    for (int64_t q = 0; q < n_pos; ++q) perm_out[p++] = L_pos[q];
    for (int64_t q = n_neg - 1; q >= 0; --q) perm_out[p++] = L_neg[q];
    free(L_pos); free(L_neg);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Per-example gradient of softmax cross-entropy for a linear model.
 *   X [N][in_dim] fp32, y [N] labels, W [(in_dim+1)][classes] fp32 (last row is
 *   the bias).  logits_c = sum_r x_r W[r][c] + W[in_dim][c];
 *   p = softmax(logits); delta = p - onehot(y);
 *   G[e][r*classes + c] = x_r * delta_c (r < in_dim), G[e][in_dim*classes + c] = delta_c.
 * Everything in double, rounded to fp32 on output. */
int oracle_softmax_pergrad(int64_t N, int64_t in_dim, int64_t classes,
                           const float *X, const int32_t *y, const float *W,
                           float *G_out)
{
    if (N < 0 || in_dim < 1 || classes < 1) return -1;
    double *logit = (double *)malloc((size_t)classes * sizeof(double));
    if (!logit) return -1;
    int64_t dd = (in_dim + 1) * classes;
    for (int64_t e = 0; e < N; ++e) {
        const float *x = X + e * in_dim;
        if (y[e] < 0 || y[e] >= classes) { free(logit); return -1; }
        for (int64_t c = 0; c < classes; ++c) {
            double a = (double)W[in_dim * classes + c];
            for (int64_t r = 0; r < in_dim; ++r)
                a += (double)x[r] * (double)W[r * classes + c];
            logit[c] = a;
        }
        double mx = logit[0];
        for (int64_t c = 1; c < classes; ++c) if (logit[c] > mx) mx = logit[c];
        double Z = 0.0;
        for (int64_t c = 0; c < classes; ++c) { logit[c] = exp(logit[c] - mx); Z += logit[c]; }
        for (int64_t c = 0; c < classes; ++c)
            logit[c] = logit[c] / Z - ((int64_t)y[e] == c ? 1.0 : 0.0);   /* delta */
        float *g = G_out + e * dd;
        for (int64_t r = 0; r < in_dim; ++r)
            for (int64_t c = 0; c < classes; ++c)
                g[r * classes + c] = (float)((double)x[r] * logit[c]);
        for (int64_t c = 0; c < classes; ++c)
            g[in_dim * classes + c] = (float)logit[c];
    }
    free(logit);
    return 0;
}

/* Cross-entropy loss of one example in double (used by the finite-difference pin). */
double oracle_softmax_loss(int64_t in_dim, int64_t classes, const float *x,
                           int32_t y, const double *W)
{
    double mx = -INFINITY, Z = 0.0, ly = 0.0;
    for (int pass = 0; pass < 2; ++pass)
        for (int64_t c = 0; c < classes; ++c) {
            double a = W[in_dim * classes + c];
            for (int64_t r = 0; r < in_dim; ++r) a += (double)x[r] * W[r * classes + c];
            if (pass == 0) { if (a > mx) mx = a; }
            else { Z += exp(a - mx); if (c == y) ly = a; }
        }
    return -(ly - mx - log(Z));
}

/* ------------------------------------------------------------------------- */
/* Parallel herding objective: max_k || sum_{j<=k} sum_i (z_{i,perm_i(j)} - zbar) ||_inf
 * with zbar the mean of all m*n vectors.  perm [m][n] or NULL (identity).
 * z is indexed by example id: z[i][perm[i][j]]. */
double oracle_parallel_herding(int64_t m, int64_t n, int64_t d, const float *z,
                               const int32_t *perm)
{
    double *zbar = (double *)calloc((size_t)d, sizeof(double));
    double *acc = (double *)calloc((size_t)d, sizeof(double));
    if (!zbar || !acc) { free(zbar); free(acc); return -1.0; }
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j)
            for (int64_t e = 0; e < d; ++e) zbar[e] += (double)z[(i * n + j) * d + e];
    for (int64_t e = 0; e < d; ++e) zbar[e] /= (double)(m * n);
    double best = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        for (int64_t i = 0; i < m; ++i) {
            int64_t id = perm ? perm[i * n + j] : j;
            const float *v = z + (i * n + id) * d;
            for (int64_t e = 0; e < d; ++e) acc[e] += (double)v[e] - zbar[e];
        }
        for (int64_t e = 0; e < d; ++e) { double a = fabs(acc[e]); if (a > best) best = a; }
    }
    free(zbar); free(acc);
    return best;
}

/* ------------------------------------------------------------------------- */
/* One training epoch of m simulated workers on the softmax-regression model.
 *   X [m][n][in_dim], y [m][n], perm_in [m][n] or NULL (identity)
 *   W [(in_dim+1)*classes] double, in/out;  v [same] double, in/out (velocity)
 *   rows_out [m][n][d] fp32: gradient of worker i at step j, in visiting order
 *   loss_out [m][n] or NULL: loss of the visited example at the weights it saw
 * Step j (workers' lines 4-7, server's lines 5-7): every worker takes the gradient
 * of example perm_in[i][j] at the current W; gbar = mean over workers;
 * v <- momentum v + gbar; W <- W - lr v (the update rule of the paper's
 * experiments, SGD with momentum).  The server's balancing of these rows does not
 * feed back into the epoch (the sign list is only used for the next epoch's order),
 * so the caller runs oracle_server_epoch on rows_out. */
int oracle_train_epoch_softmax(int64_t m, int64_t n, int64_t in_dim, int64_t classes,
                               const float *X, const int32_t *y, const int32_t *perm_in,
                               double *W, double *v, double lr, double momentum,
                               float *rows_out, double *loss_out)
{
    if (m < 1 || n < 1 || in_dim < 1 || classes < 1) return -1;
    const int64_t d = (in_dim + 1) * classes;
    double *delta = (double *)malloc((size_t)classes * sizeof(double));
    double *gbar = (double *)malloc((size_t)d * sizeof(double));
    if (!delta || !gbar) { free(delta); free(gbar); return -1; }
    for (int64_t j = 0; j < n; ++j) {
        for (int64_t p = 0; p < d; ++p) gbar[p] = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            int64_t id = perm_in ? perm_in[i * n + j] : j;
            const float *x = X + (i * n + id) * in_dim;
            int32_t label = y[i * n + id];
            double mx = -INFINITY, Z = 0.0;
            for (int64_t c = 0; c < classes; ++c) {
                double a = W[in_dim * classes + c];
                for (int64_t r = 0; r < in_dim; ++r) a += (double)x[r] * W[r * classes + c];
                delta[c] = a;
                if (a > mx) mx = a;
            }
            for (int64_t c = 0; c < classes; ++c) Z += exp(delta[c] - mx);
            if (loss_out) loss_out[i * n + j] = -(delta[label] - mx - log(Z));
            for (int64_t c = 0; c < classes; ++c)
                delta[c] = exp(delta[c] - mx) / Z - (c == label ? 1.0 : 0.0);
            float *row = rows_out + (i * n + j) * d;
            for (int64_t r = 0; r <= in_dim; ++r)
                for (int64_t c = 0; c < classes; ++c) {
                    double g = (r < in_dim ? (double)x[r] : 1.0) * delta[c];
                    row[r * classes + c] = (float)g;
                    gbar[r * classes + c] += g;
                }
        }
        for (int64_t p = 0; p < d; ++p) {
            v[p] = momentum * v[p] + gbar[p] / (double)m;
            W[p] -= lr * v[p];
        }
    }
    free(delta); free(gbar);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Centralized GraB balancing of one worker's n vectors (Sec. 2.1): the herding
 * framework is run on z_j = g_j - stale_mean (the stale mean is last epoch's average
 * gradient), each z_j gets the sign of the greedy rule of App. B.2, and the next
 * order is the reorder of Sec. 2.1 under those signs.
 *   g [n][d] fp32 in visiting order, stale_mean [d] fp32 or NULL (zero)
 *   perm_in [n] or NULL, s_out [n] signs, r_out [d] final running sum,
 *   perm_out [n], mean_out [d] or NULL: mean of g (the next stale mean),
 *   t_out, nr_out, nz_out [n] or NULL: <r,z_j>, ||r|| before, ||z_j||. */
int oracle_grab_stale_mean(int64_t n, int64_t d, const float *g, const float *stale_mean,
                           const int32_t *perm_in, int8_t *s_out, double *r_out,
                           int32_t *perm_out, double *mean_out, double *t_out,
                           double *nr_out, double *nz_out)
{
    if (n < 1 || d < 1) return -1;
    double *r = (double *)calloc((size_t)d, sizeof(double));
    double *z = (double *)malloc((size_t)d * sizeof(double));
    if (!r || !z) { free(r); free(z); return -1; }
    for (int64_t j = 0; j < n; ++j) {
        for (int64_t e = 0; e < d; ++e)
            z[e] = (double)g[j * d + e] - (stale_mean ? (double)stale_mean[e] : 0.0);
        double t, nr, nz;
        int s = oracle_greedy_balance(d, r, z, &t, &nr, &nz);
        s_out[j] = (int8_t)s;
        if (t_out) t_out[j] = t;
        if (nr_out) nr_out[j] = nr;
        if (nz_out) nz_out[j] = nz;
    }
    int rc = oracle_reorder(n, s_out, perm_in, perm_out);
    if (mean_out) {
        for (int64_t e = 0; e < d; ++e) {
            double acc = 0.0;
            for (int64_t j = 0; j < n; ++j) acc += (double)g[j * d + e];
            mean_out[e] = acc / (double)n;
        }
    }
    memcpy(r_out, r, (size_t)d * sizeof(double));
    free(r); free(z);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* RandomizedBalance (subroutine of PairBalance, Sec. 3.2): p = (1 - <r,c>)/2;
 * s = +1 with probability p, else -1; r <- r + s c.  The draw is the caller's
 * uniform u in [0,1): s = +1 iff u < p. */
int oracle_randomized_balance(int64_t d, double *r, const double *c, double u, double *t_out)
{
    double t = 0.0;
    for (int64_t e = 0; e < d; ++e) t += r[e] * c[e];
    double p = (1.0 - t) / 2.0;
    int s = (u < p) ? +1 : -1;
    for (int64_t e = 0; e < d; ++e) r[e] += (double)s * c[e];
    if (t_out) *t_out = t;
    return s;
}

/* The one-step server walk (App. C.1 loop nest) with that subroutine.
 *   z [m][n][d], u [m][n/2] draws, perm_in [m][n] or NULL
 *   eps_out [m][n/2]: exported sign (of the second row) = -s, r_out [d], perm_out [m][n],
 *   t_out [m][n/2] or NULL: <r, z2 - z1> seen at decision time. */
int oracle_randomized_epoch(int64_t m, int64_t n, int64_t d, const float *z, const float *u,
                            const int32_t *perm_in, int8_t *eps_out, double *r_out,
                            int32_t *perm_out, double *t_out)
{
    if (m < 1 || n < 2 || (n & 1) || d < 1) return -1;
    double *h = (double *)calloc((size_t)d, sizeof(double));
    double *c = (double *)malloc((size_t)d * sizeof(double));
    int8_t *per_example = (int8_t *)malloc((size_t)n);
    if (!h || !c || !per_example) { free(h); free(c); free(per_example); return -1; }
    for (int64_t j = 2; j <= n; j += 2)
        for (int64_t i = 0; i < m; ++i) {
            const float *z1 = z + (i * n + (j - 2)) * d, *z2 = z + (i * n + (j - 1)) * d;
            for (int64_t e = 0; e < d; ++e) c[e] = (double)z1[e] - (double)z2[e];
            int64_t o = i * (n / 2) + (j / 2 - 1);
            double t;
            int s = oracle_randomized_balance(d, h, c, (double)u[o], &t);
            eps_out[o] = (int8_t)(-s);
            if (t_out) t_out[o] = -t;
        }
    int rc = 0;
    for (int64_t i = 0; i < m && rc == 0; ++i) {
        for (int64_t k = 0; k < n / 2; ++k) {         /* first row gets s = -eps, second -s = eps */
            per_example[2 * k] = (int8_t)(-eps_out[i * (n / 2) + k]);
            per_example[2 * k + 1] = eps_out[i * (n / 2) + k];
        }
        rc = oracle_reorder(n, per_example, perm_in ? perm_in + i * n : NULL, perm_out + i * n);
    }
    memcpy(r_out, h, (size_t)d * sizeof(double));
    free(h); free(c); free(per_example);
    return rc;
}

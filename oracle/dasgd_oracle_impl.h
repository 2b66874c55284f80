/* DaSGD reference iteration, one precision.  Included twice by dasgd_oracle.c with
 * REAL = float / double and NAME(x) = x##_f32 / x##_f64.
 *
 * TEST INFRASTRUCTURE ONLY: a slow, plain transcription of the method used to check the
 * GPU library; the product path never calls it.
 *
 * Notation (paper, Section 3.3.1): x_k^(m) weights of worker m at iteration k, eta learning
 * rate, M workers (W here), tau local steps between averages, d delay, xi local update
 * proportion.  y_k^(m) denotes the value after the local update of step k and before any
 * merge; A_k = (1/W) sum_j y_k^(j) is the average launched at step k.
 */

typedef struct NAME(pending) {
    int64_t launch_step;
    REAL *A;
} NAME(pending);

typedef struct NAME(dasgd_oracle) {
    int W, d, tau;
    int64_t P, k;             /* k = index of the next local step (number of completed steps) */
    REAL lr, momentum, wd, xi;
    REAL *x, *v;              /* [W][P] */
    NAME(pending) *fifo;      /* ring of capacity cap, oldest at head */
    int cap, head, count;
} NAME(dasgd_oracle);

/* Local update of every replica (Eq. 2, first branch, with the optimiser constants of the
 * experiments, Section 4.1: momentum and weight decay).  Heavy-ball momentum with coupled L2
 * decay, v_0 = 0, no dampening, learning rate applied outside the buffer:
 *     g' = g + wd * x ;  v <- momentum * v + g' ;  x <- x - lr * v
 * Afterwards x holds y_k. */
void NAME(dasgd_oracle_local_update)(int W, int64_t P, REAL lr, REAL momentum, REAL wd,
                                     REAL *x, REAL *v, const REAL *g)
{
    int64_t n = (int64_t)W * P;
    #pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        REAL gp = g[e] + wd * x[e];
        REAL vn = momentum * v[e] + gp;
        v[e] = vn;
        x[e] = x[e] - lr * vn;
    }
}

/* Sum of y[j][i] over j in [lo, hi) in pairwise (tree) order. */
static REAL NAME(pairwise_sum)(const REAL *y, int64_t P, int64_t i, int lo, int hi)
{
    if (hi - lo == 1) return y[(int64_t)lo * P + i];
    int mid = lo + (hi - lo + 1) / 2;
    return NAME(pairwise_sum)(y, P, i, lo, mid) + NAME(pairwise_sum)(y, P, i, mid, hi);
}

/* Cross-replica mean: every column of (X_k - eta G_k) J in the matrix form of the update
 * rule (appendix, matrix representation) -- A[i] = (1/W) sum_j y[j][i]. */
void NAME(dasgd_oracle_mean)(int W, int64_t P, const REAL *y, REAL *A)
{
    REAL inv = (REAL)1 / (REAL)W;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < P; ++i)
        A[i] = NAME(pairwise_sum)(y, P, i, 0, W) * inv;
}

/* Delayed merge (Eq. 2, second branch): x <- xi * y_k + (1 - xi) * A_{k-d}, where x holds y_k. */
void NAME(dasgd_oracle_merge)(int W, int64_t P, REAL xi, REAL *x, const REAL *A)
{
    REAL om = (REAL)1 - xi;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < P; ++i)
        for (int j = 0; j < W; ++j) {
            int64_t e = (int64_t)j * P + i;
            x[e] = xi * x[e] + om * A[i];
        }
}

NAME(dasgd_oracle) *NAME(dasgd_oracle_create)(int W, int64_t P, int d, int tau, double lr,
                                              double momentum, double wd, double xi, const REAL *w0)
{
    if (W < 1 || P < 1 || d < 0 || tau < 1) return NULL;
    NAME(dasgd_oracle) *o = (NAME(dasgd_oracle) *)calloc(1, sizeof *o);
    if (!o) return NULL;
    o->W = W; o->P = P; o->d = d; o->tau = tau; o->k = 0;
    o->lr = (REAL)lr; o->momentum = (REAL)momentum; o->wd = (REAL)wd; o->xi = (REAL)xi;
    o->x = (REAL *)malloc(sizeof(REAL) * (size_t)W * (size_t)P);
    o->v = (REAL *)calloc((size_t)W * (size_t)P, sizeof(REAL));           /* v_0 = 0 */
    o->cap = d / tau + 2;
    o->fifo = (NAME(pending) *)calloc((size_t)o->cap, sizeof *o->fifo);
    if (!o->x || !o->v || !o->fifo) { free(o->x); free(o->v); free(o->fifo); free(o); return NULL; }
    /* every replica starts from the same point (the analysis assumes it, Lemma 1) */
    for (int j = 0; j < W; ++j)
        memcpy(o->x + (size_t)j * (size_t)P, w0, sizeof(REAL) * (size_t)P);
    return o;
}

void NAME(dasgd_oracle_destroy)(NAME(dasgd_oracle) *o)
{
    if (!o) return;
    for (int s = 0; s < o->cap; ++s) free(o->fifo[s].A);
    free(o->fifo); free(o->x); free(o->v); free(o);
}

REAL *NAME(dasgd_oracle_x)(NAME(dasgd_oracle) *o) { return o->x; }
REAL *NAME(dasgd_oracle_v)(NAME(dasgd_oracle) *o) { return o->v; }
int64_t NAME(dasgd_oracle_k)(const NAME(dasgd_oracle) *o) { return o->k; }
int NAME(dasgd_oracle_pending)(const NAME(dasgd_oracle) *o) { return o->count; }
void NAME(dasgd_oracle_set_lr)(NAME(dasgd_oracle) *o, double lr) { o->lr = (REAL)lr; }
void NAME(dasgd_oracle_set_xi)(NAME(dasgd_oracle) *o, double xi) { o->xi = (REAL)xi; }

/* One iteration k of DaSGD for all replicas; g is [W][P], the gradients at the current x.
 *   (1) local update, every step                                    (Eq. 2, first branch)
 *   (2) if (k+1) mod tau == 0: launch the average of the y_k         (every tau local steps)
 *   (3) if an average launched at step k-d is pending: merge it      (Eq. 2, second branch,
 *       trigger in the appendix form (k+1-d) mod tau == 0, which stays meaningful for d >= tau)
 * The average is taken of the pre-merge values y_k (Eq. 2's summand is x_{k-d} - eta g(x_{k-d})),
 * so (2) precedes (3); with d = 0 the same step launches and merges (plain Local SGD).
 * Returns bit 0 set if an average was launched, bit 1 set if a merge was applied, -1 on error. */
int NAME(dasgd_oracle_step)(NAME(dasgd_oracle) *o, const REAL *g)
{
    int what = 0;
    int64_t k = o->k;
    NAME(dasgd_oracle_local_update)(o->W, o->P, o->lr, o->momentum, o->wd, o->x, o->v, g);
    if ((k + 1) % o->tau == 0) {
        if (o->count == o->cap) return -1;
        int s = (o->head + o->count) % o->cap;
        if (!o->fifo[s].A) o->fifo[s].A = (REAL *)malloc(sizeof(REAL) * (size_t)o->P);
        if (!o->fifo[s].A) return -1;
        NAME(dasgd_oracle_mean)(o->W, o->P, o->x, o->fifo[s].A);
        o->fifo[s].launch_step = k;
        o->count++;
        what |= 1;
    }
    if (o->count > 0 && o->fifo[o->head].launch_step == k - o->d) {
        NAME(dasgd_oracle_merge)(o->W, o->P, o->xi, o->x, o->fifo[o->head].A);
        o->head = (o->head + 1) % o->cap;
        o->count--;
        what |= 2;
    }
    o->k = k + 1;
    return what;
}

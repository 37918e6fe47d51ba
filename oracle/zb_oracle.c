/*
 * zb_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Plain CPU simulation of the paper's full-pipeline orchestration for ZeroBubble-style
 * schedules with three ops per stage and micro-batch: forward F, backward-input B and
 * backward-weight W (Section 3, Section 4.3, Appendix "Scheduling Algorithm").
 *
 * Two things are simulated, both in exact event time (the paper's simulator advances in
 * steps of delta; here every event happens at its own integer time):
 *
 *  (1) schedule generation with the two-phase operator selection policy (Section 4.3,
 *      Algorithm 3): whenever a stage is idle it looks at its available ops -- F(i,m) once
 *      F(i-1,m) has finished plus the link delay, B(i,m) once B(i+1,m) has finished plus the
 *      link delay (B(S-1,m) once F(S-1,m) has finished), W(i,m) once B(i,m) has finished;
 *      all forwards of stage 0 are available at time 0 -- and, while its warm-up quota x_i
 *      is not used up, runs a forward if one is available and otherwise stays idle; after
 *      that it runs the available op of highest priority, B > F > W.  Within one type the
 *      lowest micro-batch goes first.  At one instant all finishes are handled first,
 *      then the idle stages choose, in stage order 0..S-1 (Algorithm 4's loop order).
 *      The result is the order in which every stage ran its 3N ops, and all times.
 *
 *  (2) fixed-order execution: a given per-stage op order (a "fixed execution plan",
 *      Section 3.2) is run under link delays with the dependency rules of Section 3.1;
 *      an op starts when its stage has finished the previous op of the order and its
 *      input has arrived.
 *
 * Readings where the listing of Algorithm 4 is garbled: a dependent op becomes available
 * at the producer's FINISH plus the delay (the listing adds the delay to the time of
 * scheduling); W(i,m) belongs to the stage that ran B(i,m); the last stage's B follows
 * its own F.  Ops are encoded as type * N + m with type 0 = F, 1 = B, 2 = W.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ZF = 0, ZB = 1, ZW = 2 };

typedef struct {
    int S, N;
    int64_t *ready;      /* [S][3][N]: time the op became available, -1 = not yet */
    uint8_t *started;    /* [S][3][N] */
    int64_t *start, *fin;/* [S][3][N] */
    int32_t *order;      /* [S][3N] */
    int32_t *n_done, *quota, *cur;   /* [S]; cur = running op or -1 */
    int64_t *busy_until, *idle, *free_at;
    int64_t *evt; int64_t n_evt, cap_evt;   /* min-heap of event times */
} zb_t;

static void evt_push(zb_t *z, int64_t t) {
    int64_t i = z->n_evt++;
    while (i > 0) {
        int64_t p = (i - 1) / 2;
        if (z->evt[p] <= t) break;
        z->evt[i] = z->evt[p];
        i = p;
    }
    z->evt[i] = t;
}

static int64_t evt_pop(zb_t *z) {
    int64_t top = z->evt[0], last = z->evt[--z->n_evt], i = 0, n = z->n_evt;
    for (;;) {
        int64_t l = 2 * i + 1, r = l + 1, c;
        if (l >= n) break;
        c = (r < n && z->evt[r] < z->evt[l]) ? r : l;
        if (z->evt[c] >= last) break;
        z->evt[i] = z->evt[c];
        i = c;
    }
    if (n > 0) z->evt[i] = last;
    return top;
}

static zb_t *zb_new(int S, int N) {
    zb_t *z = (zb_t *)calloc(1, sizeof(zb_t));
    size_t n = (size_t)S * 3 * N;
    z->S = S; z->N = N;
    z->ready = (int64_t *)malloc(n * sizeof(int64_t));
    z->started = (uint8_t *)malloc(n);
    z->start = (int64_t *)malloc(n * sizeof(int64_t));
    z->fin = (int64_t *)malloc(n * sizeof(int64_t));
    z->order = (int32_t *)malloc(n * sizeof(int32_t));
    z->n_done = (int32_t *)malloc(S * sizeof(int32_t));
    z->quota = (int32_t *)malloc(S * sizeof(int32_t));
    z->cur = (int32_t *)malloc(S * sizeof(int32_t));
    z->busy_until = (int64_t *)malloc(S * sizeof(int64_t));
    z->idle = (int64_t *)malloc(S * sizeof(int64_t));
    z->free_at = (int64_t *)malloc(S * sizeof(int64_t));
    z->cap_evt = 8 * (int64_t)n + 64;
    z->evt = (int64_t *)malloc((size_t)z->cap_evt * sizeof(int64_t));
    return z;
}

static void zb_free(zb_t *z) {
    free(z->ready); free(z->started); free(z->start); free(z->fin); free(z->order);
    free(z->n_done); free(z->quota); free(z->cur); free(z->busy_until); free(z->idle);
    free(z->free_at); free(z->evt); free(z);
}

#define IDX(z, i, ty, m) (((size_t)(i) * 3 + (ty)) * (z)->N + (m))

static int64_t dur_of(int ty, int i, const int32_t *tF, const int32_t *tB, const int32_t *tW) {
    return ty == ZF ? tF[i] : (ty == ZB ? tB[i] : tW[i]);
}

/* An op of stage i finished at time t: make its dependents available (Section 3.1). */
static void on_finish(zb_t *z, int i, int ty, int m, int64_t t, const int32_t *cf, const int32_t *cb) {
    int S = z->S;
    if (ty == ZF) {
        if (i < S - 1) { z->ready[IDX(z, i + 1, ZF, m)] = t + cf[i]; evt_push(z, t + cf[i]); }
        else           { z->ready[IDX(z, i, ZB, m)] = t; }
    } else if (ty == ZB) {
        z->ready[IDX(z, i, ZW, m)] = t;
        if (i > 0) { z->ready[IDX(z, i - 1, ZB, m)] = t + cb[i - 1]; evt_push(z, t + cb[i - 1]); }
    }
}

static void start_op(zb_t *z, int i, int ty, int m, int64_t t,
                     const int32_t *tF, const int32_t *tB, const int32_t *tW) {
    z->started[IDX(z, i, ty, m)] = 1;
    z->start[IDX(z, i, ty, m)] = t;
    z->idle[i] += t - z->free_at[i];
    z->cur[i] = ty * z->N + m;
    z->busy_until[i] = t + dur_of(ty, i, tF, tB, tW);
    z->order[(size_t)i * 3 * z->N + z->n_done[i]] = ty * z->N + m;
    evt_push(z, z->busy_until[i]);
}

/* lowest micro-batch of type ty that is available at time t and not started, or -1 */
static int first_available(zb_t *z, int i, int ty, int64_t t) {
    for (int m = 0; m < z->N; ++m) {
        int64_t r = z->ready[IDX(z, i, ty, m)];
        if (!z->started[IDX(z, i, ty, m)] && r >= 0 && r <= t) return m;
    }
    return -1;
}

static void zb_reset(zb_t *z) {
    size_t n = (size_t)z->S * 3 * z->N;
    for (size_t k = 0; k < n; ++k) { z->ready[k] = -1; z->started[k] = 0; z->start[k] = -1; z->fin[k] = -1; z->order[k] = -1; }
    for (int i = 0; i < z->S; ++i) { z->n_done[i] = 0; z->cur[i] = -1; z->busy_until[i] = 0; z->idle[i] = 0; z->free_at[i] = 0; }
    z->n_evt = 0;
}

/*
 * mode 0: generate with the selection policy (x = warm-up quotas, may be NULL in mode 1);
 * mode 1: execute the fixed order in_order[S][3N].
 * Returns the makespan, or -1 if not every op could run (deadlock).
 */
static int64_t zb_run(zb_t *z, int mode, const int32_t *tF, const int32_t *tB, const int32_t *tW,
                      const int32_t *x, const int32_t *in_order, const int32_t *cf, const int32_t *cb) {
    int S = z->S, N = z->N;
    int64_t total = (int64_t)S * 3 * N, done = 0, makespan = 0;
    zb_reset(z);
    /* a stage cannot warm up more forwards than there are micro-batches (it would idle for ever) */
    for (int i = 0; i < S; ++i) z->quota[i] = x ? (x[i] < 0 ? 0 : (x[i] > N ? N : x[i])) : 0;
    for (int m = 0; m < N; ++m) z->ready[IDX(z, 0, ZF, m)] = 0;
    evt_push(z, 0);
    while (z->n_evt > 0) {
        int64_t t = evt_pop(z);
        while (z->n_evt > 0 && z->evt[0] == t) evt_pop(z);
        for (int i = 0; i < S; ++i) {                       /* finishes first */
            if (z->cur[i] >= 0 && z->busy_until[i] == t) {
                int ty = z->cur[i] / N, m = z->cur[i] % N;
                z->cur[i] = -1;
                z->fin[IDX(z, i, ty, m)] = t;
                z->free_at[i] = t;
                z->n_done[i] += 1;
                done += 1;
                if (t > makespan) makespan = t;
                on_finish(z, i, ty, m, t, cf, cb);
            }
        }
        for (int i = 0; i < S; ++i) {                       /* then the idle stages choose */
            if (z->cur[i] >= 0 || z->n_done[i] >= 3 * N) continue;
            if (mode == 1) {
                int op = in_order[(size_t)i * 3 * N + z->n_done[i]];
                int ty = op / N, m = op % N;
                int64_t r = z->ready[IDX(z, i, ty, m)];
                if (r >= 0 && r <= t) start_op(z, i, ty, m, t, tF, tB, tW);
            } else if (z->quota[i] > 0) {                   /* warm-up: forwards only */
                int m = first_available(z, i, ZF, t);
                if (m >= 0) { z->quota[i] -= 1; start_op(z, i, ZF, m, t, tF, tB, tW); }
            } else {                                        /* priority B > F > W */
                static const int prio[3] = { ZB, ZF, ZW };
                for (int p = 0; p < 3; ++p) {
                    int m = first_available(z, i, prio[p], t);
                    if (m >= 0) { start_op(z, i, prio[p], m, t, tF, tB, tW); break; }
                }
            }
        }
    }
    if (done < total) return -1;
    for (int i = 0; i < S; ++i) z->idle[i] += makespan - z->free_at[i];
    return makespan;
}

/*
 * One pair.  mode 0: policy with quotas x[S]; mode 1: fixed order in_order[S][3N].
 * Outputs (all optional): order[S][3N], start/fin [S][3][N] int64, idle[S].
 * Returns the makespan, -1 on deadlock, -2 on bad input.
 */
int64_t adaptra_oracle_zb(int S, int N, int mode, const int32_t *tF, const int32_t *tB, const int32_t *tW,
                          const int32_t *x, const int32_t *in_order, const int32_t *cf, const int32_t *cb,
                          int32_t *out_order, int64_t *out_start, int64_t *out_fin, int64_t *out_idle) {
    if (S < 1 || N < 1 || (mode == 0 && !x) || (mode == 1 && !in_order)) return -2;
    for (int i = 0; i < S; ++i) if (tF[i] < 0 || tB[i] < 0 || tW[i] < 0) return -2;
    for (int i = 0; i + 1 < S; ++i) if (cf[i] < 0 || cb[i] < 0) return -2;
    zb_t *z = zb_new(S, N);
    int64_t mk = zb_run(z, mode, tF, tB, tW, x, in_order, cf, cb);
    size_t n = (size_t)S * 3 * N;
    if (out_order) memcpy(out_order, z->order, n * sizeof(int32_t));
    if (out_start) memcpy(out_start, z->start, n * sizeof(int64_t));
    if (out_fin) memcpy(out_fin, z->fin, n * sizeof(int64_t));
    if (out_idle) for (int i = 0; i < S; ++i) out_idle[i] = z->idle[i];
    zb_free(z);
    return mk;
}

/*
 * Many pairs: x is [S][n_cand] (structure of arrays), cf / cb are [S-1][n_scen]; pair p is
 * (candidate p % n_cand, scenario p / n_cand).  mode 0 only (policy under the scenario's
 * delays).  out_makespan[n_scen][n_cand] int32 (INT32_MAX on deadlock), out_idle
 * [S][n_scen][n_cand] or NULL.  Returns 0, or -2 on bad input.
 */
int64_t adaptra_oracle_zb_batch(int S, int N, const int32_t *tF, const int32_t *tB, const int32_t *tW,
                                int64_t n_cand, const int32_t *x, int64_t n_scen, const int32_t *cf, const int32_t *cb,
                                int32_t *out_makespan, int32_t *out_idle) {
    if (S < 1 || N < 1) return -2;
    zb_t *z = zb_new(S, N);
    int32_t xs[64], cfs[64], cbs[64];
    if (S > 64) { zb_free(z); return -2; }
    int64_t P = n_cand * n_scen;
    for (int64_t p = 0; p < P; ++p) {
        int64_t c = p % n_cand, k = p / n_cand;
        for (int i = 0; i < S; ++i) xs[i] = x[(int64_t)i * n_cand + c];
        for (int i = 0; i + 1 < S; ++i) { cfs[i] = cf[(int64_t)i * n_scen + k]; cbs[i] = cb[(int64_t)i * n_scen + k]; }
        int64_t mk = zb_run(z, 0, tF, tB, tW, xs, NULL, cfs, cbs);
        out_makespan[p] = mk < 0 ? INT32_MAX : (int32_t)mk;
        if (out_idle) for (int i = 0; i < S; ++i) out_idle[(int64_t)i * P + p] = mk < 0 ? INT32_MAX : (int32_t)z->idle[i];
    }
    zb_free(z);
    return 0;
}

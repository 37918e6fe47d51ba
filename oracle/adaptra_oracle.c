/*
 * adaptra_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, event-driven CPU simulator of one 1F1B-family pipeline
 * schedule under per-link communication delays.  It exists only to check the
 * GPU library and to be timed beside it as a baseline; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or helper with the GPU path.
 *
 * What is simulated (the paper's model, written out as a discrete-event system):
 *   - Section 3.1 (dependency rules): forward F(s,m) may start only after
 *     F(s-1,m) has finished plus the delay of link s-1 -> s; backward B(s,m)
 *     only after B(s+1,m) has finished plus the delay of link s+1 -> s.  On the
 *     last stage B(S-1,m) needs F(S-1,m) (same device, no link).  F(0,m) is
 *     available at time 0 (Appendix, schedule generation: the forwards of
 *     stage 0 are available initially).
 *   - Section 4.1 (three phases) and Section 4.3 (warm-up quota): stage s runs a
 *     fixed list of 2M ops, one at a time: w forwards (warm-up), then
 *     alternating F, B while forwards remain (steady), then the remaining
 *     backwards (cool-down).  w is the count with the last stage of plain 1F1B
 *     at 0, i.e. the paper's x_s = w_s + 1 (Algorithm 2 sets x_{S-1} = 1).
 *     w is clamped into [0, M-1]: w = M and w = M-1 give the same list.
 *   - Section 4 assumes no head-of-line blocking: a link is a pure latency, any
 *     number of messages may be in flight.
 *   - Outputs: pipeline execution time T (Table 1) = time of the last finish
 *     event; bubble of stage s = idle time of that stage inside [0, T],
 *     accumulated gap by gap (Section 1: bubbles are GPU idle periods);
 *     in-flight activations of stage s = forwards started - backwards
 *     finished, whose peak is held against the memory limit (Algorithm 1,
 *     x_max); a schedule violating Lemma 1 shows up as a simulation that
 *     stalls with ops left (deadlock).
 *
 * Events are kept in a binary min-heap ordered by (time, insertion number).
 * Times are int64 inside; results are stored as int32 microseconds.
 *
 * Flag byte per pair: 1 = feasible, 2 = deadlock, 4 = memory cap exceeded,
 * 6 = both.  A deadlocked pair reports INT32_MAX for makespan and bubbles.
 * For a deadlocked pair the memory test uses the declared count w_s + 1 (the
 * quantity Algorithm 1 bounds); for a completed simulation it uses the
 * counted peak.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OP_F = 0, OP_B = 1 };
enum { EV_FINISH = 0, EV_ARRIVE_F = 1, EV_ARRIVE_B = 2 };

typedef struct {
    int64_t time;
    int64_t seq;
    int32_t kind, stage, mb, op;
} event_t;

typedef struct {
    int S, M;
    /* per-stage program */
    int8_t  *op_type;   /* [S][2M] */
    int32_t *op_mb;     /* [S][2M] */
    int32_t *wclamp;    /* [S] */
    /* arrival tables: -1 = input not yet arrived */
    int64_t *arr_f, *arr_b;                 /* [S][M] */
    int64_t *start_f, *fin_f, *start_b, *fin_b; /* [S][M] timeline */
    /* per-stage machine state */
    int32_t *pc, *busy, *inflight, *peak;
    int64_t *free_at, *idle;
    /* event heap */
    event_t *heap;
    int64_t heap_n, heap_cap, seq;
    int64_t makespan;
} sim_t;

static sim_t *sim_new(int S, int M) {
    sim_t *z = (sim_t *)calloc(1, sizeof(sim_t));
    size_t SM = (size_t)S * (size_t)M;
    z->S = S; z->M = M;
    z->op_type = (int8_t *)malloc(2 * SM);
    z->op_mb = (int32_t *)malloc(2 * SM * sizeof(int32_t));
    z->wclamp = (int32_t *)malloc(S * sizeof(int32_t));
    z->arr_f = (int64_t *)malloc(SM * sizeof(int64_t));
    z->arr_b = (int64_t *)malloc(SM * sizeof(int64_t));
    z->start_f = (int64_t *)malloc(SM * sizeof(int64_t));
    z->fin_f = (int64_t *)malloc(SM * sizeof(int64_t));
    z->start_b = (int64_t *)malloc(SM * sizeof(int64_t));
    z->fin_b = (int64_t *)malloc(SM * sizeof(int64_t));
    z->pc = (int32_t *)malloc(S * sizeof(int32_t));
    z->busy = (int32_t *)malloc(S * sizeof(int32_t));
    z->inflight = (int32_t *)malloc(S * sizeof(int32_t));
    z->peak = (int32_t *)malloc(S * sizeof(int32_t));
    z->free_at = (int64_t *)malloc(S * sizeof(int64_t));
    z->idle = (int64_t *)malloc(S * sizeof(int64_t));
    z->heap_cap = 2 * (int64_t)SM + 4 * S + 16;
    z->heap = (event_t *)malloc((size_t)z->heap_cap * sizeof(event_t));
    return z;
}

static void sim_free(sim_t *z) {
    if (!z) return;
    free(z->op_type); free(z->op_mb); free(z->wclamp);
    free(z->arr_f); free(z->arr_b);
    free(z->start_f); free(z->fin_f); free(z->start_b); free(z->fin_b);
    free(z->pc); free(z->busy); free(z->inflight); free(z->peak);
    free(z->free_at); free(z->idle); free(z->heap); free(z);
}

static int ev_less(const event_t *a, const event_t *b) {
    if (a->time != b->time) return a->time < b->time;
    return a->seq < b->seq;
}

static void heap_push(sim_t *z, int64_t time, int kind, int stage, int mb, int op) {
    int64_t i = z->heap_n++;
    event_t e;
    e.time = time; e.seq = z->seq++; e.kind = kind; e.stage = stage; e.mb = mb; e.op = op;
    while (i > 0) {
        int64_t p = (i - 1) / 2;
        if (!ev_less(&e, &z->heap[p])) break;
        z->heap[i] = z->heap[p];
        i = p;
    }
    z->heap[i] = e;
}

static event_t heap_pop(sim_t *z) {
    event_t top = z->heap[0];
    event_t last = z->heap[--z->heap_n];
    int64_t i = 0, n = z->heap_n;
    for (;;) {
        int64_t l = 2 * i + 1, r = l + 1, c;
        if (l >= n) break;
        c = (r < n && ev_less(&z->heap[r], &z->heap[l])) ? r : l;
        if (!ev_less(&z->heap[c], &last)) break;
        z->heap[i] = z->heap[c];
        i = c;
    }
    if (n > 0) z->heap[i] = last;
    return top;
}

/* Materialise the op list of every stage (Section 4.1 phases, Section 4.3 quota). */
static void build_programs(sim_t *z, const int32_t *w, int64_t w_stride) {
    int S = z->S, M = z->M;
    for (int s = 0; s < S; ++s) {
        int64_t wr = w[(int64_t)s * w_stride];
        int wc = (int)(wr < 0 ? 0 : (wr > M - 1 ? M - 1 : wr));
        int8_t *ty = z->op_type + (size_t)s * 2 * M;
        int32_t *mb = z->op_mb + (size_t)s * 2 * M;
        int n = 0;
        z->wclamp[s] = wc;
        for (int m = 0; m < wc; ++m) { ty[n] = OP_F; mb[n] = m; ++n; }           /* warm-up   */
        for (int k = 0; k < M - wc; ++k) {                                       /* steady    */
            ty[n] = OP_F; mb[n] = wc + k; ++n;
            ty[n] = OP_B; mb[n] = k; ++n;
        }
        for (int k = M - wc; k < M; ++k) { ty[n] = OP_B; mb[n] = k; ++n; }       /* cool-down */
    }
}

/* Start the next op of stage s if the stage is free and the op's input is there. */
static void try_start(sim_t *z, int s, int64_t now, const int32_t *t_f, const int32_t *t_b) {
    int M = z->M;
    if (z->busy[s] || z->pc[s] >= 2 * M) return;
    int i = z->pc[s];
    int ty = z->op_type[(size_t)s * 2 * M + i];
    int mb = z->op_mb[(size_t)s * 2 * M + i];
    int64_t arrived = (ty == OP_F) ? z->arr_f[(size_t)s * M + mb] : z->arr_b[(size_t)s * M + mb];
    if (arrived < 0) return;                 /* input not here yet: stay idle */
    z->idle[s] += now - z->free_at[s];       /* the gap just ended */
    z->busy[s] = 1;
    if (ty == OP_F) {
        z->start_f[(size_t)s * M + mb] = now;
        z->inflight[s] += 1;
        if (z->inflight[s] > z->peak[s]) z->peak[s] = z->inflight[s];
        heap_push(z, now + t_f[s], EV_FINISH, s, mb, OP_F);
    } else {
        z->start_b[(size_t)s * M + mb] = now;
        heap_push(z, now + t_b[s], EV_FINISH, s, mb, OP_B);
    }
}

/* Run one (candidate, scenario) pair.  Returns 1 if every op ran, 0 on deadlock. */
static int simulate(sim_t *z, const int32_t *t_f, const int32_t *t_b,
                    const int32_t *w, int64_t w_stride,
                    const int32_t *cf, const int32_t *cb, int64_t c_stride) {
    int S = z->S, M = z->M;
    size_t SM = (size_t)S * M;
    build_programs(z, w, w_stride);
    for (size_t i = 0; i < SM; ++i) {
        z->arr_f[i] = -1; z->arr_b[i] = -1;
        z->start_f[i] = -1; z->fin_f[i] = -1; z->start_b[i] = -1; z->fin_b[i] = -1;
    }
    for (int m = 0; m < M; ++m) z->arr_f[m] = 0;   /* stage 0: all forwards available at t = 0 */
    for (int s = 0; s < S; ++s) {
        z->pc[s] = 0; z->busy[s] = 0; z->inflight[s] = 0; z->peak[s] = 0;
        z->free_at[s] = 0; z->idle[s] = 0;
    }
    z->heap_n = 0; z->seq = 0; z->makespan = 0;
    for (int s = 0; s < S; ++s) try_start(z, s, 0, t_f, t_b);

    while (z->heap_n > 0) {
        event_t e = heap_pop(z);
        int s = e.stage, mb = e.mb;
        int64_t now = e.time;
        if (e.kind == EV_FINISH) {
            z->busy[s] = 0;
            z->free_at[s] = now;
            z->pc[s] += 1;
            if (now > z->makespan) z->makespan = now;
            if (e.op == OP_F) {
                z->fin_f[(size_t)s * M + mb] = now;
                if (s < S - 1)
                    heap_push(z, now + cf[(int64_t)s * c_stride], EV_ARRIVE_F, s + 1, mb, OP_F);
                else
                    z->arr_b[(size_t)s * M + mb] = now;   /* last stage: B(S-1,m) needs F(S-1,m) */
            } else {
                z->fin_b[(size_t)s * M + mb] = now;
                z->inflight[s] -= 1;
                if (s > 0)
                    heap_push(z, now + cb[(int64_t)(s - 1) * c_stride], EV_ARRIVE_B, s - 1, mb, OP_B);
            }
            try_start(z, s, now, t_f, t_b);
        } else if (e.kind == EV_ARRIVE_F) {
            z->arr_f[(size_t)s * M + mb] = now;
            try_start(z, s, now, t_f, t_b);
        } else {
            z->arr_b[(size_t)s * M + mb] = now;
            try_start(z, s, now, t_f, t_b);
        }
    }
    for (int s = 0; s < S; ++s)
        if (z->pc[s] < 2 * M) return 0;                  /* ops left and nothing pending */
    for (int s = 0; s < S; ++s)
        z->idle[s] += z->makespan - z->free_at[s];       /* tail gap up to T */
    return 1;
}

/* ------------------------------------------------------------------------- */

typedef struct {
    int S, M;
    const int32_t *t_f, *t_b, *mem_cap;
    int64_t n_cand, n_scen;
    const int32_t *w, *c_fwd, *c_bwd;
    int64_t n_pairs;
    const int64_t *pair_cand, *pair_scen;
    int32_t *out_makespan, *out_bubble, *out_peak;
    uint8_t *out_flag;
    int64_t *next;           /* shared work counter */
    int64_t *n_overflow;     /* pairs whose makespan does not fit int32 */
} job_t;

#define ORACLE_CHUNK 64

static void *worker(void *arg) {
    job_t *j = (job_t *)arg;
    int S = j->S, M = j->M;
    sim_t *z = sim_new(S, M);
    for (;;) {
        int64_t p0 = __sync_fetch_and_add(j->next, (int64_t)ORACLE_CHUNK);
        if (p0 >= j->n_pairs) break;
        int64_t p1 = p0 + ORACLE_CHUNK < j->n_pairs ? p0 + ORACLE_CHUNK : j->n_pairs;
        for (int64_t p = p0; p < p1; ++p) {
            int64_t c = j->pair_cand ? j->pair_cand[p] : p % j->n_cand;
            int64_t k = j->pair_scen ? j->pair_scen[p] : p / j->n_cand;
            int done = simulate(z, j->t_f, j->t_b, j->w + c, j->n_cand,
                                j->c_fwd + k, j->c_bwd + k, j->n_scen);
            int flag = done ? 0 : 2;
            if (j->mem_cap) {
                for (int s = 0; s < S; ++s) {
                    int held = done ? z->peak[s] : z->wclamp[s] + 1;
                    if (held > j->mem_cap[s]) { flag |= 4; break; }
                }
            }
            if (flag == 0) flag = 1;
            j->out_flag[p] = (uint8_t)flag;
            if (done) {
                if (z->makespan > INT32_MAX) __sync_fetch_and_add(j->n_overflow, 1);
                j->out_makespan[p] = (int32_t)z->makespan;
            } else {
                j->out_makespan[p] = INT32_MAX;
            }
            if (j->out_bubble)
                for (int s = 0; s < S; ++s)
                    j->out_bubble[(int64_t)s * j->n_pairs + p] = done ? (int32_t)z->idle[s] : INT32_MAX;
            if (j->out_peak)
                for (int s = 0; s < S; ++s)
                    j->out_peak[(int64_t)s * j->n_pairs + p] = z->peak[s];
        }
    }
    sim_free(z);
    return NULL;
}

static int check_inputs(int S, int M, const int32_t *t_f, const int32_t *t_b,
                        int64_t n_scen, const int32_t *c_fwd, const int32_t *c_bwd) {
    if (S < 1 || M < 1) return -1;
    for (int s = 0; s < S; ++s)
        if (t_f[s] < 0 || t_b[s] < 0) return -2;
    for (int64_t i = 0; i < (int64_t)(S - 1) * n_scen; ++i)
        if (c_fwd[i] < 0 || c_bwd[i] < 0) return -2;
    return 0;
}

/*
 * Evaluate pairs.  w is [S][n_cand], c_fwd / c_bwd are [S-1][n_scen] (host).
 * If pair_cand is NULL every pair is evaluated and pair p is
 * (candidate p % n_cand, scenario p / n_cand), i.e. outputs are [n_scen][n_cand];
 * n_pairs must then equal n_cand * n_scen.  out_bubble and out_peak are
 * [S][n_pairs] and may be NULL.  Returns 0, a negative value for invalid
 * input, or the (positive) number of pairs whose makespan overflowed int32.
 */
int64_t adaptra_oracle_eval(int S, int M, const int32_t *t_f, const int32_t *t_b,
                            const int32_t *mem_cap,
                            int64_t n_cand, const int32_t *w,
                            int64_t n_scen, const int32_t *c_fwd, const int32_t *c_bwd,
                            int64_t n_pairs, const int64_t *pair_cand, const int64_t *pair_scen,
                            int32_t *out_makespan, int32_t *out_bubble, uint8_t *out_flag,
                            int32_t *out_peak, int n_threads) {
    int rc = check_inputs(S, M, t_f, t_b, n_scen, c_fwd, c_bwd);
    if (rc) return rc;
    if (!pair_cand && n_pairs != n_cand * n_scen) return -3;
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    int64_t next = 0, n_overflow = 0;
    job_t j;
    j.S = S; j.M = M; j.t_f = t_f; j.t_b = t_b; j.mem_cap = mem_cap;
    j.n_cand = n_cand; j.n_scen = n_scen; j.w = w; j.c_fwd = c_fwd; j.c_bwd = c_bwd;
    j.n_pairs = n_pairs; j.pair_cand = pair_cand; j.pair_scen = pair_scen;
    j.out_makespan = out_makespan; j.out_bubble = out_bubble; j.out_peak = out_peak;
    j.out_flag = out_flag; j.next = &next; j.n_overflow = &n_overflow;
    if (n_threads == 1) {
        worker(&j);
    } else {
        pthread_t th[256];
        for (int i = 0; i < n_threads; ++i) pthread_create(&th[i], NULL, worker, &j);
        for (int i = 0; i < n_threads; ++i) pthread_join(th[i], NULL);
    }
    return n_overflow;
}

/*
 * Full timeline of one pair, for inspection and for checking the simulator
 * against an explicit dependency graph.  w is [S], cf / cb are [S-1].
 * start/fin arrays are [S][M] int64 (-1 where an op never ran); idle and peak
 * are [S].  Returns 1 if the schedule completed, 0 on deadlock, <0 on bad input.
 */
int adaptra_oracle_timeline(int S, int M, const int32_t *t_f, const int32_t *t_b,
                            const int32_t *w, const int32_t *cf, const int32_t *cb,
                            int64_t *start_f, int64_t *fin_f, int64_t *start_b, int64_t *fin_b,
                            int64_t *idle, int32_t *peak, int64_t *makespan) {
    int rc = check_inputs(S, M, t_f, t_b, 1, cf, cb);
    if (rc) return rc;
    sim_t *z = sim_new(S, M);
    int done = simulate(z, t_f, t_b, w, 1, cf, cb, 1);
    size_t SM = (size_t)S * M;
    memcpy(start_f, z->start_f, SM * sizeof(int64_t));
    memcpy(fin_f, z->fin_f, SM * sizeof(int64_t));
    memcpy(start_b, z->start_b, SM * sizeof(int64_t));
    memcpy(fin_b, z->fin_b, SM * sizeof(int64_t));
    for (int s = 0; s < S; ++s) { idle[s] = z->idle[s]; peak[s] = z->peak[s]; }
    *makespan = z->makespan;
    sim_free(z);
    return done;
}

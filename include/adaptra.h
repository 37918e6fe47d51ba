/*
 * adaptra.h -- C ABI of the batched pipeline-schedule evaluator for MI355X (gfx950).
 *
 * The library evaluates the paper's analytical pipeline model for many
 * (schedule candidate, straggler scenario) pairs at once and searches, for each
 * scenario, the candidate with the smallest pipeline execution time.
 *
 * Model (Adaptra paper):
 *   - A candidate is a 1F1B-family schedule of S stages and M micro-batches,
 *     fixed by the warm-up forward count of every stage (Section 4.1, the three
 *     phases; Section 4.3, the warm-up quota).  Here w[s] counts warm-up
 *     forwards with the last stage of plain 1F1B at 0, so the paper's
 *     x_s = w[s] + 1 (Algorithm 2 starts from x_{S-1} = 1).  Stage s executes, in
 *     this order, one op at a time:  F(0..w-1);  then F(w+k), B(k) for
 *     k = 0..M-w-1;  then B(M-w..M-1).  w is clamped into [0, M-1] first.
 *   - A scenario gives the delay of every inter-stage link, forward and backward
 *     direction separately (Section 3.1: c_i is added on the link S_i <-> S_{i+1}).
 *   - Dependencies (Section 3.1): F(s,m) starts after F(s-1,m) has finished plus
 *     c_fwd[s-1]; B(s,m) starts after B(s+1,m) has finished plus c_bwd[s];
 *     B(S-1,m) follows F(S-1,m); every stage runs its ops in the order above.
 *     Links are pure latencies (Section 4 assumes no head-of-line blocking).
 *   - Results per pair: makespan = pipeline execution time T (Table 1);
 *     bubble[s] = idle time of stage s inside [0, T] = T - M (t_f[s] + t_b[s])
 *     (Section 1: bubbles are GPU idle periods); a flag byte:
 *         1  feasible
 *         2  deadlock: the warm-up counts increase somewhere, w[s] < w[s+1]
 *            (Lemma 1, monotonic warm-up) -- the fixed order can never complete
 *         4  memory cap exceeded: w[s] + 1 > mem_cap[s] for some s (Algorithm 1:
 *            at most x_max activations are held per device)
 *         6  both
 *     A deadlocked pair reports INT32_MAX for makespan and every bubble.  A pair
 *     that only exceeds the memory cap still reports its real times (Section 4.2
 *     lifts the cap by host offloading) but is never chosen by adaptra_best.
 *
 * All times are int32 microseconds.  Precondition (see adaptra_check_inputs):
 * 2 * M * S * (max time + max delay) < 2^31, which bounds every path in the
 * dependency graph.
 *
 * Conventions for every entry point:
 *   - The three structs live in HOST memory; every pointer inside them, every
 *     out_* pointer and the workspace are DEVICE pointers owned by the caller.
 *     The library allocates no device memory and keeps no state between calls (the test
 *     and measurement switches of adaptra_testing.h aside).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     adaptra_eval, adaptra_best, adaptra_eval_best, adaptra_seed,
 *     adaptra_sensitivity and adaptra_zb_eval only enqueue kernels on it and return; they do not
 *     synchronise, allocate or record memset nodes, so a caller may capture them
 *     into a HIP graph (after one eager call, which sets the kernels' shared-memory
 *     limits).  Outputs are valid once the stream has drained.
 *     adaptra_check_inputs and adaptra_search wait for the stream.
 *   - Return value: ADAPTRA_OK or one of the error codes below.  Per-pair
 *     conditions (deadlock, memory cap) are data, not errors.
 */
#ifndef ADAPTRA_H
#define ADAPTRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADAPTRA_OK          0
#define ADAPTRA_EINVAL      1   /* null pointer, S/M/n out of range, bad histogram spec      */
#define ADAPTRA_EWORKSPACE  2   /* workspace missing, misaligned (256 B) or too small         */
#define ADAPTRA_EHIP        3   /* a HIP call failed; see adaptra_last_hip_error              */
#define ADAPTRA_ERANGE      4   /* adaptra_check_inputs, adaptra_zb_check_inputs: a time, delay or w out of range */
#define ADAPTRA_EOVERFLOW   5   /* the same: 2 M S (max t + max c) >= 2^31 (3 M S with weight ops)             */

#define ADAPTRA_ELIMIT      6   /* adaptra_best_static: a size beyond the maxima it states                 */

#define ADAPTRA_FLAG_FEASIBLE 1
#define ADAPTRA_FLAG_DEADLOCK 2
#define ADAPTRA_FLAG_MEMCAP   4

#define ADAPTRA_MAX_STAGES  64
#define ADAPTRA_MAX_MICROBATCHES 32768

/* Problem shared by all pairs (inputs of Algorithm 2 / Algorithm 4: S, N, t^F_i, t^B_i). */
typedef struct adaptra_params {
    int32_t S;               /* stages, 1..ADAPTRA_MAX_STAGES                              */
    int32_t M;               /* micro-batches (the paper's N), 1..ADAPTRA_MAX_MICROBATCHES */
    const int32_t *t_f;      /* DEVICE [S] forward time of a stage, >= 0                   */
    const int32_t *t_b;      /* DEVICE [S] backward time of a stage, >= 0                  */
    const int32_t *mem_cap;  /* DEVICE [S] max in-flight micro-batches (x_max); NULL = none */
    int32_t hist_bins;       /* adaptra_best: bins per stage of the bubble histogram, 0 = off */
    int32_t hist_shift;      /* adaptra_best: bin = min(hist_bins-1, bubble >> hist_shift), 0..30 */
} adaptra_params_t;

/* Warm-up vectors, structure of arrays: w[s * n + c] is w_s of candidate c. */
typedef struct adaptra_candidates {
    int64_t n;               /* 1..2^31-1 */
    const int32_t *w;        /* DEVICE [S][n] */
    int32_t w_bound;         /* optional promise: no w exceeds this value; -1 = unknown.
                              * It only sizes the LDS ring of the on-chip kernels
                              * (one launch instead of one per ring depth).  Candidates
                              * that break the promise are still evaluated correctly,
                              * by the general kernel. */
} adaptra_candidates_t;

/* Link delays, structure of arrays: c_fwd[l * n + k] is the delay of link l -> l+1 in
 * scenario k, c_bwd[l * n + k] that of link l+1 -> l.  Both may be NULL when S == 1. */
typedef struct adaptra_scenarios {
    int64_t n;               /* 1..2^31-1 */
    const int32_t *c_fwd;    /* DEVICE [S-1][n], >= 0 */
    const int32_t *c_bwd;    /* DEVICE [S-1][n], >= 0 */
    const int32_t *t_f;      /* optional DEVICE [S][n]: per-scenario forward times (computation   */
    const int32_t *t_b;      /* stragglers, Section 2.2); both or neither.  NULL = params->t_f /  */
                             /* t_b in every scenario.  Ignored by adaptra_zb_eval.               */
} adaptra_scenarios_t;

/* Bytes of device scratch adaptra_eval / adaptra_best / adaptra_check_inputs need for
 * this problem size (reads only S and M of params; touches no device memory).
 * Returns 0 if the sizes are out of range. */
size_t adaptra_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen);

/* The smaller amount that adaptra_best alone needs (no per-pair scratch); a workspace of
 * adaptra_workspace_bytes serves it too. */
size_t adaptra_best_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen);

/* SYNCHRONOUS validation of the device data: enqueues a scan on `stream`, waits for
 * it and returns ADAPTRA_ERANGE if any time, delay or w is negative,
 * ADAPTRA_EOVERFLOW if 2 M S (max time + max delay) >= 2^31, else ADAPTRA_OK.
 * Optional: the other entry points do not call it. */
int adaptra_check_inputs(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                         const adaptra_scenarios_t *scens,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Evaluate every pair (Section 3.1 recurrence over the Section 4.1 stage order).
 *   out_makespan  DEVICE int32 [n_scen][n_cand]
 *   out_bubble    DEVICE int32 [S][n_scen][n_cand], or NULL to skip
 *   out_feasible  DEVICE uint8 [n_scen][n_cand] flag byte (see above)
 * Asynchronous on `stream`. */
int adaptra_eval(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                 const adaptra_scenarios_t *scens,
                 int32_t *out_makespan, int32_t *out_bubble, uint8_t *out_feasible,
                 void *workspace, size_t workspace_bytes, void *stream);

/* Per-scenario search: instead of the single analytic pick of Algorithm 2, take the
 * exact minimum of the makespan over all feasible (flag == 1) candidates, ties to the
 * lowest candidate index.
 *   out_best_idx       DEVICE int32 [n_scen]; -1 if no candidate is feasible
 *   out_best_makespan  DEVICE int32 [n_scen]; INT32_MAX if none
 *   out_best_bubble    DEVICE int32 [n_scen][S] bubbles of the winner (INT32_MAX if
 *                      none), or NULL
 *   out_hist           DEVICE uint64 [S][hist_bins]: per stage, how many feasible pairs
 *                      fall into each bubble bin; required iff params->hist_bins > 0.
 *                      It is overwritten, not accumulated.
 * Asynchronous on `stream`. */
int adaptra_best(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                 const adaptra_scenarios_t *scens,
                 int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                 uint64_t *out_hist,
                 void *workspace, size_t workspace_bytes, void *stream);

/* adaptra_best for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops that re-decide on every measured scenario,
 * harnesses that forbid hipMalloc.  Same arguments, outputs and results as adaptra_best, minus
 * the workspace: the scratch the kernels need (candidate flags, packed warm-up counts, search
 * keys, the general kernel's per-thread state) lives in a fixed array of
 * ADAPTRA_STATIC_SCRATCH_MIB MiB of device memory inside the library, one copy per GPU the
 * library is used on, held until the process ends.  The call itself allocates and frees
 * nothing (its first call on a device looks the array's address up, so make that call outside
 * a graph capture).  Limits, checked first: n_cand <= ADAPTRA_STATIC_MAX_CANDIDATES, n_scen <=
 * ADAPTRA_STATIC_MAX_SCENARIOS, M <= ADAPTRA_STATIC_MAX_MICROBATCHES, else ADAPTRA_ELIMIT and
 * nothing is enqueued.  All calls on one GPU share that GPU's array: calls that overlap in time
 * on one GPU (different streams or threads) race and give undefined results -- run them on one
 * stream, or serialise them.  The array keeps the last call's contents; nothing in it needs to
 * be cleared by the caller.  Asynchronous on `stream`. */
#define ADAPTRA_STATIC_SCRATCH_MIB        21
#define ADAPTRA_STATIC_MAX_CANDIDATES     65536
#define ADAPTRA_STATIC_MAX_SCENARIOS      4096
#define ADAPTRA_STATIC_MAX_MICROBATCHES   1024
int adaptra_best_static(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                        const adaptra_scenarios_t *scens,
                        int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                        uint64_t *out_hist, void *stream);

/* adaptra_eval and adaptra_best in one call, every pair resolved once: the search and the
 * histogram read the makespans the evaluation has just produced instead of running the
 * recurrence again for the feasible candidates.  Arguments, layouts and results are those of
 * the two calls (out_bubble, out_best_bubble and out_hist optional as there); the workspace
 * is adaptra_workspace_bytes.  Asynchronous on `stream`. */
int adaptra_eval_best(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                      const adaptra_scenarios_t *scens,
                      int32_t *out_makespan, int32_t *out_bubble, uint8_t *out_feasible,
                      int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                      uint64_t *out_hist,
                      void *workspace, size_t workspace_bytes, void *stream);

/* The paper's analytic planning (Section 4.2), one result per scenario, as a cheap seed and
 * as the reference point for the exhaustive search of adaptra_best.  Every output is
 * optional (NULL to skip) and uses w = x - 1.
 *   x_max             Algorithm 1: activations a device can hold, floor(M / M^F), >= 1
 *   w_current         DEVICE int32 [S]: the schedule in use, for the Eq. (1) test (required
 *                     iff out_not_absorbed is given); typically out_w_init of an earlier call
 *   out_w_init        DEVICE int32 [S]: Algorithm 1 (initial planning): x_0 = x_max, slack
 *                     spread as evenly as possible, x_{S-1} = 1
 *   out_w_adapted     DEVICE int32 [S][n_scen]: Algorithm 2 (dynamic adaptation):
 *                     Delta_i = min(M - 2S, max(ceil((t_f[i] + t_b[i] + c_fwd[i] + c_bwd[i]) /
 *                     (t_f[i+1] + t_b[i+1])), 2)), floored at 0, x_i = min(x_{i+1} + Delta_i, M).
 *                     The layout is that of adaptra_candidates_t.w with n = n_scen.
 *   out_not_absorbed  DEVICE uint8 [S-1][n_scen]: 1 where Eq. (1) fails for w_current, i.e. the
 *                     link's delay would cascade: t_f[i] + t_b[i] + c_fwd[i] + c_bwd[i] >
 *                     (w_current[i] - w_current[i+1]) (t_f[i+1] + t_b[i+1])
 * params->mem_cap and the histogram fields are ignored.  Asynchronous on `stream`. */
int adaptra_seed(const adaptra_params_t *params, const adaptra_scenarios_t *scens, int32_t x_max,
                 const int32_t *w_current, int32_t *out_w_init, int32_t *out_w_adapted,
                 uint8_t *out_not_absorbed, void *stream);

/* Which link's delay is on the critical path (Section 3.1, Theorem 1: a delay a schedule has
 * no slack for adds to the makespan once per micro-batch that waits on it; one it absorbs
 * adds at most its one-off lead-in): for every candidate c, scenario k and link l the finite
 * difference
 *     out_sens[c][l][k] = makespan(w_c ; c_fwd[l][k] + delta) - makespan(w_c ; scenario k),
 * obtained by evaluating the S - 1 perturbed copies of each scenario next to it with the
 * kernels of adaptra_eval.  0 = the link is off the critical path for that pair; values above
 * delta = the delay is paid more than once (cascading bubbles).  In this model a makespan
 * depends on a link's delays only through c_fwd[l] + c_bwd[l], so the same figure holds for
 * the backward direction.
 *   delta          >= 1, microseconds added to one link at a time
 *   out_makespan   DEVICE int32 [n_cand][n_scen] base makespans, or NULL   (candidate-major,
 *   out_feasible   DEVICE uint8 [n_cand][n_scen] flag bytes, or NULL        unlike adaptra_eval)
 *   out_sens       DEVICE int32 [n_cand][S-1][n_scen]; INT32_MAX for a deadlocked candidate
 * Preconditions: adaptra_eval's, with delta of headroom on the delays; n_scen * S and
 * n_cand * n_scen at most 2^31 - 1.  The workspace size comes from
 * adaptra_sensitivity_workspace_bytes.  Asynchronous on `stream`. */
size_t adaptra_sensitivity_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen);
int adaptra_sensitivity(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                        const adaptra_scenarios_t *scens, int32_t delta,
                        int32_t *out_makespan, uint8_t *out_feasible, int32_t *out_sens,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Guided search for schedule spaces that cannot be enumerated (4-7 choices per stage make
 * 5^31 vectors at S = 32): a neighbourhood descent over the slacks Delta_i = w_i - w_{i+1}
 * -- the coordinates Section 4.2's algorithms plan with -- in which every round is one batched
 * evaluation of all scenarios' neighbourhoods.  Every scenario descends on its own from
 * w_start (clamped into [0, M-1]; e.g. Algorithm 1's plan from adaptra_seed), with makespan
 * INT32_MAX until the first round has priced it.  One round, for every scenario k:
 *   1. its pool: its current point, then the point's neighbours in move order, clamped;
 *   2. every pool entry is evaluated under scenario k; the best is the feasible entry of
 *      smallest makespan, ties to the lowest pool index;
 *   3. the scenario moves to its best entry iff that is strictly better than what it has.
 * It ends after the first round without a move anywhere, or after max_iters rounds.
 *   neighbourhood 0: for l = 0..S-1: -1, then +1, on stages 0..l      (2 S moves)
 *   neighbourhood 1: for a = 0..S-1, b = a..S-1: -1, then +1, on stages a..b   (S (S+1) moves)
 *   out_w          DEVICE int32 [S][n_scen]: the point each scenario ended on
 *   out_makespan   DEVICE int32 [n_scen]: its makespan; INT32_MAX if no feasible point was seen
 *   out_rounds     HOST int32: rounds run (may be NULL)
 *   out_evaluated  HOST int64: pairs evaluated in total: moves + 1 per round for every scenario that moved in
 *                  the round before (all of them in the first round); a scenario at rest is not evaluated
 *                  again, its result could not change (with S = 1 or M = 1 all are, every round) (may be NULL)
 * params->mem_cap and per-scenario stage times are honoured; the histogram fields are ignored.
 * n_scen * (moves + 1) <= 2^31 - 1.  SYNCHRONOUS: each round waits for the stream (the host
 * needs to know whether anything moved). */
size_t adaptra_search_workspace_bytes(const adaptra_params_t *params, int64_t n_scen, int32_t neighbourhood);
int adaptra_search(const adaptra_params_t *params, const adaptra_scenarios_t *scens,
                   const int32_t *w_start, int32_t neighbourhood, int32_t max_iters,
                   int32_t *out_w, int32_t *out_makespan, int32_t *out_rounds, int64_t *out_evaluated,
                   void *workspace, size_t workspace_bytes, void *stream);

/* ZeroBubble-style schedules: three ops per stage and micro-batch -- forward F, backward-input
 * B, backward-weight W (t_w: DEVICE int32 [S], >= 0) -- generated by the paper's two-phase
 * operator selection policy (Section 4.3, Algorithm 3; simulation of Algorithm 4 in exact event
 * time): an idle stage runs forwards only until its warm-up quota x_s = w_s + 1 is used up,
 * then the available op of highest priority B > F > W, lowest micro-batch first within a type;
 * F(s,m) becomes available when F(s-1,m) has finished plus c_fwd[s-1], B(s,m) when B(s+1,m)
 * has finished plus c_bwd[s] (B(S-1,m) when F(S-1,m) has finished), W(s,m) when B(s,m) has
 * finished.  Precondition beyond adaptra_eval's: t_f, t_b >= 1 (no two dependent ops in one
 * instant), and 3 M S (max time + max delay) < 2^31 -- adaptra_zb_check_inputs tests both on
 * the device data.  mem_cap and the histogram fields of
 * params are ignored; w is clamped into [0, M-1].
 *   plan_scenario = -1  every pair generates its schedule under its own scenario's delays
 *                       (the pipeline as Adaptra would re-plan it);
 *   plan_scenario = k   the schedule of each candidate is generated once, under scenario k, and
 *                       then executed as a fixed plan under every scenario (Section 3.2: a
 *                       framework runs a fixed execution plan), e.g. k = the no-straggler case.
 *   out_makespan  DEVICE int32 [n_scen][n_cand]
 *   out_bubble    DEVICE int32 [S][n_scen][n_cand] = makespan - M (t_f + t_b + t_w), or NULL
 * The workspace size comes from adaptra_zb_workspace_bytes.  Asynchronous on `stream`. */
size_t adaptra_zb_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen);

/* SYNCHRONOUS validation of adaptra_zb_eval's preconditions on the device data (Section 3.1:
 * an op runs for its duration and its successor waits for it -- with forward and backward times
 * of at least 1 us no two dependent ops share an instant, which is what lets adaptra_zb_eval
 * decide stage by stage in order of time).  Enqueues a scan on `stream`, waits for it and
 * returns ADAPTRA_ERANGE if a forward or backward time is below 1, or a weight time, delay or
 * w is negative; ADAPTRA_EOVERFLOW if 3 M S (max time + max delay) >= 2^31; else ADAPTRA_OK.
 * Outside these ranges adaptra_zb_eval still returns, but its schedule may differ from the
 * policy's.  Workspace as for adaptra_zb_eval.  Optional: adaptra_zb_eval does not call it. */
int adaptra_zb_check_inputs(const adaptra_params_t *params, const int32_t *t_w, const adaptra_candidates_t *cands,
                            const adaptra_scenarios_t *scens, void *workspace, size_t workspace_bytes, void *stream);

int adaptra_zb_eval(const adaptra_params_t *params, const int32_t *t_w, const adaptra_candidates_t *cands,
                    const adaptra_scenarios_t *scens, int64_t plan_scenario,
                    int32_t *out_makespan, int32_t *out_bubble,
                    void *workspace, size_t workspace_bytes, void *stream);

/* hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
int adaptra_last_hip_error(void);

/* Library version, major * 1000 + minor. */
int adaptra_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADAPTRA_H */

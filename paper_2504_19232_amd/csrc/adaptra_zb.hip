// adaptra_zb.hip -- ZeroBubble-style schedules (forward F, backward-input B, backward-weight W)
// with the paper's two-phase operator selection policy, evaluated for many (warm-up vector,
// straggler scenario) pairs.  gfx950, int32 microseconds.
//
// Model (Adaptra paper): dependency rules of Section 3.1 (F(i,m) after F(i-1,m) + delay,
// B(i,m) after B(i+1,m) + delay, W(i,m) after B(i,m), B(S-1,m) after F(S-1,m)); the policy of
// Section 4.3 / Algorithm 3: an idle stage runs forwards only until its warm-up quota
// x_i = w_i + 1 is used up, afterwards the available op of highest priority B > F > W, the
// lowest micro-batch first within a type; the simulation of Algorithm 4, but in exact event
// time: an op becomes available at the producer's finish plus the link delay.
//
// Evaluation order on the GPU: one lane per pair.  A stage's next action is fully determined
// by the ready times already posted to it (an op's ready time is posted when its producer
// STARTS, since the finish time is then known), so the lane repeatedly takes the stage whose
// next action is earliest (ties to the lower stage), starts that op, posts the ready times it
// creates and refreshes the next-action times of the three stages involved.  Ready times
// posted later are strictly later than the current time because forward and backward ops last
// at least 1 us (a precondition of this entry point), so the decision at the earliest action
// time can never be overturned.  Within a type ops run in micro-batch order and their ready
// times are non-decreasing, so "the lowest available micro-batch" is a per-type cursor.
//
// State per lane lives in global scratch laid out [index][thread] (coalesced across lanes):
//   ready[S][3][N], busy[S], quota[S], cursor[S][3], act_time[S], act_type[S]
// and, for plan replay, the generated order [C][S][3N] of the plan scenario.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"

namespace {

using adaptra_detail::kThreadsPerBlock;
constexpr int kInf = INT32_MAX;

struct ZbArgs {
    int S, N;
    const int *t_f, *t_b, *t_w;
    long long C, K;
    const int *w, *cf, *cb;
    long long plan_scenario;      // -1: every pair generates under its own scenario
    int phase;                    // 0: generate (+ outputs unless a plan is wanted), 1: record plans, 2: replay plans
    int *out_makespan, *out_bubble;
    int *scratch;                 // [per_thread][threads]
    int *plans;                   // [C][S][3N], ops as type * N + m
    long long threads;
};

struct Lane {
    int *base;
    long long nt;
    int S, N;
    __device__ int &ready(int i, int ty, int m) const { return base[(((long long)i * 3 + ty) * N + m) * nt]; }
    __device__ int &busy(int i) const { return base[((long long)3 * S * N + i) * nt]; }
    __device__ int &quota(int i) const { return base[((long long)3 * S * N + S + i) * nt]; }
    __device__ int &cursor(int i, int ty) const { return base[((long long)3 * S * N + 2 * S + i * 3 + ty) * nt]; }
    __device__ int &act_time(int i) const { return base[((long long)3 * S * N + 5 * S + i) * nt]; }
    __device__ int &act_type(int i) const { return base[((long long)3 * S * N + 6 * S + i) * nt]; }
};

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int imax2(int a, int b) { return a > b ? a : b; }

// Next action of stage i from what has been posted so far: the time it can act and the op type
// it will then run (Algorithm 3), or kInf if nothing it may run has been posted yet.
// With a plan, the next op is the plan's, whatever its type.
__device__ void refresh_action(const Lane &L, int i, const int *plan, int done_i) {
    const int N = L.N;
    if (plan) {
        if (done_i >= 3 * N) { L.act_time(i) = kInf; return; }
        const int op = plan[done_i];
        const int ty = op / N, m = op % N;
        const int r = L.ready(i, ty, m);
        L.act_type(i) = ty;
        L.act_time(i) = r == kInf ? kInf : imax2(L.busy(i), r);
        return;
    }
    const int cf = L.cursor(i, 0), cb = L.cursor(i, 1), cw = L.cursor(i, 2);
    const int rf = cf < N ? L.ready(i, 0, cf) : kInf;
    const int rb = cb < N ? L.ready(i, 1, cb) : kInf;
    const int rw = cw < N ? L.ready(i, 2, cw) : kInf;
    const int busy = L.busy(i);
    if (L.quota(i) > 0) {                                   // warm-up: forwards only
        L.act_type(i) = 0;
        L.act_time(i) = rf == kInf ? kInf : imax2(busy, rf);
        return;
    }
    const int first = imin(rb, imin(rf, rw));
    if (first == kInf) { L.act_time(i) = kInf; return; }
    const int t = imax2(busy, first);
    L.act_time(i) = t;
    L.act_type(i) = rb <= t ? 1 : (rf <= t ? 0 : 2);         // priority B > F > W among those ready at t
}

__global__ __launch_bounds__(kThreadsPerBlock) void k_zb(ZbArgs a) {
    const long long tid = (long long)blockIdx.x * kThreadsPerBlock + threadIdx.x;
    const int S = a.S, N = a.N;
    const long long n_items = a.phase == 1 ? a.C : a.C * a.K;
    Lane L{a.scratch + tid, a.threads, S, N};
    for (long long item = tid; item < n_items; item += a.threads) {
        const long long c = a.phase == 1 ? item : item % a.C;
        const long long k = a.phase == 1 ? a.plan_scenario : item / a.C;
        const int *plan_base = a.phase == 2 ? a.plans + c * (long long)S * 3 * N : nullptr;
        int *record = a.phase == 1 ? a.plans + c * (long long)S * 3 * N : nullptr;
        // set-up: nothing posted except the forwards of stage 0 (available at time 0)
        for (int i = 0; i < S; ++i) {
            for (int m = 0; m < N; ++m) {
                L.ready(i, 0, m) = i == 0 ? 0 : kInf;
                L.ready(i, 1, m) = kInf;
                L.ready(i, 2, m) = kInf;
            }
            int wi = a.w[(long long)i * a.C + c];
            wi = wi < 0 ? 0 : (wi > N - 1 ? N - 1 : wi);
            L.busy(i) = 0;
            L.quota(i) = wi + 1;                              // x_i = w_i + 1 warm-up forwards
            L.cursor(i, 0) = 0; L.cursor(i, 1) = 0; L.cursor(i, 2) = 0;
        }
        for (int i = 0; i < S; ++i) refresh_action(L, i, plan_base ? plan_base + (long long)i * 3 * N : nullptr, 0);

        const int total = 3 * S * N;
        int makespan = 0;
        for (int step = 0; step < total; ++step) {
            int best = 0, best_t = L.act_time(0);
            for (int i = 1; i < S; ++i) {
                const int t = L.act_time(i);
                if (t < best_t) { best_t = t; best = i; }
            }
            if (best_t == kInf) { makespan = kInf; break; }   // cannot happen for valid input
            const int i = best, ty = L.act_type(i);
            const int done_i = L.cursor(i, 0) + L.cursor(i, 1) + L.cursor(i, 2);
            int m;
            if (plan_base) m = plan_base[(long long)i * 3 * N + done_i] % N;
            else m = L.cursor(i, ty);
            const int dur = ty == 0 ? a.t_f[i] : (ty == 1 ? a.t_b[i] : a.t_w[i]);
            const int fin = best_t + dur;
            L.busy(i) = fin;
            makespan = imax2(makespan, fin);
            L.cursor(i, ty) += 1;
            if (ty == 0 && L.quota(i) > 0) L.quota(i) -= 1;
            if (record) record[(long long)i * 3 * N + done_i] = ty * N + m;
            int touched_lo = i, touched_hi = i;
            if (ty == 0) {
                if (i < S - 1) { L.ready(i + 1, 0, m) = fin + a.cf[(long long)i * a.K + k]; touched_hi = i + 1; }
                else L.ready(i, 1, m) = fin;
            } else if (ty == 1) {
                L.ready(i, 2, m) = fin;
                if (i > 0) { L.ready(i - 1, 1, m) = fin + a.cb[(long long)(i - 1) * a.K + k]; touched_lo = i - 1; }
            }
            for (int j = touched_lo; j <= touched_hi; ++j) {
                const int dj = j == i ? done_i + 1 : L.cursor(j, 0) + L.cursor(j, 1) + L.cursor(j, 2);
                refresh_action(L, j, plan_base ? plan_base + (long long)j * 3 * N : nullptr, dj);
            }
        }
        if (a.phase != 1) {
            const long long P = a.C * a.K;
            a.out_makespan[item] = makespan;
            if (a.out_bubble)
                for (int i = 0; i < S; ++i)
                    a.out_bubble[(long long)i * P + item] =
                        makespan == kInf ? kInf : makespan - N * (a.t_f[i] + a.t_b[i] + a.t_w[i]);
        }
    }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct ZbPlan {
    long long threads;
    size_t off_scratch, off_plans, total;
};

bool plan_zb(int S, int N, long long C, long long K, ZbPlan *p) {
    if (S < 1 || S > ADAPTRA_MAX_STAGES || N < 1 || N > ADAPTRA_MAX_MICROBATCHES) return false;
    if (C < 1 || C > INT32_MAX || K < 1 || K > INT32_MAX) return false;
    const long long per_thread = (3ll * S * N + 7ll * S) * 4;
    long long nt = (512ll << 20) / per_thread;               // about 512 MiB of lane state at most
    if (nt > 65536) nt = 65536;
    if (nt < 1024) nt = 1024;
    nt = nt / kThreadsPerBlock * kThreadsPerBlock;
    p->threads = nt;
    size_t o = 0;
    p->off_scratch = o; o += align256((size_t)nt * per_thread);
    p->off_plans = o;   o += align256((size_t)C * S * 3 * N * 4);
    p->total = o;
    return true;
}

}  // namespace

extern "C" {

size_t adaptra_zb_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen) {
    ZbPlan p;
    if (!params || !plan_zb(params->S, params->M, n_cand, n_scen, &p)) return 0;
    return p.total;
}

int adaptra_zb_eval(const adaptra_params_t *params, const int32_t *t_w, const adaptra_candidates_t *cands,
                    const adaptra_scenarios_t *scens, int64_t plan_scenario,
                    int32_t *out_makespan, int32_t *out_bubble,
                    void *workspace, size_t workspace_bytes, void *stream) {
    if (!params || !cands || !scens || !t_w || !out_makespan) return ADAPTRA_EINVAL;
    ZbPlan p;
    if (!plan_zb(params->S, params->M, cands->n, scens->n, &p)) return ADAPTRA_EINVAL;
    if (!params->t_f || !params->t_b || !cands->w) return ADAPTRA_EINVAL;
    if (params->S > 1 && (!scens->c_fwd || !scens->c_bwd)) return ADAPTRA_EINVAL;
    if (plan_scenario < -1 || plan_scenario >= scens->n) return ADAPTRA_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < p.total) return ADAPTRA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    ZbArgs a{};
    a.S = params->S; a.N = params->M;
    a.t_f = params->t_f; a.t_b = params->t_b; a.t_w = t_w;
    a.C = cands->n; a.K = scens->n;
    a.w = cands->w; a.cf = scens->c_fwd; a.cb = scens->c_bwd;
    a.plan_scenario = plan_scenario;
    a.out_makespan = out_makespan; a.out_bubble = out_bubble;
    a.scratch = (int *)((char *)workspace + p.off_scratch);
    a.plans = (int *)((char *)workspace + p.off_plans);
    a.threads = p.threads;
    const long long P = a.C * a.K;
    if (plan_scenario < 0) {
        a.phase = 0;
        const long long n = P < a.threads ? P : a.threads;
        a.threads = (n + kThreadsPerBlock - 1) / kThreadsPerBlock * kThreadsPerBlock;
        hipLaunchKernelGGL(k_zb, dim3((unsigned)(a.threads / kThreadsPerBlock)), dim3(kThreadsPerBlock), 0, st, a);
        ADAPTRA_CHECK_LAUNCH();
        return ADAPTRA_OK;
    }
    const long long full = a.threads;
    a.phase = 1;                                             // one plan per candidate, under the plan scenario
    long long n = a.C < full ? a.C : full;
    a.threads = (n + kThreadsPerBlock - 1) / kThreadsPerBlock * kThreadsPerBlock;
    hipLaunchKernelGGL(k_zb, dim3((unsigned)(a.threads / kThreadsPerBlock)), dim3(kThreadsPerBlock), 0, st, a);
    ADAPTRA_CHECK_LAUNCH();
    a.phase = 2;                                             // every pair replays its candidate's plan
    n = P < full ? P : full;
    a.threads = (n + kThreadsPerBlock - 1) / kThreadsPerBlock * kThreadsPerBlock;
    hipLaunchKernelGGL(k_zb, dim3((unsigned)(a.threads / kThreadsPerBlock)), dim3(kThreadsPerBlock), 0, st, a);
    ADAPTRA_CHECK_LAUNCH();
    return ADAPTRA_OK;
}

}  // extern "C"

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
// creates and refreshes the next-action times of the stages involved.  Ready times posted
// later are strictly later than the current time because forward and backward ops last at
// least 1 us (a precondition of this entry point), so the decision at the earliest action
// time can never be overturned.  Within a type ops run in micro-batch order and their ready
// times are non-decreasing, so "the lowest available micro-batch" is a per-type cursor, and
// the ready times of one (stage, type) form a queue: posted in micro-batch order, consumed in
// micro-batch order.
//
// Where the state lives.  The queues (up to N entries each) are in global scratch, laid out
// [index][thread] so that a wavefront's access is one 256-byte line.  Everything a decision
// needs is on chip, in LDS laid out [stage][array][lane] (conflict-free for any per-lane
// stage index; a stage's fields at fixed offsets from its base): per stage the busy-until time, the cached next-action time, the three
// cursors, the warm-up quota x, and the HEAD of each of the three queues (the ready time of
// the cursor's micro-batch, or "not posted yet").  A post that lands on the head goes straight
// to LDS and never to memory; a step touches global memory only to append behind a head and
// to fetch the next head after a consume -- about three accesses instead of the forty of a
// version that kept all state in memory.  One wavefront per block, 9 S KiB / 4 of LDS each.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"

namespace {

constexpr int kInf = INT32_MAX;
constexpr int kZbBlock = 64;          // one wavefront per block: LDS, not threads, bounds the occupancy
constexpr int kZbArrays = 9;          // busy, act, nF, nB, nW, headF, headB, headW, x

struct ZbArgs {
    int S, N;
    const int *t_f, *t_b, *t_w;
    long long C, K;
    const int *w, *cf, *cb;
    long long plan_scenario;      // -1: every pair generates under its own scenario
    int phase;                    // 0: generate (+ outputs unless a plan is wanted), 1: record plans, 2: replay plans
    int *out_makespan, *out_bubble;
    int *scratch;                 // queues [S][3][N][threads]
    int *plans;                   // [C][S][3N], ops as type * N + m
    long long threads;
};

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int imax2(int a, int b) { return a > b ? a : b; }

// The lane's view of its state.
struct Lane {
    int *lds;                     // this lane's column: element (stage, array) at lds[(stage * kZbArrays + array) * 64]:
                                  // a stage's fields sit at fixed offsets from the stage's base address
    const int *dur_table;         // LDS copy of t_f, t_b, t_w: [3][S]
    int *queue;                   // this thread's column of the global queues
    long long nt;
    int S, N;
    __device__ int &busy(int i) const { return lds[(i * kZbArrays + 0) * 64]; }
    __device__ int &act(int i) const { return lds[(i * kZbArrays + 1) * 64]; }
    __device__ int &count(int i, int ty) const { return lds[(i * kZbArrays + 2 + ty) * 64]; }
    __device__ int &head(int i, int ty) const { return lds[(i * kZbArrays + 5 + ty) * 64]; }
    __device__ int &quota(int i) const { return lds[(i * kZbArrays + 8) * 64]; }
    __device__ int &ready(int i, int ty, int m) const { return queue[(((long long)i * 3 + ty) * N + m) * nt]; }
    __device__ int cursor(int i, int ty) const { return count(i, ty); }
    __device__ void advance(int i, int ty) const { count(i, ty) += 1; }
    __device__ int x(int i) const { return quota(i); }
    __device__ int done(int i) const { return count(i, 0) + count(i, 1) + count(i, 2); }

    // Ready times of (i, ty) posted so far: a forward of stage i is posted when the forward of
    // stage i-1 starts (stage 0: all at time 0), a backward when the backward of stage i+1
    // starts (last stage: when its own forward starts), a weight op when the stage's own
    // backward starts.
    __device__ int posted(int i, int ty) const {
        if (ty == 0) return i == 0 ? N : cursor(i - 1, 0);
        if (ty == 1) return i == S - 1 ? cursor(i, 0) : cursor(i + 1, 1);
        return cursor(i, 1);
    }
    // Appends the ready time r of micro-batch m to the queue of (i, ty).
    __device__ void post(int i, int ty, int m, int r) const {
        if (m == cursor(i, ty)) head(i, ty) = r;
        else ready(i, ty, m) = r;
    }
    // Next action of stage i from what has been posted so far (Algorithm 3): the time it can
    // act, or kInf if nothing it may run has been posted yet.  With a plan the next op is the
    // plan's, whatever its type.
    __device__ void refresh(int i, const int *plan) const {
        const int b = busy(i);
        if (plan) {
            const int d = done(i);
            if (d >= 3 * N) { act(i) = kInf; return; }
            const int r = head(i, plan[d] / N);
            act(i) = r == kInf ? kInf : imax2(b, r);
            return;
        }
        const int rf = head(i, 0);
        if (cursor(i, 0) < x(i)) {                              // warm-up: forwards only
            act(i) = rf == kInf ? kInf : imax2(b, rf);
            return;
        }
        const int first = imin(head(i, 1), imin(rf, head(i, 2)));
        act(i) = first == kInf ? kInf : imax2(b, first);
    }
};

__global__ __launch_bounds__(kZbBlock) void k_zb(ZbArgs a) {
    extern __shared__ int zb_lds[];
    const long long tid = (long long)blockIdx.x * kZbBlock + threadIdx.x;
    const int S = a.S, N = a.N;
    const long long n_items = a.phase == 1 ? a.C : a.C * a.K;
    int *const dur_table = zb_lds + kZbArrays * S * 64;
    for (int i = threadIdx.x; i < 3 * S; i += kZbBlock)
        dur_table[i] = i < S ? a.t_f[i] : (i < 2 * S ? a.t_b[i - S] : a.t_w[i - 2 * S]);
    __syncthreads();
    const Lane L{zb_lds + threadIdx.x, dur_table, a.scratch + tid, a.threads, S, N};
    for (long long item = tid; item < n_items; item += a.threads) {
        const long long c = a.phase == 1 ? item : item % a.C;
        const long long k = a.phase == 1 ? a.plan_scenario : item / a.C;
        const int *plan_base = a.phase == 2 ? a.plans + c * (long long)S * 3 * N : nullptr;
        int *record = a.phase == 1 ? a.plans + c * (long long)S * 3 * N : nullptr;
        // set-up: nothing posted except the forwards of stage 0 (available at time 0)
        for (int i = 0; i < S; ++i) {
            int wi = a.w[(long long)i * a.C + c];
            wi = wi < 0 ? 0 : (wi > N - 1 ? N - 1 : wi);
            L.busy(i) = 0;
            L.count(i, 0) = 0; L.count(i, 1) = 0; L.count(i, 2) = 0;
            L.quota(i) = wi + 1;                                // x_i = w_i + 1 warm-up forwards
            L.head(i, 0) = i == 0 ? 0 : kInf;
            L.head(i, 1) = kInf;
            L.head(i, 2) = kInf;
        }
        for (int i = 0; i < S; ++i) L.refresh(i, plan_base ? plan_base + (long long)i * 3 * N : nullptr);

        const int total = 3 * S * N;
        int makespan = 0;
        for (int step = 0; step < total; ++step) {
            int i = 0, t = L.act(0);
            for (int j = 1; j < S; ++j) {
                const int tj = L.act(j);
                if (tj < t) { t = tj; i = j; }
            }
            if (t == kInf) { makespan = kInf; break; }          // cannot happen for valid input
            const int *plan_i = plan_base ? plan_base + (long long)i * 3 * N : nullptr;
            const int done_i = L.done(i);
            int ty;
            if (plan_i) ty = plan_i[done_i] / N;
            else if (L.cursor(i, 0) < L.x(i)) ty = 0;
            else ty = L.head(i, 1) <= t ? 1 : (L.head(i, 0) <= t ? 0 : 2);   // priority B > F > W among those ready at t
            const int m = L.cursor(i, ty);
            const int dur = L.dur_table[ty * S + i];
            const int fin = t + dur;
            L.busy(i) = fin;
            makespan = imax2(makespan, fin);
            if (record) record[(long long)i * 3 * N + done_i] = ty * N + m;
            // consume: the queue's next entry becomes the head (stage 0's forwards are all ready at 0)
            L.advance(i, ty);
            if (m + 1 < L.posted(i, ty)) L.head(i, ty) = (ty == 0 && i == 0) ? 0 : L.ready(i, ty, m + 1);
            else L.head(i, ty) = kInf;
            int lo = i, hi = i;
            if (ty == 0) {
                if (i < S - 1) { L.post(i + 1, 0, m, fin + a.cf[(long long)i * a.K + k]); hi = i + 1; }
                else L.post(i, 1, m, fin);
            } else if (ty == 1) {
                L.post(i, 2, m, fin);
                if (i > 0) { L.post(i - 1, 1, m, fin + a.cb[(long long)(i - 1) * a.K + k]); lo = i - 1; }
            }
            for (int j = lo; j <= hi; ++j) L.refresh(j, plan_base ? plan_base + (long long)j * 3 * N : nullptr);
        }
        if (a.phase != 1) {
            const long long P = a.C * a.K;
            a.out_makespan[item] = makespan;
            if (a.out_bubble)
                for (int i = 0; i < S; ++i)
                    a.out_bubble[(long long)i * P + item] =
                        makespan == kInf ? kInf : makespan - N * (dur_table[i] + dur_table[S + i] + dur_table[2 * S + i]);
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
    // Enough threads to fill the chip at the occupancy the LDS state allows (at most 160 KiB
    // per CU, 32 wavefronts per CU, 256 CUs), within about 2 GiB of queue memory.
    const long long per_thread = 3ll * S * N * 4;
    const long long lds_per_wave = (long long)kZbArrays * S * 64 * 4 + 3ll * S * 4;
    long long waves_per_cu = (160ll << 10) / lds_per_wave;
    if (waves_per_cu > 32) waves_per_cu = 32;
    if (waves_per_cu < 1) return false;
    long long nt = 256 * waves_per_cu * kZbBlock;
    const long long cap = (2048ll << 20) / per_thread / kZbBlock * kZbBlock;
    if (nt > cap) nt = cap;
    if (nt < 16 * kZbBlock) nt = 16 * kZbBlock;
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
    const size_t lds = (size_t)kZbArrays * a.S * 64 * 4 + (size_t)3 * a.S * 4;
    if (lds > 48 * 1024) {                                   // above the default dynamic-LDS limit
        hipError_t e = hipFuncSetAttribute((const void *)k_zb, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return adaptra_detail::hip_fail(e);
    }
    const long long full = p.threads;
    auto launch = [&](long long items) -> int {              // threads: a multiple of the block, at most `full`
        const long long n = items < full ? items : full;
        a.threads = (n + kZbBlock - 1) / kZbBlock * kZbBlock;
        hipLaunchKernelGGL(k_zb, dim3((unsigned)(a.threads / kZbBlock)), dim3(kZbBlock), lds, st, a);
        ADAPTRA_CHECK_LAUNCH();
        return ADAPTRA_OK;
    };
    if (plan_scenario < 0) {
        a.phase = 0;
        return launch(P);
    }
    a.phase = 1;                                             // one plan per candidate, under the plan scenario
    int rc = launch(a.C);
    if (rc) return rc;
    a.phase = 2;                                             // every pair replays its candidate's plan
    return launch(P);
}

}  // extern "C"

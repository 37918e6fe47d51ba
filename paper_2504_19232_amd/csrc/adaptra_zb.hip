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
// Where the state lives.  Only two kinds of ready time ever have to be remembered: a forward's
// (posted by the stage before) and a backward's (posted by the stage after).  A weight op is
// available as soon as its backward has STARTED -- it becomes ready when that backward finishes,
// and its own stage is busy until then anyway -- so "a W is available" is just nW < nB; the same
// holds for the last stage's backwards (ready when its own forward finishes: nB < nF) and for
// stage 0's forwards (ready at time 0).  The two real queues per stage (up to N entries each)
// are in global scratch, laid out [index][thread] so that a wavefront's access is one 256-byte
// line.  Everything a decision needs is on chip, in LDS: the cached next-action times as one
// array [stage][lane] (the earliest-action scan reads two stages per instruction at static
// offsets), and per stage a block of eight fields [stage][field][lane] at fixed offsets from the
// stage's base (conflict-free for any per-lane stage index): busy-until, the cursors nF, nB and
// nW (nW shares a word with the warm-up quota x), the HEAD of each queue (the ready time of the
// cursor's micro-batch, or "nothing posted"), and the delays of the two links the stage sends
// over.  A post that lands on an empty queue goes straight to the head in LDS and never to
// memory, and only then can it change the receiver's next action; a step touches global memory
// only to append behind a head and to fetch the next head after a consume.  One wavefront per
// block, (8 S + 8 ceil(S/8)) x 256 bytes of LDS each.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"

namespace {

constexpr int kInf = INT32_MAX;
constexpr int kZbBlock = 64;          // one wavefront per block: LDS, not threads, bounds the occupancy
constexpr int kZbFields = 8;          // per-stage block of LDS fields, each 64 lanes wide
enum : int { fBusy = 0, fNF = 1, fNB = 2, fNWX = 3, fHeadF = 4, fHeadB = 5, fCF = 6, fCB = 7 };
constexpr int kStage = kZbFields * 64;   // ints from one stage's block to the next
constexpr int kNone = 3;              // "no op left" in a plan (types: 0 = F, 1 = B, 2 = W)

struct ZbArgs {
    int S, N;
    const int *t_f, *t_b, *t_w;
    long long C, K;
    const int *w, *cf, *cb;
    long long plan_scenario;      // -1: every pair generates under its own scenario
    int *out_makespan, *out_bubble;
    int *scratch;                 // queues [S][2][N][threads]
    uint8_t *plans;               // [C][S][3N], op types in the order a stage ran them
    unsigned threads;
};

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int imax2(int a, int b) { return a > b ? a : b; }

// Next action of a stage from its own fields (Algorithm 3): the time it can act, or kInf if
// nothing it may run has been posted yet.  nWx = nW | x << 16; when a plan is replayed
// (PHASE 2) the upper half holds the type of the plan's next op instead of the quota.
template <int PHASE>
__device__ __forceinline__ int next_action(int busy, int nF, int nB, int nWx, int headF, int headB) {
    const int headW = (nWx & 0xffff) < nB ? 0 : kInf;            // ready since its backward finished
    const int hi = (int)((unsigned)nWx >> 16);
    int first;
    if (PHASE == 2) first = hi == 0 ? headF : (hi == 1 ? headB : (hi == 2 ? headW : kInf));
    else first = nF < hi ? headF : imin(headB, imin(headF, headW));   // warm-up: forwards only
    return first == kInf ? kInf : imax2(busy, first);
}

// PHASE 0: generate with the policy and write the outputs; 1: generate under the plan scenario
// and record each stage's op types; 2: replay the recorded plans under every scenario.
template <int PHASE>
__global__ __launch_bounds__(kZbBlock) void k_zb(ZbArgs a) {
    extern __shared__ int zb_lds[];
    const long long tid = (long long)blockIdx.x * kZbBlock + threadIdx.x;
    const int S = a.S, N = a.N, Spad = (S + 7) & ~7;
    const long long n_items = PHASE == 1 ? a.C : a.C * a.K;
    int *const act = zb_lds + threadIdx.x;                        // [Spad][64]
    int *const fld = zb_lds + Spad * 64 + threadIdx.x;            // [S][kZbFields][64]
    int *const dur = zb_lds + Spad * 64 + S * kStage;             // [S][4]: t_f, t_b, t_w, 0
    for (int i = threadIdx.x; i < 4 * S; i += kZbBlock) {
        const int s = i >> 2, ty = i & 3;
        dur[i] = ty == 0 ? a.t_f[s] : (ty == 1 ? a.t_b[s] : (ty == 2 ? a.t_w[s] : 0));
    }
    __syncthreads();
    int *const queue = a.scratch + tid;
    const unsigned nt = a.threads;
    for (long long item = tid; item < n_items; item += nt) {
        const long long c = PHASE == 1 ? item : item % a.C;
        const long long k = PHASE == 1 ? a.plan_scenario : item / a.C;
        uint8_t *const plan = a.plans + c * (long long)S * 3 * N;     // stage i's ops at plan + i * 3N
        // set-up: nothing posted except the forwards of stage 0 (available at time 0)
        for (int i = S; i < Spad; ++i) act[i * 64] = kInf;
        for (int i = 0; i < S; ++i) {
            int wi = a.w[(long long)i * a.C + c];
            wi = wi < 0 ? 0 : (wi > N - 1 ? N - 1 : wi);
            const int hi = PHASE == 2 ? plan[(long long)i * 3 * N] : wi + 1;   // x_i = w_i + 1 warm-up forwards
            int *st = fld + i * kStage;
            st[fBusy * 64] = 0;
            st[fNF * 64] = 0;
            st[fNB * 64] = 0;
            st[fNWX * 64] = hi << 16;
            st[fHeadF * 64] = i == 0 ? 0 : kInf;
            st[fHeadB * 64] = kInf;
            st[fCF * 64] = i < S - 1 ? a.cf[(long long)i * a.K + k] : 0;
            st[fCB * 64] = i > 0 ? a.cb[(long long)(i - 1) * a.K + k] : 0;
            act[i * 64] = next_action<PHASE>(0, 0, 0, hi << 16, i == 0 ? 0 : kInf, kInf);
        }

        const int total = 3 * S * N;
        int makespan = 0;
        for (int step = 0; step < total; ++step) {
            // the stage whose next action is earliest, ties to the lower stage
            int i = 0, t = kInf;
            for (int b = 0; b < Spad; b += 8) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int tj = act[(b + j) * 64];
                    if (tj < t) { t = tj; i = b + j; }
                }
            }
            if (t == kInf) { makespan = kInf; break; }          // cannot happen for valid input
            int *const st = fld + i * kStage;
            int nF = st[fNF * 64], nB = st[fNB * 64], nWx = st[fNWX * 64];
            int headF = st[fHeadF * 64], headB = st[fHeadB * 64];
            const int hi = (int)((unsigned)nWx >> 16), nW = nWx & 0xffff;
            int ty;
            if (PHASE == 2) ty = hi;
            else ty = nF < hi ? 0 : (headB <= t ? 1 : (headF <= t ? 0 : 2));   // priority B > F > W among those ready at t
            const int m = ty == 0 ? nF : (ty == 1 ? nB : nW);
            const int done = nF + nB + nW;
            const int fin = t + dur[i * 4 + ty];
            makespan = imax2(makespan, fin);
            if (PHASE == 1) plan[(long long)i * 3 * N + done] = (uint8_t)ty;
            nF += ty == 0;
            nB += ty == 1;
            nWx += ty == 2;
            if (PHASE == 2) {
                const int next_ty = done + 1 < 3 * N ? plan[(long long)i * 3 * N + done + 1] : kNone;
                nWx = (nWx & 0xffff) | next_ty << 16;
            }
            const bool last = i == S - 1;
            if (ty < 2) {
                // consume: the queue's next entry becomes the head.  Entries posted so far = ops of
                // that type the producing stage has started; stage 0's forwards and the last
                // stage's backwards come from no other stage and are ready whenever it is idle.
                const bool own = ty == 0 ? i == 0 : last;
                const int *producer = own ? st + fNF * 64 : (ty == 0 ? st - kStage + fNF * 64 : st + kStage + fNB * 64);
                const int posted = own ? (ty == 0 ? N : nF) : *producer;
                int next = kInf;
                if (m + 1 < posted) next = own ? 0 : queue[(unsigned long long)(unsigned)((i * 2 + ty) * N + m + 1) * nt];
                if (ty == 0) headF = next; else headB = next;
            }
            if (last && ty == 0) headB = 0;                     // its own forward makes a backward available
            st[fBusy * 64] = fin;
            st[fNF * 64] = nF;
            st[fNB * 64] = nB;
            st[fNWX * 64] = nWx;
            st[fHeadF * 64] = headF;
            st[fHeadB * 64] = headB;
            act[i * 64] = next_action<PHASE>(fin, nF, nB, nWx, headF, headB);
            // post the ready time this op creates: F(i,m) -> F(i+1,m), B(i,m) -> B(i-1,m)
            const int j = ty == 0 ? i + 1 : i - 1;
            if (ty < 2 && j >= 0 && j < S) {
                const int r = fin + st[(ty == 0 ? fCF : fCB) * 64];
                int *const sj = ty == 0 ? st + kStage : st - kStage;
                int hFj = sj[fHeadF * 64], hBj = sj[fHeadB * 64];
                if ((ty == 0 ? hFj : hBj) == kInf) {            // empty queue: r is its head, the receiver may act earlier
                    if (ty == 0) hFj = r; else hBj = r;
                    sj[(fHeadF + ty) * 64] = r;
                    act[j * 64] = next_action<PHASE>(sj[fBusy * 64], sj[fNF * 64], sj[fNB * 64], sj[fNWX * 64], hFj, hBj);
                } else {
                    queue[(unsigned long long)(unsigned)((j * 2 + ty) * N + m) * nt] = r;
                }
            }
        }
        if (PHASE != 1) {
            const long long P = a.C * a.K;
            a.out_makespan[item] = makespan;
            if (a.out_bubble)
                for (int i = 0; i < S; ++i)
                    a.out_bubble[(long long)i * P + item] =
                        makespan == kInf ? kInf : makespan - N * (dur[i * 4] + dur[i * 4 + 1] + dur[i * 4 + 2]);
        }
    }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct ZbPlan {
    unsigned threads;
    size_t lds, off_scratch, off_plans, total;
};

bool plan_zb(int S, int N, long long C, long long K, ZbPlan *p) {
    if (S < 1 || S > ADAPTRA_MAX_STAGES || N < 1 || N > ADAPTRA_MAX_MICROBATCHES) return false;
    if (C < 1 || C > INT32_MAX || K < 1 || K > INT32_MAX) return false;
    // Enough threads to fill the chip at the occupancy the LDS state allows (at most 160 KiB
    // per CU, 32 wavefronts per CU, 256 CUs), within about 2 GiB of queue memory.
    const long long per_thread = 2ll * S * N * 4;
    const int Spad = (S + 7) & ~7;
    p->lds = ((size_t)Spad * 64 + (size_t)S * kStage + 4 * (size_t)S) * 4;
    long long waves_per_cu = (160ll << 10) / (long long)p->lds;
    if (waves_per_cu > 32) waves_per_cu = 32;
    if (waves_per_cu < 1) return false;
    long long nt = 256 * waves_per_cu * kZbBlock;
    const long long cap = (2048ll << 20) / per_thread / kZbBlock * kZbBlock;
    if (nt > cap) nt = cap;
    if (nt < 16 * kZbBlock) nt = 16 * kZbBlock;
    p->threads = (unsigned)nt;
    size_t o = 0;
    p->off_scratch = o; o += align256((size_t)nt * per_thread);
    p->off_plans = o;   o += align256((size_t)C * S * 3 * N);
    p->total = o;
    return true;
}

template <int PHASE>
int launch_zb(ZbArgs a, long long items, unsigned full, size_t lds, hipStream_t st) {
    if (lds > 48 * 1024) {                                   // above the default dynamic-LDS limit
        hipError_t e = hipFuncSetAttribute((const void *)k_zb<PHASE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return adaptra_detail::hip_fail(e);
    }
    const long long n = items < (long long)full ? items : (long long)full;
    a.threads = (unsigned)((n + kZbBlock - 1) / kZbBlock * kZbBlock);   // a multiple of the block, at most `full`
    hipLaunchKernelGGL(k_zb<PHASE>, dim3(a.threads / kZbBlock), dim3(kZbBlock), lds, st, a);
    ADAPTRA_CHECK_LAUNCH();
    return ADAPTRA_OK;
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
    a.plans = (uint8_t *)workspace + p.off_plans;
    const long long P = a.C * a.K;
    if (plan_scenario < 0) return launch_zb<0>(a, P, p.threads, p.lds, st);
    int rc = launch_zb<1>(a, a.C, p.threads, p.lds, st);      // one plan per candidate, under the plan scenario
    if (rc) return rc;
    return launch_zb<2>(a, P, p.threads, p.lds, st);         // every pair replays its candidate's plan
}

}  // extern "C"

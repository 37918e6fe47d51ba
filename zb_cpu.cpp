#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <limits.h>
#define __device__
#define __global__
#define __forceinline__ inline
#define __launch_bounds__(x)
#define __syncthreads()
#define ADAPTRA_MAX_STAGES 64
#define ADAPTRA_MAX_MICROBATCHES 32768
struct Idx { unsigned x; };
static Idx blockIdx, threadIdx;
static int *zb_lds;


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

extern "C" int zb_cpu(int S, int N, long long C, long long K, const int *tf, const int *tb, const int *tw,
                      const int *w, const int *cf, const int *cb, long long plan_scenario,
                      int *out_mk, int *out_bub, unsigned threads) {
    ZbArgs a{}; a.S=S; a.N=N; a.t_f=tf; a.t_b=tb; a.t_w=tw; a.C=C; a.K=K; a.w=w; a.cf=cf; a.cb=cb;
    a.plan_scenario=plan_scenario; a.out_makespan=out_mk; a.out_bubble=out_bub;
    const int Spad=(S+7)&~7;
    size_t lds_ints=(size_t)Spad*64+(size_t)S*kStage+4*(size_t)S;
    a.scratch=(int*)malloc((size_t)threads*2*S*N*4);
    a.plans=(uint8_t*)malloc((size_t)C*S*3*N);
    auto run=[&](int phase, long long items){
        long long n = items < threads ? items : threads;
        unsigned th=(unsigned)((n+63)/64*64);
        for (unsigned b=0;b<th/64;++b){
            zb_lds=(int*)malloc(lds_ints*4);
            blockIdx.x=b;
            ZbArgs f=a; f.threads=th; f.C=0;   // fill pass: tables only
            for(unsigned t=0;t<64;++t){ threadIdx.x=t; if(phase==0)k_zb<0>(f); else if(phase==1)k_zb<1>(f); else k_zb<2>(f);}
            f.C=a.C;
            for(unsigned t=0;t<64;++t){ threadIdx.x=t; if(phase==0)k_zb<0>(f); else if(phase==1)k_zb<1>(f); else k_zb<2>(f);}
            free(zb_lds);
        }
    };
    if (plan_scenario<0) run(0,C*K); else { run(1,C); run(2,C*K); }
    free(a.scratch); free(a.plans);
    return 0;
}

#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <limits.h>
#include <pthread.h>
#include <thread>
#include <vector>
#define __device__
#define __global__
#define __forceinline__ inline
#define __launch_bounds__(x)
#define __shared__ static
#define atomicAdd(p, v) __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST)
static pthread_barrier_t bar;
#define __syncthreads() pthread_barrier_wait(&bar)
#define ADAPTRA_MAX_STAGES 64
#define ADAPTRA_MAX_MICROBATCHES 32768
struct Idx { unsigned x; };
struct int4 { int x, y, z, w; };
struct int2 { int x, y; };
static Idx blockIdx, gridDim;
static thread_local Idx threadIdx;
static int *zb_lds;


constexpr int kInf = INT32_MAX;
constexpr int kZbBlock = 64;          // one wavefront per block: LDS, not threads, bounds the occupancy
constexpr int kZbFields = 4;          // per-stage block of LDS fields, each 64 lanes wide
enum : int { fNFB = 0, fNWX = 1, fHeadF = 2, fHeadB = 3 };   // nFB = nF | nB << 16, nWx = nW | x << 16
constexpr int kStage = kZbFields * 64;   // ints from one stage's block to the next
constexpr int kNone = 3;              // "no op left" in a plan (types: 0 = F, 1 = B, 2 = W)
// A head holds the ready time of the queue's first entry (>= 0), or, while the queue is empty,
// the complement of the stage's busy-until time (< 0): read as unsigned, "empty" sorts after
// every time, and a post that lands on an empty queue -- the only one that makes the receiver
// look at its next action again -- finds the receiver's busy-until time in the slot it fills.
__device__ __forceinline__ unsigned empty_head(int busy) { return ~(unsigned)busy; }
__device__ __forceinline__ bool is_empty(unsigned head) { return (int)head < 0; }

struct ZbArgs {
    int S, N;
    const int *t_f, *t_b, *t_w;
    long long C, K;
    const int *w, *cf, *cb;
    long long plan_scenario;      // -1: every pair generates under its own scenario
    int *out_makespan, *out_bubble;
    int *scratch;                 // queues [S][2][N][threads]
    uint8_t *plans;               // [C][S][3N], op types in the order a stage ran them
    unsigned threads;             // of the launch = stride of the queues
    unsigned long long *next_unit;   // work counter of this launch, zero when it starts
};

__device__ __forceinline__ unsigned umin(unsigned a, unsigned b) { return a < b ? a : b; }
__device__ __forceinline__ int imax2(int a, int b) { return a > b ? a : b; }

// Next action of a stage from its own fields (Algorithm 3): the time it can act, or kInf if
// nothing it may run has been posted yet.  When a plan is replayed (PHASE 2) the upper half of
// nWx holds the type of the plan's next op instead of the quota.
template <int PHASE>
__device__ __forceinline__ int next_action(int busy, int nFB, int nWx, unsigned headF, unsigned headB) {
    const int nF = nFB & 0xffff, nB = (int)((unsigned)nFB >> 16);
    const unsigned headW = (nWx & 0xffff) < nB ? 0u : ~0u;       // ready since its backward finished
    const int hi = (int)((unsigned)nWx >> 16);
    unsigned first;
    if (PHASE == 2) first = hi == 0 ? headF : (hi == 1 ? headB : (hi == 2 ? headW : ~0u));
    else first = nF < hi ? headF : umin(headB, umin(headF, headW));   // warm-up: forwards only
    return is_empty(first) ? kInf : imax2(busy, (int)first);
}

// PHASE 0: generate with the policy and write the outputs; 1: generate under the plan scenario
// and record each stage's op types; 2: replay the recorded plans under every scenario.
template <int PHASE>
__global__ __launch_bounds__(kZbBlock) void k_zb(ZbArgs a) {
    const int S = a.S, N = a.N, Spad = (S + 7) & ~7;
    int *const act = zb_lds + threadIdx.x;                        // [Spad][64]
    int *const fld = zb_lds + Spad * 64 + threadIdx.x;            // [S][kZbFields][64]
    int *const dur = zb_lds + Spad * 64 + S * kStage;             // [S][4]: t_f, t_b, t_w, 0
    int *const delay = dur + 4 * S;                               // [S][2]: forward delay of link i -> i+1, backward delay of link i-1 <- i
    for (int i = threadIdx.x; i < 4 * S; i += kZbBlock) {
        const int s = i >> 2, ty = i & 3;
        dur[i] = ty == 0 ? a.t_f[s] : (ty == 1 ? a.t_b[s] : (ty == 2 ? a.t_w[s] : 0));
    }
    int *const queue = a.scratch + ((long long)blockIdx.x * kZbBlock + threadIdx.x);
    const unsigned nt = a.threads;
    // A unit of work = one scenario x 64 consecutive candidates (the last chunk may be short:
    // its spare lanes repeat the last candidate and write nothing).  Wavefronts draw units from
    // a counter, so one that becomes resident late (the launch may hold a few more than fit at
    // once) takes what is left instead of a fixed share.
    __shared__ long long unit_drawn;
    const long long chunks = (a.C + kZbBlock - 1) / kZbBlock;
    const long long n_units = PHASE == 1 ? chunks : chunks * a.K;
    for (;;) {
        __syncthreads();                                          // the previous unit is finished in every lane
        if (threadIdx.x == 0) unit_drawn = (long long)atomicAdd(a.next_unit, 1ull);
        __syncthreads();
        const long long unit = unit_drawn;
        if (unit >= n_units) break;
        const long long k = PHASE == 1 ? a.plan_scenario : unit / chunks;
        const long long c_lane = (unit % chunks) * kZbBlock + threadIdx.x;
        const bool live = c_lane < a.C;
        const long long c = live ? c_lane : a.C - 1;
        uint8_t *const plan = a.plans + c * (long long)S * 3 * N;     // stage i's ops at plan + i * 3N
        for (int i = threadIdx.x; i < S; i += kZbBlock) {
            delay[i * 2] = i < S - 1 ? a.cf[(long long)i * a.K + k] : 0;
            delay[i * 2 + 1] = i > 0 ? a.cb[(long long)(i - 1) * a.K + k] : 0;
        }
        __syncthreads();
        // set-up: nothing posted except the forwards of stage 0 (available at time 0)
        for (int i = S; i < Spad; ++i) act[i * 64] = kInf;
        for (int i = 0; i < S; ++i) {
            int wi = a.w[(long long)i * a.C + c];
            wi = wi < 0 ? 0 : (wi > N - 1 ? N - 1 : wi);
            const int hi = PHASE == 2 ? plan[(long long)i * 3 * N] : wi + 1;   // x_i = w_i + 1 warm-up forwards
            int *st = fld + i * kStage;
            st[fNFB * 64] = 0;
            st[fNWX * 64] = hi << 16;
            st[fHeadF * 64] = (int)(i == 0 ? 0u : empty_head(0));
            st[fHeadB * 64] = (int)empty_head(0);
            act[i * 64] = next_action<PHASE>(0, 0, hi << 16, i == 0 ? 0u : empty_head(0), empty_head(0));
        }

        const int total = 3 * S * N;
        int makespan = 0;
        for (int step = 0; step < total; ++step) {
            // the stage whose next action is earliest, ties to the lower stage
            int i = 0, t = kInf;
            for (int b = 0; b < Spad; b += 8) {
                int tb = act[b * 64], jb = 0;
#pragma unroll
                for (int j = 1; j < 8; ++j) {
                    const int tj = act[(b + j) * 64];
                    if (tj < tb) { tb = tj; jb = j; }
                }
                if (tb < t) { t = tb; i = b + jb; }
            }
            if (t == kInf) { makespan = kInf; break; }          // cannot happen for valid input
            // Everything whose address depends on the stage alone is read now, in one round trip:
            // the stage's fields, its three durations and two delays, the cursors of the two
            // producing stages.
            int *const st = fld + i * kStage;
            const bool first = i == 0, last = i == S - 1;
            int nFB = st[fNFB * 64], nWx = st[fNWX * 64];
            unsigned headF = (unsigned)st[fHeadF * 64], headB = (unsigned)st[fHeadB * 64];
            const int4 dur_i = *reinterpret_cast<const int4 *>(dur + i * 4);
            const int2 delay_i = *reinterpret_cast<const int2 *>(delay + i * 2);
            const int nFB_prev = *(first ? st + fNFB * 64 : st - kStage + fNFB * 64);
            const int nFB_next = *(last ? st + fNFB * 64 : st + kStage + fNFB * 64);
            const int nF = nFB & 0xffff, nB = (int)((unsigned)nFB >> 16);
            const int hi = (int)((unsigned)nWx >> 16), nW = nWx & 0xffff;
            int ty;
            if (PHASE == 2) ty = hi;
            else ty = nF < hi ? 0 : (headB <= (unsigned)t ? 1 : (headF <= (unsigned)t ? 0 : 2));   // priority B > F > W among those ready at t
            // the stage this op posts to: F(i,m) -> F(i+1,m), B(i,m) -> B(i-1,m); its fields are
            // read before this stage's own are written (another stage, or unused)
            const int j = ty == 0 ? i + 1 : i - 1;
            const bool posts = ty < 2 && j >= 0 && j < S;
            int *const sj = posts ? (ty == 0 ? st + kStage : st - kStage) : st;
            const int nFB_j = sj[fNFB * 64], nWx_j = sj[fNWX * 64];
            unsigned headF_j = (unsigned)sj[fHeadF * 64], headB_j = (unsigned)sj[fHeadB * 64];

            const int m = ty == 0 ? nF : (ty == 1 ? nB : nW);
            const int done = nF + nB + nW;
            const int fin = t + (ty == 0 ? dur_i.x : (ty == 1 ? dur_i.y : dur_i.z));
            makespan = imax2(makespan, fin);
            if (PHASE == 1 && live) plan[(long long)i * 3 * N + done] = (uint8_t)ty;
            nFB += ty == 0 ? 1 : (ty == 1 ? 0x10000 : 0);
            nWx += ty == 2;
            if (PHASE == 2) {
                const int next_ty = done + 1 < 3 * N ? plan[(long long)i * 3 * N + done + 1] : kNone;
                nWx = (nWx & 0xffff) | next_ty << 16;
            }
            if (ty < 2) {
                // consume: the queue's next entry becomes the head.  Entries posted so far = ops of
                // that type the producing stage has started; stage 0's forwards and the last
                // stage's backwards come from no other stage and are ready whenever it is idle.
                const bool own = ty == 0 ? first : last;
                const int posted = ty == 0 ? (first ? N : (nFB_prev & 0xffff))
                                           : (last ? (nFB & 0xffff) : (int)((unsigned)nFB_next >> 16));
                unsigned next = ~0u;
                if (m + 1 < posted) next = own ? 0u : (unsigned)queue[(unsigned long long)(unsigned)((i * 2 + ty) * N + m + 1) * nt];
                if (ty == 0) headF = next; else headB = next;
            }
            if (is_empty(headF)) headF = empty_head(fin);       // busy until fin from now on
            if (is_empty(headB)) headB = empty_head(fin);
            if (last && ty == 0) headB = 0;                     // its own forward makes a backward available
            st[fNFB * 64] = nFB;
            st[fNWX * 64] = nWx;
            st[fHeadF * 64] = (int)headF;
            st[fHeadB * 64] = (int)headB;
            act[i * 64] = next_action<PHASE>(fin, nFB, nWx, headF, headB);
            if (posts) {
                const int r = fin + (ty == 0 ? delay_i.x : delay_i.y);
                const unsigned slot = ty == 0 ? headF_j : headB_j;
                if (is_empty(slot)) {                           // r becomes the head: the receiver may act earlier
                    if (ty == 0) headF_j = (unsigned)r; else headB_j = (unsigned)r;
                    sj[(fHeadF + ty) * 64] = r;
                    act[j * 64] = next_action<PHASE>((int)~slot, nFB_j, nWx_j, headF_j, headB_j);
                } else {
                    queue[(unsigned long long)(unsigned)((j * 2 + ty) * N + m) * nt] = r;
                }
            }
        }
        if (PHASE != 1 && live) {
            const long long P = a.C * a.K, item = k * a.C + c;
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
    size_t lds_ints=(size_t)Spad*64+(size_t)S*kStage+6*(size_t)S;
    a.plans=(uint8_t*)malloc((size_t)C*S*3*N);
    pthread_barrier_init(&bar, nullptr, 64);
    auto run=[&](int phase, long long scen){
        long long units=(C+63)/64*scen;
        long long waves = units < threads/64 ? units : threads/64;
        a.threads=(unsigned)waves*64;
        a.scratch=(int*)malloc((size_t)a.threads*2*S*N*4);
        gridDim.x=(unsigned)waves;
        unsigned long long ctr=0; a.next_unit=&ctr;
        for (unsigned b=0;b<waves;++b){
            zb_lds=(int*)malloc(lds_ints*4);
            blockIdx.x=b;
            std::vector<std::thread> th;
            for(unsigned t=0;t<64;++t) th.emplace_back([&,t]{ threadIdx.x=t; if(phase==0)k_zb<0>(a); else if(phase==1)k_zb<1>(a); else k_zb<2>(a); });
            for(auto&x:th) x.join();
            free(zb_lds);
        }
        free(a.scratch);
    };
    if (plan_scenario<0) run(0,K); else { run(1,1); run(2,K); }
    free(a.plans);
    return 0;
}

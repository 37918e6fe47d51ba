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
#define __host__
#define __shared__ static
#define atomicAdd(p, v) __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST)
static pthread_barrier_t bar;
#define __syncthreads() pthread_barrier_wait(&bar)
#define ADAPTRA_MAX_STAGES 64
#define ADAPTRA_MAX_MICROBATCHES 32768
struct Idx { unsigned x; };
struct int4 { int x, y, z, w; };
struct int2 { int x, y; };
static Idx blockIdx, gridDim, blockDim;
static thread_local Idx threadIdx;
static int *zb_lds;


constexpr int kInf = INT32_MAX;
constexpr int kZbBlock = 64;          // one wavefront per block: LDS, not threads, bounds the occupancy
constexpr int kNone = 3;              // "no op left" in a plan (types: 0 = F, 1 = B, 2 = W)
// A head holds the ready time of the queue's first entry (>= 0), or, while the queue is empty,
// the complement of the stage's busy-until time (< 0): read as unsigned, "empty" sorts after
// every time, and a post that lands on an empty queue -- the only one that makes the receiver
// look at its next action again -- finds the receiver's busy-until time in the slot it fills.
__device__ __forceinline__ unsigned empty_head(int busy) { return ~(unsigned)busy; }
__device__ __forceinline__ bool is_empty(unsigned head) { return (int)head < 0; }

// The cursors of a stage (ops of each type started so far) and one more number `hi`: the
// warm-up quota x, or, when a plan is replayed, the types of the plan's next ops (2 bits each,
// the next one lowest).  Wide form, any N: two words, nF | nB << 16 and nW | hi << 16.  Narrow
// form, N <= 255 and never for a replay: one word, nF | nB << 8 | nW << 16 | hi << 24 -- one
// LDS field less per stage, i.e. more resident wavefronts.  The heads follow the cursors in a
// stage's block of fields.
template <bool NARROW>
struct Cursors {
    static constexpr int kFields = NARROW ? 3 : 4;       // fields of a stage's block, each 64 lanes wide
    static constexpr int kStage = kFields * 64;          // ints from one stage's block to the next
    static constexpr int kHeadF = (NARROW ? 1 : 2) * 64, kHeadB = kHeadF + 64;   // offsets in the block
    int a, b;
    __device__ __forceinline__ static Cursors start(int hi) {
        Cursors c;
        c.a = NARROW ? hi << 24 : 0;
        c.b = NARROW ? 0 : hi << 16;
        return c;
    }
    __device__ __forceinline__ static Cursors load(const int *st) {
        Cursors c;
        c.a = st[0];
        c.b = NARROW ? 0 : st[64];
        return c;
    }
    __device__ __forceinline__ void store(int *st) const {
        st[0] = a;
        if (!NARROW) st[64] = b;
    }
    __device__ __forceinline__ int nF() const { return NARROW ? a & 0xff : a & 0xffff; }
    __device__ __forceinline__ int nB() const { return NARROW ? (a >> 8) & 0xff : (int)((unsigned)a >> 16); }
    __device__ __forceinline__ int nW() const { return NARROW ? (a >> 16) & 0xff : b & 0xffff; }
    __device__ __forceinline__ int hi() const { return NARROW ? (int)((unsigned)a >> 24) : (int)((unsigned)b >> 16); }
    __device__ __forceinline__ void started(int ty) {
        if (NARROW) a += ty == 0 ? 1 : (ty == 1 ? 0x100 : 0x10000);
        else { a += ty == 0 ? 1 : (ty == 1 ? 0x10000 : 0); b += ty == 2; }
    }
    // replay only (wide form): the window of coming ops
    __device__ __forceinline__ void set_window(unsigned types) { b = (b & 0xffff) | (int)(types << 16); }
    __device__ __forceinline__ void advance_window() { b = (b & 0xffff) | (int)(((unsigned)b >> 2) & 0xffff0000u); }
};

struct ZbArgs {
    int S, N;
    const int *t_f, *t_b, *t_w;
    long long C, K;
    const int *w, *cf, *cb;
    long long plan_scenario;      // -1: every pair generates under its own scenario
    int *out_makespan, *out_bubble;
    int *scratch;                 // queues [S][2][N][threads]
    uint8_t *plans;               // [C][S][3N], op types in the order a stage ran them (written by PHASE 1)
    const uint32_t *packed;       // [ceil(C/64)][S][packed_words(N)][64 candidates], the same at 2 bits per op (see
                                  // packed_words), read by PHASE 2: the lanes of a wavefront read neighbouring words
    unsigned threads;             // of the launch = stride of the queues
    unsigned long long *next_unit;   // work counter of this launch, zero when it starts
};

__device__ __forceinline__ unsigned umin(unsigned a, unsigned b) { return a < b ? a : b; }
__device__ __forceinline__ int imax2(int a, int b) { return a > b ? a : b; }

// A packed plan holds 16 ops per word, 2 bits each, and consecutive words overlap by half: word
// q starts at op 8 q.  A window of kWindow = 8 ops that starts at any op therefore lies inside
// ONE word, (op / 8), at bit 2 (op % 8).  Words per stage, including the window at the very end:
__host__ __device__ inline int packed_words(int N) { return 3 * N / 8 + 1; }
constexpr int kWindow = 8;            // ops of a plan held on chip per stage (16 bits of `hi`)

// Next action of a stage from its own fields (Algorithm 3): the time it can act, or kInf if
// nothing it may run has been posted yet.
template <int PHASE, bool NARROW>
__device__ __forceinline__ int next_action(int busy, const Cursors<NARROW> &c, unsigned headF, unsigned headB) {
    const unsigned headW = c.nW() < c.nB() ? 0u : ~0u;           // ready since its backward finished
    unsigned first;
    if (PHASE == 2) {
        const int ty = c.hi() & 3;
        first = ty == 0 ? headF : (ty == 1 ? headB : (ty == 2 ? headW : ~0u));
    } else {
        first = c.nF() < c.hi() ? headF : umin(headB, umin(headF, headW));   // warm-up: forwards only
    }
    return is_empty(first) ? kInf : imax2(busy, (int)first);
}

// PHASE 0: generate with the policy and write the outputs; 1: generate under the plan scenario
// and record each stage's op types; 2: replay the recorded plans under every scenario.
template <int PHASE, bool NARROW>
__global__ __launch_bounds__(kZbBlock) void k_zb(ZbArgs a) {
    static_assert(!(PHASE == 2 && NARROW), "a replay keeps its window of coming ops in the wide form");
    typedef Cursors<NARROW> Cur;
    constexpr int kStage = Cur::kStage;
    const int S = a.S, N = a.N, Spad = (S + 7) & ~7;
    int *const act = zb_lds + threadIdx.x;                        // [Spad][64]
    int *const fld = zb_lds + Spad * 64 + threadIdx.x;            // [S][Cur::kFields][64]
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
        // word q of stage i of this lane's plan at packed_lane[(i * packed_words(N) + q) * 64]
        const uint32_t *const packed_lane = a.packed + (c / kZbBlock) * (long long)S * packed_words(N) * kZbBlock + c % kZbBlock;
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
            // x_i = w_i + 1 warm-up forwards; a replay starts with the first ops of its plan
            const Cur cur = Cur::start(PHASE == 2 ? (int)(packed_lane[(long long)i * packed_words(N) * kZbBlock] & 0xffff) : wi + 1);
            const unsigned headF = i == 0 ? 0u : empty_head(0), headB = empty_head(0);
            int *st = fld + i * kStage;
            cur.store(st);
            st[Cur::kHeadF] = (int)headF;
            st[Cur::kHeadB] = (int)headB;
            act[i * 64] = next_action<PHASE>(0, cur, headF, headB);
        }

        const int total = 3 * S * N;
        int makespan = 0;
        for (int step = 0; step < total; ++step) {
            if (PHASE == 2 && step % (kWindow - 1) == 0 && step > 0) {
                // A stage runs at most kWindow - 1 ops in as many steps, so its window never runs
                // out of a next op: re-reading every stage's window here, for all lanes at once,
                // keeps the plan's memory latency out of the steps in between.  The next op of a
                // stage does not change by this.
                for (int i = 0; i < S; ++i) {
                    int *const st = fld + i * kStage;
                    Cur cur = Cur::load(st);
                    const int done = cur.nF() + cur.nB() + cur.nW();
                    const uint32_t word = packed_lane[((long long)i * packed_words(N) + (done >> 3)) * kZbBlock];
                    cur.set_window(word >> ((done & 7) * 2));
                    cur.store(st);
                }
            }
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
            Cur cur = Cur::load(st);
            unsigned headF = (unsigned)st[Cur::kHeadF], headB = (unsigned)st[Cur::kHeadB];
            const int4 dur_i = *reinterpret_cast<const int4 *>(dur + i * 4);
            const int2 delay_i = *reinterpret_cast<const int2 *>(delay + i * 2);
            Cur prev, next;                                     // only their first word is needed
            prev.a = *(first ? st : st - kStage);
            next.a = *(last ? st : st + kStage);
            prev.b = next.b = 0;
            const int nF = cur.nF(), nB = cur.nB(), nW = cur.nW();
            int ty;
            if (PHASE == 2) ty = cur.hi() & 3;
            else ty = nF < cur.hi() ? 0 : (headB <= (unsigned)t ? 1 : (headF <= (unsigned)t ? 0 : 2));   // priority B > F > W among those ready at t
            // the stage this op posts to: F(i,m) -> F(i+1,m), B(i,m) -> B(i-1,m); its fields are
            // read before this stage's own are written (another stage, or unused)
            const int j = ty == 0 ? i + 1 : i - 1;
            const bool posts = ty < 2 && j >= 0 && j < S;
            int *const sj = posts ? (ty == 0 ? st + kStage : st - kStage) : st;
            const Cur cur_j = Cur::load(sj);
            unsigned headF_j = (unsigned)sj[Cur::kHeadF], headB_j = (unsigned)sj[Cur::kHeadB];

            const int m = ty == 0 ? nF : (ty == 1 ? nB : nW);
            const int done = nF + nB + nW;
            const int fin = t + (ty == 0 ? dur_i.x : (ty == 1 ? dur_i.y : dur_i.z));
            makespan = imax2(makespan, fin);
            if (PHASE == 1 && live) plan[(long long)i * 3 * N + done] = (uint8_t)ty;
            cur.started(ty);
            if (PHASE == 2) cur.advance_window();
            if (ty < 2) {
                // consume: the queue's next entry becomes the head.  Entries posted so far = ops of
                // that type the producing stage has started; stage 0's forwards and the last
                // stage's backwards come from no other stage and are ready whenever it is idle.
                const bool own = ty == 0 ? first : last;
                const int posted = ty == 0 ? (first ? N : prev.nF()) : (last ? cur.nF() : next.nB());
                unsigned head = ~0u;
                if (m + 1 < posted) head = own ? 0u : (unsigned)queue[(unsigned long long)(unsigned)((i * 2 + ty) * N + m + 1) * nt];
                if (ty == 0) headF = head; else headB = head;
            }
            if (is_empty(headF)) headF = empty_head(fin);       // busy until fin from now on
            if (is_empty(headB)) headB = empty_head(fin);
            if (last && ty == 0) headB = 0;                     // its own forward makes a backward available
            cur.store(st);
            st[Cur::kHeadF] = (int)headF;
            st[Cur::kHeadB] = (int)headB;
            act[i * 64] = next_action<PHASE>(fin, cur, headF, headB);
            if (posts) {
                const int r = fin + (ty == 0 ? delay_i.x : delay_i.y);
                const unsigned slot = ty == 0 ? headF_j : headB_j;
                if (is_empty(slot)) {                           // r becomes the head: the receiver may act earlier
                    if (ty == 0) headF_j = (unsigned)r; else headB_j = (unsigned)r;
                    sj[ty == 0 ? Cur::kHeadF : Cur::kHeadB] = r;
                    act[j * 64] = next_action<PHASE>((int)~slot, cur_j, headF_j, headB_j);
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

// Plans from one byte per op, [C][S][3N], to 2 bits per op, 16 ops per word from op 8 q on, kNone
// behind the end of a stage's ops, laid out [chunk of 64 candidates][S][word][candidate].
__global__ void k_zb_pack(const uint8_t *plans, uint32_t *packed, long long C, int S, int N) {
    const int words = packed_words(N);
    const long long chunks = (C + kZbBlock - 1) / kZbBlock;
    const long long n = chunks * S * words * kZbBlock, stride = (long long)gridDim.x * blockDim.x;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += stride) {
        const int lane = (int)(idx % kZbBlock);
        const int q = (int)(idx / kZbBlock % words);
        const int i = (int)(idx / kZbBlock / words % S);
        const long long c = idx / kZbBlock / words / S * kZbBlock + lane;
        uint32_t v = 0;
        for (int j = 0; j < 16; ++j) {
            const int op = q * 8 + j;
            v |= (uint32_t)(c < C && op < 3 * N ? plans[(c * S + i) * 3 * N + op] : kNone) << (2 * j);
        }
        packed[idx] = v;
    }
}


extern "C" int zb_cpu(int S, int N, long long C, long long K, const int *tf, const int *tb, const int *tw,
                      const int *w, const int *cf, const int *cb, long long plan_scenario,
                      int *out_mk, int *out_bub, unsigned threads, int narrow) {
    ZbArgs a{}; a.S=S; a.N=N; a.t_f=tf; a.t_b=tb; a.t_w=tw; a.C=C; a.K=K; a.w=w; a.cf=cf; a.cb=cb;
    a.plan_scenario=plan_scenario; a.out_makespan=out_mk; a.out_bubble=out_bub;
    const int Spad=(S+7)&~7;
    auto lds_ints_for=[&](int stage){ return (size_t)Spad*64+(size_t)S*stage+6*(size_t)S; };
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
            zb_lds=(int*)malloc(lds_ints_for((narrow && phase!=2) ? Cursors<true>::kStage : Cursors<false>::kStage)*4);
            blockIdx.x=b;
            std::vector<std::thread> th;
            for(unsigned t=0;t<64;++t) th.emplace_back([&,t]{ threadIdx.x=t; if(phase==0){ if(narrow) k_zb<0,true>(a); else k_zb<0,false>(a);} else if(phase==1){ if(narrow) k_zb<1,true>(a); else k_zb<1,false>(a);} else k_zb<2,false>(a); });
            for(auto&x:th) x.join();
            free(zb_lds);
        }
        free(a.scratch);
    };
    if (plan_scenario<0) run(0,K); else { run(1,1); uint32_t *pk=(uint32_t*)malloc((size_t)((C+63)/64)*64*S*packed_words(N)*4); blockIdx.x=0; gridDim.x=1; blockDim.x=1; threadIdx.x=0; k_zb_pack(a.plans,pk,C,S,N); a.packed=pk; run(2,K); free(pk); }
    free(a.plans);
    return 0;
}

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
// offsets), and per stage a block of four fields [stage][field][lane] at fixed offsets from the
// stage's base (conflict-free for any per-lane stage index): the cursors (nF and nB share a
// word, nW shares one with the warm-up quota x) and the HEAD of each queue (the ready time of
// the cursor's micro-batch; an empty queue's slot keeps the stage's busy-until time instead).
// A post that lands on an empty queue goes straight to the head in LDS and never to memory, and
// only then can it change the receiver's next action; a step touches global memory only to
// append behind a head and to fetch the next head after a consume.  One wavefront per block
// works on 64 candidates of ONE scenario at a time, so the link delays are a small table shared
// by its lanes.  LDS per wavefront: (4 S + 8 ceil(S/8)) x 256 bytes -- the occupancy limit of
// this kernel, whose step is a chain of dependent LDS round trips that only more resident
// wavefronts can hide.
//
// Fixed plans (generated once per candidate under one scenario, then run under all of them) need
// none of this when replayed: k_zb_replay_folded and k_zb_replay_scen put the scenarios on the
// lanes and run a recorded order.  Their recording is a launch of few pairs, for which
// k_zb_record_stages spreads a candidate's stages over neighbouring lanes instead (k_zb<1, ., .>
// where that launch would not fit the chip at once).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"

namespace {

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
    uint8_t *plans;               // [C][S][3N], op types in the order a stage ran them (written by PHASE 1), or null
    const uint32_t *packed;       // [ceil(C/64)][S][packed_words(N)][64 candidates], the same at 2 bits per op (see
                                  // packed_words), read by PHASE 2: the lanes of a wavefront read neighbouring words
    uint16_t *order;              // [C][order_stride] or null: stage | type << 6 | slot << 8 of every op in the order
                                  // PHASE 1 started them -- a topological order of the plan's dependency graph; slot
                                  // = micro-batch, N for a weight op (k_zb_replay_scen; N <= 255)
    uint4 *order_folded;          // [C][order_stride] or null: the same order without the weight ops, written by
                                  // k_zb_record_stages for k_zb_replay_folded, every field ready for use: .x = 256 stage
                                  // | 256 (type S + stage) << 16 of a forward or backward op, .y = the time the stage
                                  // spent on weight ops since its last forward or backward op (they run back to back
                                  // from the moment it is free), .z = the op's duration, .w = 256 micro-batch
    int *tail_w;                  // [C][S]: the time of a stage's weight ops behind its last backward op
    uint8_t *plan_ok;             // [C]: the recording ran to its end
    long long order_stride;       // entries per candidate, a multiple of 16
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
constexpr long long kScenReplayFrom = 8;   // scenarios from which a replay puts them on the lanes
constexpr int kXcds = 8;              // accelerator dies of an MI355X; workgroup b is dispatched to die b mod 8
constexpr int kCus = 256;             // compute units of an MI355X

// Next action of a stage from its own fields (Algorithm 3): the time it can act, or 2^31 or more if
// nothing it may run has been posted yet.
template <int PHASE, bool NARROW>
__device__ __forceinline__ unsigned next_action(int busy, const Cursors<NARROW> &c, unsigned headF, unsigned headB) {
    const unsigned headW = c.nW() < c.nB() ? 0u : ~0u;           // ready since its backward finished
    unsigned first;
    if (PHASE == 2) {
        const int ty = c.hi() & 3;
        first = ty == 0 ? headF : (ty == 1 ? headB : (ty == 2 ? headW : ~0u));
    } else {
        first = c.nF() < c.hi() ? headF : umin(headB, umin(headF, headW));   // warm-up: forwards only
    }
    return first > (unsigned)busy ? first : (unsigned)busy;      // "nothing posted" stays at or above 2^31: behind every time
}

// PHASE 0: generate with the policy and write the outputs; 1: generate under the plan scenario
// and record each stage's op types; 2: replay the recorded plans under every scenario.
// QLDS: the two queues per stage in LDS behind the other state instead of in global scratch --
// for a launch whose wavefronts are so few (the recording of fixed plans: one scenario) that each
// has a CU's LDS to itself and nothing hides the latency of its queue accesses to memory.
template <int PHASE, bool NARROW, bool QLDS = false>
__global__ __launch_bounds__(kZbBlock) void k_zb(ZbArgs a) {
    static_assert(!(PHASE == 2 && NARROW), "a replay keeps its window of coming ops in the wide form");
    typedef Cursors<NARROW> Cur;
    constexpr int kStage = Cur::kStage;
    extern __shared__ int zb_lds[];
    const int S = a.S, N = a.N, Spad = (S + 7) & ~7;
    int *const act = zb_lds + threadIdx.x;                        // [Spad][64]
    int *const fld = zb_lds + Spad * 64 + threadIdx.x;            // [S][Cur::kFields][64]
    int *const dur = zb_lds + Spad * 64 + S * kStage;             // [S][4]: t_f, t_b, t_w, 0
    int *const delay = dur + 4 * S;                               // [S][2]: forward delay of link i -> i+1, backward delay of link i-1 <- i
    for (int i = threadIdx.x; i < 4 * S; i += kZbBlock) {
        const int s = i >> 2, ty = i & 3;
        dur[i] = ty == 0 ? a.t_f[s] : (ty == 1 ? a.t_b[s] : (ty == 2 ? a.t_w[s] : 0));
    }
    // queue entry e of this lane at queue[e * nt].  Entry numbers stay below 2 S N <= 2^22 and nt
    // below 2^20, their product below the 2^29 ints of the queue memory (threads_for): both
    // products of the address are 24-bit multiplies (full rate; a 32 x 32 -> 64-bit one runs at a
    // quarter of it, and two of those per queue access were a fifth of a step's vector cycles)
    int *const queue = QLDS ? delay + 2 * S + threadIdx.x : a.scratch + ((long long)blockIdx.x * kZbBlock + threadIdx.x);
    const unsigned nt = QLDS ? (unsigned)kZbBlock : a.threads;
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
        for (int i = S; i < Spad; ++i) act[i * 64] = -1;            // read as unsigned: behind every time
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
            act[i * 64] = (int)next_action<PHASE>(0, cur, headF, headB);
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
            int i = 0;
            unsigned t_min = ~0u;
            for (int b = 0; b < Spad; b += 8) {
                unsigned tb = (unsigned)act[b * 64];
                int jb = 0;
#pragma unroll
                for (int j = 1; j < 8; ++j) {
                    const unsigned tj = (unsigned)act[(b + j) * 64];
                    if (tj < tb) { tb = tj; jb = j; }
                }
                if (tb < t_min) { t_min = tb; i = b + jb; }
            }
            if ((int)t_min < 0) { makespan = kInf; break; }     // nothing can act: cannot happen for valid input
            const int t = (int)t_min;
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
            if (PHASE == 1 && live) {
                plan[(long long)i * 3 * N + done] = (uint8_t)ty;
                if (a.order) a.order[c * a.order_stride + step] = (uint16_t)(i | ty << 6 | (ty == 2 ? N : m) << 8);
            }
            cur.started(ty);
            if (PHASE == 2) cur.advance_window();
            if (ty < 2) {
                // consume: the queue's next entry becomes the head.  Entries posted so far = ops of
                // that type the producing stage has started; stage 0's forwards and the last
                // stage's backwards come from no other stage and are ready whenever it is idle.
                const bool own = ty == 0 ? first : last;
                const int posted = ty == 0 ? (first ? N : prev.nF()) : (last ? cur.nF() : next.nB());
                unsigned head = ~0u;
                if (m + 1 < posted) head = own ? 0u : (unsigned)queue[__umul24(__umul24((unsigned)(i * 2 + ty), (unsigned)N) + (unsigned)(m + 1), nt)];
                if (ty == 0) headF = head; else headB = head;
            }
            if (is_empty(headF)) headF = empty_head(fin);       // busy until fin from now on
            if (is_empty(headB)) headB = empty_head(fin);
            if (last && ty == 0) headB = 0;                     // its own forward makes a backward available
            cur.store(st);
            st[Cur::kHeadF] = (int)headF;
            st[Cur::kHeadB] = (int)headB;
            act[i * 64] = (int)next_action<PHASE>(fin, cur, headF, headB);
            if (posts) {
                const int r = fin + (ty == 0 ? delay_i.x : delay_i.y);
                const unsigned slot = ty == 0 ? headF_j : headB_j;
                if (is_empty(slot)) {                           // r becomes the head: the receiver may act earlier
                    if (ty == 0) headF_j = (unsigned)r; else headB_j = (unsigned)r;
                    sj[ty == 0 ? Cur::kHeadF : Cur::kHeadB] = r;
                    act[j * 64] = (int)next_action<PHASE>((int)~slot, cur_j, headF_j, headB_j);
                } else {
                    queue[__umul24(__umul24((unsigned)(j * 2 + ty), (unsigned)N) + (unsigned)m, nt)] = r;
                }
            }
        }
        if (PHASE == 1 && live && a.order) a.plan_ok[c] = makespan != kInf;
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

// Recording with the STAGES on the lanes: G lanes (8 or 16, a power of two >= S) per candidate,
// 64 / G candidates per wavefront.  The recording runs every candidate under ONE scenario, so
// with a lane per pair it is a few lone wavefronts whose 3 S N steps nothing overlaps.  With a
// lane per (candidate, stage) a stage's whole state -- cursors, the heads of its two queues,
// its busy-until time, its durations and delays -- is in that lane's registers under static
// names, the earliest next action of a candidate is a minimum over G neighbouring lanes (DPP),
// a post goes to the neighbouring lane by a DPP shift, and only the queues behind the heads
// are in LDS ([micro-batch][lane]).  And the stages of a candidate advance TOGETHER: if t is
// the candidate's earliest next action, nothing that has not been posted yet can become ready
// before t + L, L = the least (duration + link delay) of any op that posts, because the op that
// will post it starts at t or later.  So every stage whose next action lies before t + L takes
// it in the same step -- its decision (Algorithm 3) can no longer be overturned -- and the ops
// of one step do not depend on each other (what one of them posts is ready at t + L at the
// earliest).  Same policy and same schedules as k_zb<1, ., .>, in about a fifth of the steps on
// 1F1B-like warm-ups; the order written for k_zb_replay_scen is topological as before (ops of
// one step in stage order).
template <int kCtrl>
__device__ __forceinline__ unsigned zb_dpp(unsigned keep, unsigned v) {
    return (unsigned)__builtin_amdgcn_update_dpp((int)keep, (int)v, kCtrl, 0xf, 0xf, false);
}
template <int G>
__device__ __forceinline__ unsigned zb_group_umin(unsigned v) {
    v = umin(v, zb_dpp<0xB1>(~0u, v));                            // quad_perm [1,0,3,2]: lane ^ 1
    v = umin(v, zb_dpp<0x4E>(~0u, v));                            // quad_perm [2,3,0,1]: lane ^ 2
    v = umin(v, zb_dpp<0x141>(~0u, v));                           // row_half_mirror: the two quads of 8 lanes
    if (G >= 16) v = umin(v, zb_dpp<0x140>(~0u, v));              // row_mirror: the two halves of a row
    if (G >= 32) v = umin(v, (unsigned)__builtin_amdgcn_ds_swizzle((int)v, 0x401F));                           // lane ^ 16
    if (G == 64) v = umin(v, (unsigned)__builtin_amdgcn_ds_bpermute((int)((threadIdx.x ^ 32) << 2), (int)v));  // lane ^ 32
    return v;
}
// v of the lane before / after this one (another row of 16 lanes from 32-lane groups on: through
// the LDS crossbar); `none` where a DPP row ends -- the caller drops what crosses a group's end anyway
template <int G>
__device__ __forceinline__ unsigned zb_from_previous_lane(unsigned v, unsigned none) {
    if (G <= 16) return zb_dpp<0x111>(none, v);                   // row_shr:1
    return (unsigned)__builtin_amdgcn_ds_bpermute((int)(((threadIdx.x - 1) & 63) << 2), (int)v);
}
template <int G>
__device__ __forceinline__ unsigned zb_from_next_lane(unsigned v, unsigned none) {
    if (G <= 16) return zb_dpp<0x101>(none, v);                   // row_shl:1
    return (unsigned)__builtin_amdgcn_ds_bpermute((int)(((threadIdx.x + 1) & 63) << 2), (int)v);
}
// the bits of a wavefront-wide vote that belong to this lane's group of G lanes, lowest stage first
template <int G>
__device__ __forceinline__ unsigned long long zb_group_bits(unsigned long long vote) {
    if (G == 64) return vote;
    const unsigned half = (unsigned)(threadIdx.x < 32 ? vote : vote >> 32);
    return (half >> (threadIdx.x & ~(G - 1) & 31)) & (G == 32 ? ~0u : (1u << (G & 31)) - 1);
}

template <int G, bool FOLDED>
__global__ __launch_bounds__(kZbBlock) void k_zb_record_stages(ZbArgs a) {
    static_assert(G == 8 || G == 16 || G == 32 || G == 64, "a group of lanes is half a DPP row, a row, two or all four");
    extern __shared__ int zb_lds[];
    constexpr unsigned kNever = ~0u;                              // as a ready time: nothing of that type is available
    const int S = a.S, N = a.N, lane = threadIdx.x;
    const int i = lane % G;                                       // this lane's stage (none if i >= S)
    const long long c_lane = (long long)blockIdx.x * (kZbBlock / G) + lane / G;
    const bool exists = c_lane < a.C && i < S;
    const long long c = c_lane < a.C ? c_lane : a.C - 1;
    const int is = i < S ? i : S - 1;
    const bool first = i == 0, last = i == S - 1, posts_f = i < S - 1, posts_b = i > 0 && i < S;
    const long long k = a.plan_scenario;
    const int t_f = a.t_f[is], t_b = a.t_b[is], t_w = a.t_w[is];
    const int delay_f = posts_f ? a.cf[(long long)is * a.K + k] : 0;         // link i -> i + 1
    const int delay_b = posts_b ? a.cb[(long long)(is - 1) * a.K + k] : 0;   // link i - 1 <- i
    int wi = a.w[(long long)is * a.C + c];
    wi = wi < 0 ? 0 : (wi > N - 1 ? N - 1 : wi);
    const int x = wi + 1;                                         // warm-up quota
    // look-ahead of the candidate; any smaller value is valid too, and 2^30 keeps t + L in 32 bits
    const unsigned own_f = posts_f ? (unsigned)t_f + (unsigned)delay_f : kNever;
    const unsigned own_b = posts_b ? (unsigned)t_b + (unsigned)delay_b : kNever;
    const unsigned look = umin(zb_group_umin<G>(umin(own_f, own_b)), 1u << 30);
    int *const qF = zb_lds + lane;                                // [N][64]: ready time of forward m of this stage
    int *const qB = qF + N * 64;                                  // [N][64]: of backward m
    uint8_t *const plan = a.plans + (c * S + is) * 3ll * N;       // this stage's op types
    // Ops started per type; ready times received so far; the ready time of the next forward and
    // backward, kNever while none is available.  Stage 0's forwards are all ready at time 0; the
    // last stage's backwards follow its own forwards (ready while it is still busy with them).
    int nF = 0, nB = 0, nW = 0, recvF = 0, recvB = 0, busy = 0;
    unsigned headF = first && i < S ? 0u : kNever, headB = kNever;
    auto next_key = [&]() {
        const unsigned headW = nW < nB ? 0u : kNever;             // ready since its backward finished
        const unsigned soonest = nF < x ? headF : umin(headB, umin(headF, headW));   // warm-up: forwards only
        return soonest > (unsigned)busy ? soonest : (unsigned)busy;                  // kNever stays kNever
    };
    unsigned key = next_key();
    int recorded = 0;                                             // ops of this candidate written to the order so far (FOLDED: forward and backward ops)
    int weight_time = 0;                                          // spent on weight ops since this stage's last forward or backward op
    const int total = 3 * S * N;
    const unsigned long long below_me = (1ull << i) - 1;
    for (int step = 0; step < total; ++step) {
        const unsigned t = zb_group_umin<G>(key);                 // the candidate's earliest next action
        if (__ballot(t != kNever) == 0) break;                    // every candidate of the wavefront is through (or stuck)
        const bool act = key != kNever && key - t < look;         // final: nothing unposted is ready before t + look
        const int ty = nF < x ? 0 : (headB <= key ? 1 : (headF <= key ? 0 : 2));     // B > F > W among those ready
        const int m = ty == 0 ? nF : (ty == 1 ? nB : nW);
        const int fin = (int)key + (ty == 0 ? t_f : (ty == 1 ? t_b : t_w));
        // Position in the order: the candidate's ops of this step in stage order.  In the FOLDED
        // order weight ops get no entry: a weight op starts the moment its stage is free (its
        // backward op ran on the same stage before), so all a replay has to know is how long the
        // stage spent on them before its next forward or backward op.
        const unsigned long long in_group = zb_group_bits<G>(__ballot(act && (!FOLDED || ty < 2)));
        if (act) {
            if (exists) {
                if (a.plans) plan[nF + nB + nW] = (uint8_t)ty;
                const long long at = c * a.order_stride + recorded + __popcll(in_group & below_me);
                if (FOLDED) {
                    if (a.order_folded && ty < 2)
                        a.order_folded[at] = make_uint4((unsigned)(i << 8 | (ty * S + i) << 24), (unsigned)weight_time,
                                                        (unsigned)(ty == 0 ? t_f : t_b), (unsigned)(m << 8));
                } else if (a.order) {
                    a.order[at] = (uint16_t)(i | ty << 6 | (ty == 2 ? N : m) << 8);
                }
            }
            weight_time = ty == 2 ? weight_time + t_w : 0;
            busy = fin;
            nF += ty == 0; nB += ty == 1; nW += ty == 2;
            // the op's own queue moves on to its next entry, if that has been posted
            if (ty == 0) headF = first ? (nF < N ? 0u : kNever) : (nF < recvF ? (unsigned)qF[nF * 64] : kNever);
            if (ty == 1 && !last) headB = nB < recvB ? (unsigned)qB[nB * 64] : kNever;
            if (last) headB = nB < nF ? 0u : kNever;
        }
        recorded += __popcll(in_group);
        // what the op makes available next door: F(i,m) -> F(i+1,m), B(i,m) -> B(i-1,m)
        const unsigned post_f = act && ty == 0 ? (unsigned)(fin + delay_f) : kNever;
        const unsigned post_b = act && ty == 1 ? (unsigned)(fin + delay_b) : kNever;
        unsigned got_f = zb_from_previous_lane<G>(post_f, kNever);   // from the lane of stage i - 1
        unsigned got_b = zb_from_next_lane<G>(post_b, kNever);       // from the lane of stage i + 1
        if (first || i >= S) got_f = kNever;                      // that lane belongs to another candidate
        if (i >= S - 1) got_b = kNever;
        if (got_f != kNever) {
            qF[recvF * 64] = (int)got_f;
            if (headF == kNever) headF = got_f;                   // the queue was empty: nF == recvF
            ++recvF;
        }
        if (got_b != kNever) {
            qB[recvB * 64] = (int)got_b;
            if (headB == kNever) headB = got_b;
            ++recvB;
        }
        key = next_key();
    }
    if (FOLDED ? a.order_folded != nullptr : a.order != nullptr) {
        const unsigned long long unfinished = zb_group_bits<G>(__ballot(i < S && !(nF == N && nB == N && nW == N)));
        if (FOLDED && exists) a.tail_w[c * S + i] = weight_time;
        if (first && c_lane < a.C) a.plan_ok[c] = unfinished == 0;
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

// Fixed plans with the SCENARIOS on the lanes: one wavefront = one candidate's plan under 64
// scenarios.  A fixed plan needs no decisions: its times are the longest paths of the dependency
// graph of Section 3.1 (each stage's ops in the plan's order, F(i,m) after F(i-1,m) + delay,
// B(i,m) after B(i+1,m) + delay), so the ops can be taken in ANY topological order -- here the
// order in which the generating launch started them (an op starts after everything it depends on
// has started, forward and backward ops lasting at least 1 us).  That order, with stage, type
// and micro-batch of every op, is the same for all 64 lanes, i.e. scalar, and was written down
// by the generating launch (ZbArgs::order); a lane keeps only times, in LDS [index][lane]: the
// busy-until time of each stage and one ready time per micro-batch (written by the stage that
// ran the micro-batch last, read by the next stage of its chain: the forward chain up to the
// last stage, then the backward chain down again).  Every op is the same five steps,
//     fin = max(busy[i], ready[slot]) + duration;  busy[i] = fin;  ready[slot] = fin + delay,
// without a case distinction: a forward of stage 0 finds 0 in its slot, a backward of the last
// stage its own forward's finish (not later than the stage is busy), and a weight op uses a slot
// of its own with a "delay" of -2^31, so that what it leaves there never exceeds a busy time.
// Per op: four LDS reads in one round trip (the duration is a broadcast read), one max, two
// adds, two LDS writes, and the scalar decoding of the entry.
struct ZbReplayRows {
    int *busy, *ready, *delay;        // this lane's column of [S], [N + 1], [3][S] rows of 64 lanes
    const int *dur;                   // [3][S] ints
    int S;
};
__device__ __forceinline__ int zb_replay_op(const ZbReplayRows &t, unsigned entry, int makespan) {
    const int i = entry & 63, row = (int)((entry >> 6) & 3) * t.S + i, slot = (int)(entry >> 8);
    const int b = t.busy[i * 64], r = t.ready[slot * 64], d = t.delay[row * 64], length = t.dur[row];
    const int fin = imax2(b, r) + length;
    t.busy[i * 64] = fin;
    t.ready[slot * 64] = fin + d;
    return imax2(makespan, fin);
}

__global__ __launch_bounds__(kZbBlock) void k_zb_replay_scen(ZbArgs a) {
    extern __shared__ int zb_lds[];
    const int S = a.S, N = a.N, lane = threadIdx.x;
    ZbReplayRows t;
    t.S = S;
    t.busy = zb_lds + lane;                           // [S][64]
    t.ready = t.busy + S * 64;                        // [N + 1][64]; slot N is the weight ops'
    t.delay = t.ready + (N + 1) * 64;                 // [3][S][64]: link i -> i+1, link i-1 <- i, -2^31
    int *const dur = zb_lds + (4 * S + N + 1) * 64;   // [3][S]: t_f, t_b, t_w
    t.dur = dur;
    // Block -> (candidate, tile of 64 scenarios).  A lane's results lie C ints apart, so the 4-byte
    // stores of one wavefront share no cache line; those of NEIGHBOURING candidates do (16 per 64
    // bytes).  Workgroups go round the 8 XCDs by their index, each XCD with an L2 of its own, so
    // each XCD takes one contiguous eighth of the candidates: the wavefronts that fill a line then
    // run next to each other on the same L2, which merges their stores before the line goes to
    // memory (with candidate = block index the same stores reached HBM as 11 times the bytes).
    const long long n_tiles = (a.K + kZbBlock - 1) / kZbBlock;
    const long long per_xcd = (a.C + kXcds - 1) / kXcds;
    const long long in_xcd = blockIdx.x / kXcds;
    const long long c = (blockIdx.x % kXcds) * per_xcd + in_xcd / n_tiles;
    if (in_xcd / n_tiles >= per_xcd || c >= a.C) return;          // the last eighth may be short
    const long long k_lane = (in_xcd % n_tiles) * kZbBlock + lane;
    const bool live = k_lane < a.K;
    const long long k = live ? k_lane : a.K - 1;
    for (int i = lane; i < 3 * S; i += kZbBlock) dur[i] = i < S ? a.t_f[i] : (i < 2 * S ? a.t_b[i - S] : a.t_w[i - 2 * S]);
    for (int i = 0; i < S; ++i) {
        t.busy[i * 64] = 0;
        t.delay[i * 64] = i < S - 1 ? a.cf[(long long)i * a.K + k] : 0;
        t.delay[(S + i) * 64] = i > 0 ? a.cb[(long long)(i - 1) * a.K + k] : 0;
        t.delay[(2 * S + i) * 64] = INT32_MIN;       // finish (>= 0) + this is negative, and does not wrap
    }
    for (int m = 0; m <= N; ++m) t.ready[m * 64] = 0;
    __syncthreads();                                  // the durations (one wavefront: no more than a wait)
    const uint16_t *const order = a.order + c * a.order_stride;
    const int total = 3 * S * N;
    int makespan = 0;
    // 16 entries per (scalar) load, the next 16 fetched while these run
    const uint4 *const order16 = reinterpret_cast<const uint4 *>(order);
    const bool recorded = a.plan_ok[c] != 0;          // else the entries are not a plan: nothing is run
    uint4 lo = order16[0], hi = order16[1];
    int base = recorded ? 0 : total;
    for (; base + 16 <= total; base += 16) {
        const unsigned word[8] = {(unsigned)__builtin_amdgcn_readfirstlane((int)lo.x), (unsigned)__builtin_amdgcn_readfirstlane((int)lo.y),
                                  (unsigned)__builtin_amdgcn_readfirstlane((int)lo.z), (unsigned)__builtin_amdgcn_readfirstlane((int)lo.w),
                                  (unsigned)__builtin_amdgcn_readfirstlane((int)hi.x), (unsigned)__builtin_amdgcn_readfirstlane((int)hi.y),
                                  (unsigned)__builtin_amdgcn_readfirstlane((int)hi.z), (unsigned)__builtin_amdgcn_readfirstlane((int)hi.w)};
        if (base + 16 < total) {                      // inside the candidate's padded row
            lo = order16[base / 8 + 2];
            hi = order16[base / 8 + 3];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) makespan = zb_replay_op(t, (word[j >> 1] >> ((j & 1) * 16)) & 0xffffu, makespan);
    }
    for (; base < total; ++base)
        makespan = zb_replay_op(t, (unsigned)__builtin_amdgcn_readfirstlane((int)order[base]), makespan);
    if (!recorded) makespan = kInf;                   // the recording stopped: so does every replay of it
    if (live) {
        const long long P = a.C * a.K, item = k * a.C + c;
        a.out_makespan[item] = makespan;
        if (a.out_bubble)
            for (int i = 0; i < S; ++i)
                a.out_bubble[(long long)i * P + item] = makespan == kInf ? kInf : makespan - N * (dur[i] + dur[S + i] + dur[2 * S + i]);
    }
}

// The same replay on an order without weight ops (ZbArgs::order_folded).  W(i,m) depends on
// B(i,m) alone, which ran on the same stage before it, so a weight op starts the moment its stage
// is free and only pushes the stage's busy-until time; the recording has added up what a stage
// spends on weight ops between two of its other ops (the same in every scenario), and the op after
// them is  fin = max(busy[i] + weight time, ready[m]) + duration.  A third fewer ops, no slot and
// no delay row for weight ops; the makespan is the latest busy-until time, the weight ops behind
// a stage's last backward op (ZbArgs::tail_w) included.
// REGS = 16 or 32 (at most that many stages): a lane's busy-until times and link delays are in
// registers, arrays that the compiler indexes with the op's (uniform) stage or row number
// (s_set_gpr_idx), and LDS holds only the N ready times -- no round trip for them, and two to
// four times the wavefronts per CU.  The compiler keeps such an array in registers if it has at
// most 32 elements and every access under a run-time index is a plain load or store of its own
// (they are set below under static indices; a conditional between two of them is written as two
// loads and a select): at 16 stages both directions' delays share one array under the row
// number, at 32 each direction has its own.  REGS = 0 (up to 64 stages): all rows in LDS.
template <int REGS>
__global__ __launch_bounds__(kZbBlock) void k_zb_replay_folded(ZbArgs a) {
    static_assert(REGS == 0 || REGS == 16 || REGS == 32, "register arrays of 16 or 32 stages, or none");
    constexpr int kRegs = REGS ? REGS : 1, kBack = REGS == 32 ? 32 : 1, kDelays = REGS ? 32 : 1;
    extern __shared__ int zb_lds[];
    const int S = a.S, N = a.N, lane = threadIdx.x;
    int *const ready = zb_lds + lane;                 // [N][64]
    int *const busy = ready + N * 64;                 // REGS = 0: [S][64]
    int *const delay = busy + S * 64;                 // REGS = 0: [2][S][64]: link i -> i+1, link i-1 <- i
    int *const dur = zb_lds + ((REGS ? 0 : 3 * S) + N) * 64;   // [3][S]: t_f, t_b, t_w
    int busy_r[kRegs];
    int delay_r[kDelays];                             // REGS = 16: link i -> i+1 at i, link i-1 <- i at S + i; 32: link i -> i+1 at i
    int back_r[kBack];                                // REGS = 32: link i-1 <- i at i
    // block -> (candidate, tile of 64 scenarios) as in k_zb_replay_scen
    const long long n_tiles = (a.K + kZbBlock - 1) / kZbBlock;
    const long long per_xcd = (a.C + kXcds - 1) / kXcds;
    const long long in_xcd = blockIdx.x / kXcds;
    const long long c = (blockIdx.x % kXcds) * per_xcd + in_xcd / n_tiles;
    if (in_xcd / n_tiles >= per_xcd || c >= a.C) return;
    const long long k_lane = (in_xcd % n_tiles) * kZbBlock + lane;
    const bool live = k_lane < a.K;
    const long long k = live ? k_lane : a.K - 1;
    for (int i = lane; i < 3 * S; i += kZbBlock) dur[i] = i < S ? a.t_f[i] : (i < 2 * S ? a.t_b[i - S] : a.t_w[i - 2 * S]);
    if (REGS) {
#pragma unroll
        for (int i = 0; i < kRegs; ++i) busy_r[i] = 0;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int forward = j < S - 1 ? a.cf[(long long)j * a.K + k] : 0;
            if (REGS == 16) {
                delay_r[j % kDelays] = j > S && j < 2 * S ? a.cb[(long long)(j - S - 1) * a.K + k] : forward;
            } else {
                delay_r[j % kDelays] = forward;
                back_r[j % kBack] = j > 0 && j < S ? a.cb[(long long)(j - 1) * a.K + k] : 0;
            }
        }
    } else {
        for (int i = 0; i < S; ++i) {
            busy[i * 64] = 0;
            delay[i * 64] = i < S - 1 ? a.cf[(long long)i * a.K + k] : 0;
            delay[(S + i) * 64] = i > 0 ? a.cb[(long long)(i - 1) * a.K + k] : 0;
        }
    }
    for (int m = 0; m < N; ++m) ready[m * 64] = 0;
    __syncthreads();
    // Everything uniform comes out of the entry ready for use: the byte offsets of the LDS rows
    // ([index][lane] ints: 256 bytes a row), stage and row number, and the two times, which are
    // scalar operands of the adds.
    auto at = [](int *rows, unsigned bytes) { return reinterpret_cast<int *>(reinterpret_cast<char *>(rows) + bytes); };
    auto run = [&](unsigned offsets, unsigned weight_time, unsigned length, unsigned m256) {
        const int i = (int)((offsets >> 8) & 0xffu), row = (int)(offsets >> 24);
        int *const ready_m = at(ready, m256), *const busy_i = at(busy, offsets & 0xffffu);
        int d, b;
        if (REGS == 16) {
            d = delay_r[row % kDelays];
        } else if (REGS == 32) {
            const int forward = delay_r[i % kDelays], backward = back_r[i % kBack];
            d = row < S ? forward : backward;
        } else {
            d = *at(delay, offsets >> 16);
        }
        b = REGS ? busy_r[i % kRegs] : *busy_i;
        const int fin = imax2(b + (int)weight_time, *ready_m) + (int)length;
        if (REGS) busy_r[i % kRegs] = fin; else *busy_i = fin;
        *ready_m = fin + d;
    };
    // Lane j of the wavefront holds entry base + j of the order (one 16-byte load per lane and 64
    // ops, the next 64 entries fetched while these run); an op takes its entry's four words from
    // that lane into scalar registers.  (Scalar loads would deliver them there directly, but they
    // share the counter the LDS accesses wait on, so every wait of an op would also sit out the
    // memory latency of the entries fetched ahead: 0.39 against 0.29 ms on 2^20 pairs.)
    auto run_lane = [&](const uint4 &e, int j) {
        run((unsigned)__builtin_amdgcn_readlane((int)e.x, j), (unsigned)__builtin_amdgcn_readlane((int)e.y, j),
            (unsigned)__builtin_amdgcn_readlane((int)e.z, j), (unsigned)__builtin_amdgcn_readlane((int)e.w, j));
    };
    const uint4 *const order = a.order_folded + c * a.order_stride + lane;
    const int total = 2 * S * N;
    const bool recorded = __builtin_amdgcn_readfirstlane((int)a.plan_ok[c]) != 0;   // else the entries are not a plan: nothing is run
    int base = recorded ? 0 : total;
    uint4 cur = order[0];
    for (; base + 64 <= total; base += 64) {
        const uint4 next = order[base + 64];          // still inside the candidate's padded row
#pragma unroll
        for (int j = 0; j < 64; ++j) run_lane(cur, j);
        cur = next;
    }
    for (int j = 0; base + j < total; ++j) run_lane(cur, j);
    int makespan = 0;
    if (REGS) {
#pragma unroll
        for (int i = 0; i < kRegs; ++i)
            if (i < S) makespan = imax2(makespan, busy_r[i] + a.tail_w[c * S + i]);
    } else {
        for (int i = 0; i < S; ++i) makespan = imax2(makespan, busy[i * 64] + a.tail_w[c * S + i]);
    }
    if (!recorded) makespan = kInf;                   // the recording stopped: so does every replay of it
    if (live) {
        const long long P = a.C * a.K, item = k * a.C + c;
        a.out_makespan[item] = makespan;
        if (a.out_bubble)
            for (int i = 0; i < S; ++i)
                a.out_bubble[(long long)i * P + item] = makespan == kInf ? kInf : makespan - N * (dur[i] + dur[S + i] + dur[2 * S + i]);
    }
}

__global__ void k_zb_reset(unsigned long long *counters) {
    if (threadIdx.x < 2) counters[threadIdx.x] = 0;
}

// Range scan for adaptra_zb_check_inputs.  found[0] counts entries out of range: a forward or
// backward time below 1 (two dependent ops would share an instant, which the evaluation order
// of k_zb excludes), a negative weight time, delay or w; found[1] / found[2] = largest time /
// delay.  found[] is zero when the kernel starts.
__global__ __launch_bounds__(adaptra_detail::kThreadsPerBlock) void k_zb_check(ZbArgs a, int *found) {
    const long long nw = (long long)a.S * a.C, nc = (long long)(a.S - 1) * a.K;
    const long long n = nw + 2 * nc + 3 * a.S;
    const long long stride = (long long)gridDim.x * blockDim.x;
    int bad = 0, maxt = 0, maxc = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (i < nw) {
            bad += a.w[i] < 0;
        } else if (i < nw + 2 * nc) {
            const int v = i < nw + nc ? a.cf[i - nw] : a.cb[i - nw - nc];
            bad += v < 0;
            maxc = imax2(maxc, v);
        } else {
            const long long j = i - nw - 2 * nc;
            const int v = j < a.S ? a.t_f[j] : (j < 2 * a.S ? a.t_b[j - a.S] : a.t_w[j - 2 * a.S]);
            bad += j < 2 * a.S ? v < 1 : v < 0;
            maxt = imax2(maxt, v);
        }
    }
    if (bad) atomicAdd(&found[0], bad);
    if (maxt) atomicMax(&found[1], maxt);
    if (maxc) atomicMax(&found[2], maxc);
}

__global__ void k_zb_check_reset(int *found) {
    if (threadIdx.x < 4) found[threadIdx.x] = 0;
}


struct ZbPlan {
    bool narrow;                  // generation (PHASE 0, 1) in the one-word form of the cursors
    bool scen_lanes;              // replay with the scenarios on the lanes (k_zb_replay_scen)
    int record_group;             // lanes per candidate of the recording with the stages on the lanes (0: a lane per candidate)
    size_t lds_record;
    unsigned threads, threads_replay;
    long long order_stride;
    bool folded;                  // recording with the stages on the lanes + replay without weight ops
    size_t lds_folded, off_tail;
    size_t lds, lds_replay, lds_scen, off_counters, off_scratch, off_plans, off_packed, off_order, off_plan_ok, total;
};

// Enough threads to fill the chip at the occupancy the LDS state allows (at most 160 KiB per CU,
// 32 wavefronts per CU, 256 CUs), within about 2 GiB of queue memory.
unsigned threads_for(size_t lds, long long per_thread) {
    long long waves_per_cu = (160ll << 10) / (long long)lds;
    if (waves_per_cu > 32) waves_per_cu = 32;
    long long nt = 256 * waves_per_cu * kZbBlock;
    const long long cap = (2048ll << 20) / per_thread / kZbBlock * kZbBlock;
    if (nt > cap) nt = cap;
    if (nt < 16 * kZbBlock) nt = 16 * kZbBlock;
    return (unsigned)nt;
}

bool plan_zb(int S, int N, long long C, long long K, ZbPlan *p) {
    if (S < 1 || S > ADAPTRA_MAX_STAGES || N < 1 || N > ADAPTRA_MAX_MICROBATCHES) return false;
    if (C < 1 || C > INT32_MAX || K < 1 || K > INT32_MAX) return false;
    const long long per_thread = 2ll * S * N * 4;
    const int Spad = (S + 7) & ~7;
    auto lds_bytes = [&](int stage_ints) { return ((size_t)Spad * 64 + (size_t)S * stage_ints + 6 * (size_t)S + 2) * 4; };
    p->narrow = N <= 255;
    p->lds = lds_bytes(p->narrow ? Cursors<true>::kStage : Cursors<false>::kStage);
    p->lds_replay = lds_bytes(Cursors<false>::kStage);
    if (p->lds_replay > (160u << 10)) return false;
    p->threads = threads_for(p->lds, per_thread);
    p->threads_replay = threads_for(p->lds_replay, per_thread);
    size_t o = 0;
    p->off_counters = o; o += 256;
    p->off_scratch = o; o += adaptra_detail::align256((size_t)p->threads * per_thread);
    p->off_plans = o;   o += adaptra_detail::align256((size_t)C * S * 3 * N);
    p->off_packed = o;  o += adaptra_detail::align256((size_t)((C + kZbBlock - 1) / kZbBlock) * kZbBlock * S * packed_words(N) * 4);
    // Scenario lanes fill 64 lanes with K scenarios of one candidate, candidate lanes with 64
    // candidates of one scenario, at several times the work per pair: scenario lanes from
    // kScenReplayFrom scenarios on, while the slot of an op fits its entry's byte, a wavefront's
    // state the LDS of a CU and the grid its limit.
    p->order_stride = (3ll * S * N + 15) / 16 * 16 + 16;        // the loads run one block of 16 ahead
    p->lds_scen = (((size_t)4 * S + (size_t)N + 1) * 64 + 3 * (size_t)S) * 4;
    p->scen_lanes = K >= kScenReplayFrom && N <= 255 && p->lds_scen <= (160u << 10) &&
                    ((C + kXcds - 1) / kXcds) * kXcds * ((K + kZbBlock - 1) / kZbBlock) <= INT32_MAX;
    // The recording with the stages on the lanes is the quicker one while all its wavefronts
    // are resident at once (its queues, 2 N rows of 64 lanes, are what limits that).
    p->record_group = S <= 8 ? 8 : (S <= 16 ? 16 : (S <= 32 ? 32 : 64));
    p->lds_record = (size_t)2 * N * kZbBlock * 4;
    if (p->record_group) {
        const long long blocks = (C * p->record_group + kZbBlock - 1) / kZbBlock;
        long long per_cu = p->lds_record <= (160u << 10) ? (long long)((160u << 10) / p->lds_record) : 0;
        if (per_cu > 32) per_cu = 32;
        if (blocks > kCus * per_cu) p->record_group = 0;
    }
    p->folded = p->scen_lanes && p->record_group != 0;
    p->lds_folded = (((size_t)(S <= 32 ? 0 : 3 * S) + (size_t)N) * 64 + 3 * (size_t)S) * 4;   // up to 32 stages only the ready times are in LDS
    if (p->folded) p->order_stride = (2ll * S * N + 63) / 64 * 64 + 64;        // the loads run 64 entries ahead
    p->off_order = o;   o += adaptra_detail::align256(p->scen_lanes ? (size_t)C * (size_t)p->order_stride * (p->folded ? 16 : 2) : 0);
    p->off_tail = o;    o += adaptra_detail::align256(p->folded ? (size_t)C * S * 4 : 0);
    p->off_plan_ok = o; o += adaptra_detail::align256(p->scen_lanes ? (size_t)C : 0);
    p->total = o;
    return true;
}

template <int PHASE, bool NARROW, bool QLDS = false>
int launch_zb(ZbArgs a, long long scenarios, unsigned full, size_t lds, hipStream_t st) {
    if (lds > 48 * 1024) {                                   // above the default dynamic-LDS limit
        hipError_t e = hipFuncSetAttribute((const void *)k_zb<PHASE, NARROW, QLDS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return adaptra_detail::hip_fail(e);
    }
    const long long units = (a.C + kZbBlock - 1) / kZbBlock * scenarios;   // one wavefront each, at most `full` threads at a time
    a.threads = (unsigned)(units < (long long)(full / kZbBlock) ? units : (long long)(full / kZbBlock)) * kZbBlock;
    hipLaunchKernelGGL((k_zb<PHASE, NARROW, QLDS>), dim3(a.threads / kZbBlock), dim3(kZbBlock), lds, st, a);
    ADAPTRA_CHECK_LAUNCH();
    return ADAPTRA_OK;
}

template <int REGS>
int launch_replay_folded(const ZbArgs &a, long long blocks, size_t lds, hipStream_t st) {
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)k_zb_replay_folded<REGS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return adaptra_detail::hip_fail(e);
    }
    hipLaunchKernelGGL((k_zb_replay_folded<REGS>), dim3((unsigned)blocks), dim3(kZbBlock), lds, st, a);
    ADAPTRA_CHECK_LAUNCH();
    return ADAPTRA_OK;
}

template <int G, bool FOLDED>
int launch_record(const ZbArgs &a, size_t lds, hipStream_t st) {
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)k_zb_record_stages<G, FOLDED>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return adaptra_detail::hip_fail(e);
    }
    const unsigned blocks = (unsigned)((a.C * G + kZbBlock - 1) / kZbBlock);
    hipLaunchKernelGGL((k_zb_record_stages<G, FOLDED>), dim3(blocks), dim3(kZbBlock), lds, st, a);
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

int adaptra_zb_check_inputs(const adaptra_params_t *params, const int32_t *t_w, const adaptra_candidates_t *cands,
                            const adaptra_scenarios_t *scens, void *workspace, size_t workspace_bytes, void *stream) {
    if (!params || !cands || !scens || !t_w) return ADAPTRA_EINVAL;
    ZbPlan p;
    if (!plan_zb(params->S, params->M, cands->n, scens->n, &p)) return ADAPTRA_EINVAL;
    if (!params->t_f || !params->t_b || !cands->w) return ADAPTRA_EINVAL;
    if (params->S > 1 && (!scens->c_fwd || !scens->c_bwd)) return ADAPTRA_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < p.total) return ADAPTRA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    ZbArgs a{};
    a.S = params->S; a.N = params->M;
    a.t_f = params->t_f; a.t_b = params->t_b; a.t_w = t_w;
    a.C = cands->n; a.K = scens->n;
    a.w = cands->w; a.cf = scens->c_fwd; a.cb = scens->c_bwd;
    int *found = (int *)((char *)workspace + p.off_counters) + 16;     // behind the work counters
    hipLaunchKernelGGL(k_zb_check_reset, dim3(1), dim3(64), 0, st, found);
    ADAPTRA_CHECK_LAUNCH();
    const long long n = (long long)a.S * a.C + 2ll * (a.S - 1) * a.K + 3 * a.S;
    hipLaunchKernelGGL(k_zb_check, dim3((unsigned)adaptra_detail::blocks_for(n, 4096)), dim3(adaptra_detail::kThreadsPerBlock), 0, st, a, found);
    ADAPTRA_CHECK_LAUNCH();
    int host[4] = {0, 0, 0, 0};
    hipError_t e = hipMemcpyAsync(host, found, sizeof(host), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return adaptra_detail::hip_fail(e);
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return adaptra_detail::hip_fail(e);
    if (host[0] != 0) return ADAPTRA_ERANGE;
    if (3ll * a.N * a.S * ((long long)host[1] + (long long)host[2]) >= (1ll << 31)) return ADAPTRA_EOVERFLOW;
    return ADAPTRA_OK;
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
    // each stage's op types are read by the replay with the candidates on the lanes only
    a.plans = p.scen_lanes && p.record_group ? nullptr : (uint8_t *)workspace + p.off_plans;
    uint32_t *packed = (uint32_t *)((char *)workspace + p.off_packed);
    a.packed = packed;
    unsigned long long *counters = (unsigned long long *)((char *)workspace + p.off_counters);
    hipLaunchKernelGGL(k_zb_reset, dim3(1), dim3(64), 0, st, counters);
    ADAPTRA_CHECK_LAUNCH();
    a.order = p.scen_lanes && !p.folded && plan_scenario >= 0 ? (uint16_t *)((char *)workspace + p.off_order) : nullptr;
    a.order_folded = p.folded && plan_scenario >= 0 ? (uint4 *)((char *)workspace + p.off_order) : nullptr;
    a.tail_w = (int *)((char *)workspace + p.off_tail);
    a.plan_ok = (uint8_t *)workspace + p.off_plan_ok;
    a.order_stride = p.order_stride;
    a.next_unit = counters;
    if (plan_scenario < 0)
        return p.narrow ? launch_zb<0, true>(a, a.K, p.threads, p.lds, st) : launch_zb<0, false>(a, a.K, p.threads, p.lds, st);
    // one plan per candidate, under the plan scenario
    // With no more wavefronts than CUs each has a CU's LDS to itself: the queues go there.
    const size_t lds_queues = p.lds + (size_t)2 * a.S * a.N * kZbBlock * 4;
    const bool queues_in_lds = (a.C + kZbBlock - 1) / kZbBlock <= kCus && lds_queues <= (160u << 10);
    int rc;
    if (p.record_group) {
        const bool f = p.folded;
        switch (p.record_group) {
            case 8:  rc = f ? launch_record<8, true>(a, p.lds_record, st) : launch_record<8, false>(a, p.lds_record, st); break;
            case 16: rc = f ? launch_record<16, true>(a, p.lds_record, st) : launch_record<16, false>(a, p.lds_record, st); break;
            case 32: rc = f ? launch_record<32, true>(a, p.lds_record, st) : launch_record<32, false>(a, p.lds_record, st); break;
            default: rc = f ? launch_record<64, true>(a, p.lds_record, st) : launch_record<64, false>(a, p.lds_record, st); break;
        }
    } else if (queues_in_lds)
        rc = p.narrow ? launch_zb<1, true, true>(a, 1, kCus * kZbBlock, lds_queues, st) : launch_zb<1, false, true>(a, 1, kCus * kZbBlock, lds_queues, st);
    else
        rc = p.narrow ? launch_zb<1, true>(a, 1, p.threads, p.lds, st) : launch_zb<1, false>(a, 1, p.threads, p.lds, st);
    if (rc) return rc;
    if (p.folded) {
        const long long blocks = (a.C + kXcds - 1) / kXcds * kXcds * ((a.K + kZbBlock - 1) / kZbBlock);
        return a.S <= 16 ? launch_replay_folded<16>(a, blocks, p.lds_folded, st)
             : a.S <= 32 ? launch_replay_folded<32>(a, blocks, p.lds_folded, st)
                         : launch_replay_folded<0>(a, blocks, p.lds_folded, st);
    }
    if (p.scen_lanes) {
        if (p.lds_scen > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)k_zb_replay_scen, hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds_scen);
            if (e != hipSuccess) return adaptra_detail::hip_fail(e);
        }
        const long long blocks = (a.C + kXcds - 1) / kXcds * kXcds * ((a.K + kZbBlock - 1) / kZbBlock);
        hipLaunchKernelGGL(k_zb_replay_scen, dim3((unsigned)blocks), dim3(kZbBlock), p.lds_scen, st, a);
        ADAPTRA_CHECK_LAUNCH();
        return ADAPTRA_OK;
    }
    const long long words = (a.C + kZbBlock - 1) / kZbBlock * kZbBlock * a.S * packed_words(a.N);
    hipLaunchKernelGGL(k_zb_pack, dim3((unsigned)adaptra_detail::blocks_for(words, 1 << 16)), dim3(adaptra_detail::kThreadsPerBlock), 0, st,
                       a.plans, packed, a.C, a.S, a.N);
    ADAPTRA_CHECK_LAUNCH();
    a.next_unit = counters + 1;
    return launch_zb<2, false>(a, a.K, p.threads_replay, p.lds_replay, st);   // every pair replays its candidate's plan
}

}  // extern "C"

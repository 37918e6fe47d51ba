// adaptra.hip -- gfx950 kernels and the C ABI of the batched pipeline-schedule evaluator.
//
// Model and notation follow the Adaptra paper: S stages, M micro-batches, w[s] warm-up
// forwards of stage s (the paper's x_s = w[s] + 1), link delays c_fwd / c_bwd, the
// dependency rules of Section 3.1 and the stage order of Sections 4.1 / 4.3.  Everything
// is int32 microseconds; there is no floating point on this path.
//
// Kernels
//   k_prepass            per candidate: clamp w, Lemma 1 test (deadlock), memory-cap test
//                        (Algorithm 1's x_max), flag byte, ring-depth class, packed w bytes
//   k_resolve_scen_lanes the hot kernel: one wavefront = one candidate at a time x 64
//                        scenarios (one per lane); stage frontiers in VGPRs, the forward
//                        frontier of the in-flight micro-batches in an LDS ring
//   k_resolve_cand_lanes few scenarios, or a scenario per candidate: one lane per pair,
//                        stage frontiers and link delays in VGPRs, micro-batch ring in LDS
//   k_resolve_general    any S / M / warm-up depth: one lane per pair (64 candidates of one
//                        scenario per wavefront), state in global scratch, DPP argmin
//   k_eval_epilogue      after the resolve kernels: flag byte and bubbles of every pair,
//                        sentinels for deadlocked pairs (one coalesced streaming pass)
//   k_sens_epilogue      adaptra_sensitivity: differences against the base scenarios
//   k_best_init / k_best_finalize   search keys and histogram set-up / decoding
//   k_best_from_eval     adaptra_eval_best: the search over the makespans the evaluation left
//   k_check_inputs       range scan for adaptra_check_inputs
//   k_seed               the paper's analytic planning (Algorithm 1, Algorithm 2, Eq. (1))
//
// Order of evaluation used by both resolve kernels: with w non-increasing over stages
// (Lemma 1) the rounds r = -w[0] .. M-1, each a forward sweep s = 0..S-1 over
// F(s, w[s] + r) followed (r >= 0) by a backward sweep s = S-1..0 over B(s, r), visit every
// op after all of its predecessors and every stage's ops in that stage's own order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"

namespace {

constexpr int kNeg = -(1 << 30);          // "no earlier op": below every shifted time
#ifndef ADAPTRA_CHUNK
#define ADAPTRA_CHUNK 16
#endif
constexpr int kChunk = ADAPTRA_CHUNK;      // candidates one wavefront works through, at most
#ifndef ADAPTRA_WPB
#define ADAPTRA_WPB 4
#endif
constexpr int kWavesPerBlock = ADAPTRA_WPB;
constexpr int kBlock = 64 * kWavesPerBlock;
constexpr int kClassDead = 255;           // deadlocked: never resolved
constexpr int kClassDeep = 254;           // warm-up depth beyond the LDS ring: general kernel
constexpr int kNumRingClasses = 16;       // ring of 8 * (class + 1) slots: up to 128 slots = 32 KiB per wavefront
constexpr int kMaxLdsHistBytes = 16384;
#ifndef ADAPTRA_PD
#define ADAPTRA_PD 4
#endif
// Wavefront priorities inside the hot kernel (s_setprio): a wavefront in a forward sweep -- LDS
// traffic and independent instructions -- goes ahead of one in a backward sweep, whose
// instructions all wait on each other and fill the gaps just as well.  Measured on configuration
// 3: 49.3 -> 47.2 ms; any two different levels do, the other way round costs 2 ms.
constexpr int kPrioForward = 2, kPrioBackward = 0;
#ifndef ADAPTRA_WAVES32
#define ADAPTRA_WAVES32 4
#endif
constexpr int kPrefetchStages = ADAPTRA_PD;        // ring reads run this many stages ahead of their use
constexpr unsigned long long kNoKey = ~0ull;

struct KArgs {
    int S, M;
    const int *t_f, *t_b, *mem_cap;
    long long C, K;
    long long Kin;                         // scenarios in the input arrays; K = Kin * (1 + links) when the
    int sens_delta;                        // scenario axis also carries the link-perturbed copies
    const int *w, *cf, *cb;
    const int *tfs, *tbs;                  // optional per-scenario stage times [S][K] (compute stragglers)
    unsigned char *cand_flag, *cand_class, *cand_wq;
    int wq_stride;                         // bytes per candidate in cand_wq
    int *out_makespan, *out_bubble;
    unsigned char *out_feasible;
    unsigned long long *keys, *hist;
    int *best_idx, *best_makespan, *best_bubble;
    int hist_bins, hist_shift, hist_in_lds;
    int *scratch;
    int cls_lo, cls_hi, ring_slots, general_all;
    int pair_div;                          // > 0: candidate c is evaluated under scenario c / pair_div only
    int direct_out;                        // hot kernel, eval: it writes the final outputs itself (see there)
    long long n_chunks;
    int chunk;                             // candidates per wavefront of the hot kernel (1..kChunk)
    int n_ktiles;
    int *status;                           // [0..3] input check, [16..32] candidates per ring class
    int *mk_t;                             // eval: makespan, candidate-major [C][K]
    int *tpad;                             // t_f at [0..63], t_b at [64..127], zero beyond stage S-1
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }
// One count into hist[bin] for every lane that calls (the callers' lanes are the scenarios of
// one candidate, whose bubbles mostly fall into one or two bins: as single atomics those would
// queue up on one address).  The lanes sharing the first lane's bin are counted with one
// atomic, then the same for the next bin still open; what is left counts for itself.
template <class Count>
__device__ __forceinline__ void hist_count(Count *hist, int bin, int lane) {
    unsigned long long open = __ballot(true);
    bool mine = true;
    for (int group = 0; group < 2 && open; ++group) {
        const int lead = __ffsll((long long)open) - 1;
        const int lead_bin = __builtin_amdgcn_readlane(bin, lead);
        const unsigned long long same = __ballot(mine && bin == lead_bin);
        if (lane == lead) atomicAdd(&hist[lead_bin], (Count)__popcll(same));
        open &= ~same;
        mine = mine && bin != lead_bin;
    }
    if (mine) atomicAdd(&hist[bin], (Count)1);
}
// Ring offset of a stage, one slot (256 B) further, wrapping to slot 0.  The offset is kept
// biased by -ring_bytes (mod 2^32) so that the wrap shows up as the carry of the add: two
// SALU ops instead of add, compare, select.  The bias is folded into the lane's base address.
__device__ __forceinline__ unsigned ring_next(unsigned t, unsigned bias) {
    asm("s_add_u32 %0, %0, 0x100\n\ts_cmov_b32 %0, %1" : "+s"(t) : "s"(bias) : "scc");
    return t;
}

// The two uniform chores of a forward step, in one asm block so that the scheduler keeps
// them next to the step's VALU work (separate asm statements get s_nop spacers):
//   - returns bit `kBit` of the 64-bit mask set ? b : a.  One SALU op spreads the bit over
//     vcc (a signed one-bit field extract), one VALU op selects; a branch around a move
//     measured slower, hoisted lane masks would need two SGPRs per stage.
//   - advances the stage's ring offset `t` by one slot (see ring_next).
template <int kBit>
__device__ __forceinline__ int select_by_bit_and_advance(unsigned long long mask, int a, int b,
                                                         unsigned &t, unsigned bias) {
    int o;
    asm("s_bfe_i64 vcc, %2, %3\n\tv_cndmask_b32 %0, %4, %5, vcc\n\t"
        "s_add_u32 %1, %1, 0x100\n\ts_cmov_b32 %1, %6"
        : "=v"(o), "+s"(t) : "s"(mask), "n"(kBit | (1 << 16)), "v"(a), "v"(b), "s"(bias) : "scc", "vcc");
    return o;
}

typedef __attribute__((address_space(3))) int lds_int;

// Compile-time stage loops: the stage index must be a constant (register arrays, asm
// immediates), so they are unrolled by template recursion rather than by a pragma.
template <int kI>
struct StageIndex {
    static constexpr int value = kI;
};
template <int kBegin, int kEnd, class F>
__device__ __forceinline__ void stages_up(F &&f) {
    if constexpr (kBegin < kEnd) {
        f(StageIndex<kBegin>{});
        stages_up<kBegin + 1, kEnd>(f);
    }
}
template <int kBegin, int kEnd, class F>          // kBegin down to kEnd, inclusive
__device__ __forceinline__ void stages_down(F &&f) {
    if constexpr (kBegin >= kEnd) {
        f(StageIndex<kBegin>{});
        stages_down<kBegin - 1, kEnd>(f);
    }
}
// stages kBegin, kBegin+1, ... while the stage index is below `limit` (uniform): the first
// stage at or past the limit ends the sweep with a single branch.
template <int kBegin, int kEnd, class F>
__device__ __forceinline__ void stages_below(int limit, F &&f) {
    if constexpr (kBegin < kEnd) {
        if (kBegin < limit) {
            f(StageIndex<kBegin>{});
            stages_below<kBegin + 1, kEnd>(limit, f);
        }
    }
}
#define ADAPTRA_STAGE_LAMBDA(si) [&](auto si) __attribute__((always_inline))

// Kernel arguments of the hot kernel, read where they are used.  The struct is the
// kernel's only parameter, so it sits at the start of the kernarg segment; going through
// an opaque copy of that pointer makes every use a fresh scalar load (a scalar-cache hit)
// instead of two dozen values kept in SGPRs across the round loops, where the stage
// constants and ring offsets need the room.
typedef const __attribute__((address_space(4))) KArgs *KArgsPtr;
__device__ __forceinline__ KArgsPtr kargs() {
    KArgsPtr p = (KArgsPtr)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(p));
    return p;
}
__device__ __forceinline__ int clampw(int w, int M) { return w < 0 ? 0 : (w > M - 1 ? M - 1 : w); }

// ---------------------------------------------------------------------------------------
// Wavefront-wide minimum of a 64-bit key: DPP butterflies inside each row of 16 lanes,
// ds_swizzle across the two rows of a half, v_readlane across the halves.
template <int kCtrl>
__device__ __forceinline__ unsigned long long dpp_min_step(unsigned long long v) {
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    unsigned olo = (unsigned)__builtin_amdgcn_update_dpp((int)lo, (int)lo, kCtrl, 0xf, 0xf, false);
    unsigned ohi = (unsigned)__builtin_amdgcn_update_dpp((int)hi, (int)hi, kCtrl, 0xf, 0xf, false);
    unsigned long long o = ((unsigned long long)ohi << 32) | olo;
    return o < v ? o : v;
}

__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
    v = dpp_min_step<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    v = dpp_min_step<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    v = dpp_min_step<0x141>(v);   // row_half_mirror: joins the two quads of 8 lanes
    v = dpp_min_step<0x140>(v);   // row_mirror: joins the two halves of a row
    {
        unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
        unsigned olo = (unsigned)__builtin_amdgcn_ds_swizzle((int)lo, 0x401F);   // lane ^ 16
        unsigned ohi = (unsigned)__builtin_amdgcn_ds_swizzle((int)hi, 0x401F);
        unsigned long long o = ((unsigned long long)ohi << 32) | olo;
        v = o < v ? o : v;
    }
    unsigned long long a = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(v >> 32), 0) << 32) |
                           (unsigned)__builtin_amdgcn_readlane((int)v, 0);
    unsigned long long b = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(v >> 32), 32) << 32) |
                           (unsigned)__builtin_amdgcn_readlane((int)v, 32);
    return a < b ? a : b;
}

// ---------------------------------------------------------------------------------------
// Per candidate, independent of the scenario: w' = clamp(w, 0, M-1); deadlock iff some
// w'[s] < w'[s+1] (Lemma 1); memory cap exceeded iff some w'[s] + 1 > mem_cap[s]
// (Algorithm 1, x_max).  Also packs w' into bytes for the hot kernel and bins the
// candidate by the ring depth it needs, w'[0] + 1 slots.
__global__ __launch_bounds__(kBlock) void k_prepass(KArgs a) {
    __shared__ int class_count[kNumRingClasses + 1];
    if (threadIdx.x <= kNumRingClasses) class_count[threadIdx.x] = 0;
    if (blockIdx.x == 0 && threadIdx.x < 128) {             // stage times padded with zeros (candidate-lanes kernel)
        const int i = threadIdx.x & 63;
        a.tpad[threadIdx.x] = i < a.S ? (threadIdx.x < 64 ? a.t_f[i] : a.t_b[i]) : 0;
    }
    __syncthreads();
    long long c = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (c < a.C) {
    const int S = a.S, M = a.M;
    bool dead = false, mem = false;
    int prev = INT32_MAX, w0 = 0;
    // One pass over the stages, four at a time: the Lemma 1 and memory tests, and w as bytes for
    // the ring kernels (wq_stride is a multiple of 4; bytes past S are the padding stages of the
    // kernel size the pipeline runs in, w = 0).  The bytes of a candidate no ring kernel takes
    // are never read.
    unsigned *const q = (unsigned *)(a.cand_wq + c * a.wq_stride);
    for (int s4 = 0; s4 < a.wq_stride; s4 += 4) {
        unsigned packed = 0;
        for (int j = 0; j < 4; ++j) {
            const int s = s4 + j;
            if (s >= S) break;
            const int ws = clampw(a.w[(long long)s * a.C + c], M);
            if (s == 0) w0 = ws;
            if (prev < ws) dead = true;
            if (a.mem_cap && ws + 1 > a.mem_cap[s]) mem = true;
            prev = ws;
            packed |= (unsigned)(ws & 0xff) << (8 * j);
        }
        q[s4 / 4] = packed;
    }
    int flag = (dead ? ADAPTRA_FLAG_DEADLOCK : 0) | (mem ? ADAPTRA_FLAG_MEMCAP : 0);
    if (flag == 0) flag = ADAPTRA_FLAG_FEASIBLE;
    int cls;
    if (dead) cls = kClassDead;
    else if (w0 + 1 > 8 * kNumRingClasses) cls = kClassDeep;
    else cls = (w0 + 8) / 8 - 1;            // ring of 8 * (cls + 1) >= w0 + 1 slots
    a.cand_flag[c] = (unsigned char)flag;
    a.cand_class[c] = (unsigned char)cls;
    if (!dead) atomicAdd(&class_count[cls == kClassDeep ? kNumRingClasses : cls], 1);
    }
    __syncthreads();       // how many candidates need which ring depth: lets the kernels that
    if (threadIdx.x <= kNumRingClasses && class_count[threadIdx.x])   // have no share exit at once
        atomicAdd(&a.status[16 + threadIdx.x], class_count[threadIdx.x]);
}

// Runs after the resolve kernels, which leave the makespan of every pair that is not
// deadlocked in the candidate-major scratch mk_t[C][K].  Each block transposes one tile of
// 64 candidates x 64 scenarios through LDS and writes, coalesced along the candidate axis:
// makespan, flag byte, and bubble[s] = makespan - M (t_f[s] + t_b[s]) (idle time of stage s
// inside [0, makespan]); INT32_MAX for deadlocked pairs.
__global__ __launch_bounds__(kBlock) void k_eval_epilogue(KArgs a) {
    __shared__ int tile[64][65];
    __shared__ int tau[ADAPTRA_MAX_STAGES];
    const long long ctiles = (a.C + 63) / 64;
    const long long c0 = ((long long)blockIdx.x % ctiles) * 64;
    const long long k0 = ((long long)blockIdx.x / ctiles) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    if (a.direct_out) {
        // The scenario-lanes kernel has written the outputs of every candidate of ring class
        // <= cls_hi (and the sentinels of the deadlocked ones) itself: only tiles that hold a
        // candidate left to the general kernel remain, and those are redone as a whole.
        const long long c = c0 + tx;
        const bool left = c < a.C && !(a.cand_flag[c] & ADAPTRA_FLAG_DEADLOCK) && a.cand_class[c] > a.cls_hi;
        if (!__syncthreads_or(left)) return;
    }
    if (threadIdx.x < a.S) tau[threadIdx.x] = a.t_f[threadIdx.x] + a.t_b[threadIdx.x];   // unless per scenario
    for (int i = ty; i < 64; i += kWavesPerBlock) {          // row = candidate, lanes = scenarios
        const long long c = c0 + i, k = k0 + tx;
        if (c < a.C && k < a.K && !(a.cand_flag[c] & ADAPTRA_FLAG_DEADLOCK)) tile[i][tx] = a.mk_t[c * a.K + k];
    }
    __syncthreads();
    const long long P = a.C * a.K;
    const long long c = c0 + tx;
    if (c >= a.C) return;
    const int flag = a.cand_flag[c];
    const bool dead = flag & ADAPTRA_FLAG_DEADLOCK;
    for (int i = ty; i < 64; i += kWavesPerBlock) {          // row = scenario, lanes = candidates
        const long long k = k0 + i;
        if (k >= a.K) break;
        const long long p = k * a.C + c;
        const int mk = dead ? INT32_MAX : tile[tx][i];
        a.out_makespan[p] = mk;
        a.out_feasible[p] = (unsigned char)flag;
        if (a.out_bubble)
            for (int s = 0; s < a.S; ++s) {
                const int tau_s = a.tfs ? a.tfs[(long long)s * a.K + k] + a.tbs[(long long)s * a.K + k] : tau[s];
                a.out_bubble[(long long)s * P + p] = dead ? INT32_MAX : mk - a.M * tau_s;
            }
    }
}

// Sensitivity epilogue.  The resolve kernels ran with the scenario axis holding Kin base
// scenarios followed by, for every link l, a copy with c_fwd[l] raised by sens_delta:
// mk_t[c][v * Kin + k], v = 0 base, v = 1 + l.  Writes, candidate-major (coalesced along k):
//   out_makespan[c][k]   = base makespan                      (a.out_makespan, optional)
//   out_feasible[c][k]   = flag byte of the candidate         (a.out_feasible, optional)
//   out_sens[c][l][k]    = makespan(c_fwd[l] + delta) - base  (a.out_bubble)
// INT32_MAX for a deadlocked candidate.
__global__ __launch_bounds__(kBlock) void k_sens_epilogue(KArgs a) {
    const long long n = a.C * a.Kin;
    const long long i = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const long long c = i / a.Kin, k = i % a.Kin;
    const bool dead = a.cand_flag[c] & ADAPTRA_FLAG_DEADLOCK;
    const int base = dead ? INT32_MAX : a.mk_t[c * a.K + k];
    if (a.out_makespan) a.out_makespan[i] = base;
    if (a.out_feasible) a.out_feasible[i] = a.cand_flag[c];
    for (int l = 0; l + 1 < a.S; ++l)
        a.out_bubble[(c * (a.S - 1) + l) * a.Kin + k] = dead ? INT32_MAX : a.mk_t[c * a.K + (1 + l) * a.Kin + k] - base;
}

__global__ __launch_bounds__(kBlock) void k_best_init(KArgs a) {
    const long long n = a.K + (a.hist ? (long long)a.S * a.hist_bins : 0);
    const long long stride = (long long)gridDim.x * kBlock;
    for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        if (i < a.K) a.keys[i] = kNoKey;
        else a.hist[i - a.K] = 0ull;
    }
}

// The search over makespans that adaptra_eval's resolve kernels have just left in mk_t[C][K]
// (adaptra_eval_best): nothing is resolved twice.  One wavefront = 64 scenarios (lanes) x a
// run of 64 candidates; only the rows of feasible candidates are read (coalesced along the
// scenario axis).  Keys and histogram as in the resolve kernels' search.
// RUNS > 0 (pipelines of up to RUNS stages, with a histogram): a lane -- one scenario -- walks
// the candidates of its tile and keeps, per stage, the bin of the last bubble and how often it
// came in a row; only a change of bin costs an atomic.  Neighbouring candidates mostly share
// their bins, so this replaces S atomics (or wavefront votes) per pair by a compare and an add.
template <int RUNS>
__global__ __launch_bounds__(kBlock) void k_best_from_eval(KArgs a) {
    extern __shared__ unsigned hist_lds_scan[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const bool lds_hist = a.hist && a.hist_in_lds;
    if (lds_hist) {
        for (int i = threadIdx.x; i < a.S * a.hist_bins; i += kBlock) hist_lds_scan[i] = 0;
        __syncthreads();
    }
    const long long ktiles = (a.K + 63) / 64;
    const long long task = (long long)blockIdx.x * kWavesPerBlock + wv;
    const long long k = (task % ktiles) * 64 + lane;
    const long long c0 = (task / ktiles) * 64;
    const bool kvalid = k < a.K;
    unsigned long long key = kNoKey;
    int run_bin[RUNS > 0 ? RUNS : 1], run_len[RUNS > 0 ? RUNS : 1], busy[RUNS > 0 ? RUNS : 1];
    if constexpr (RUNS > 0) {
#pragma unroll
        for (int s = 0; s < RUNS; ++s) {
            run_bin[s] = 0;
            run_len[s] = 0;
            busy[s] = 0;
            if (s < a.S && kvalid)
                busy[s] = a.M * (a.tfs ? a.tfs[(long long)s * a.K + k] + a.tbs[(long long)s * a.K + k] : a.t_f[s] + a.t_b[s]);
        }
    }
    auto count_run = [&](int s, int bin, int n) {
        if (lds_hist) atomicAdd(&hist_lds_scan[s * a.hist_bins + bin], (unsigned)n);
        else atomicAdd(&a.hist[s * a.hist_bins + bin], (unsigned long long)n);
    };
    // The feasible candidates of this tile as a mask (lane j looks at candidate c0 + j), then
    // four of them at a time so that their loads are in flight together.
    unsigned long long feasible = __ballot(c0 + lane < a.C && a.cand_flag[c0 + lane < a.C ? c0 + lane : 0] == ADAPTRA_FLAG_FEASIBLE);
    while (feasible) {
        long long cs[4];
        int mks[4], n = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (feasible) {
                cs[u] = c0 + (__ffsll((long long)feasible) - 1);
                feasible &= feasible - 1;
                n = u + 1;
            } else {
                cs[u] = cs[0];
            }
            mks[u] = kvalid ? a.mk_t[cs[u] * a.K + k] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u >= n || !kvalid) continue;
            const long long c = cs[u];
            const int mk = mks[u];
            const unsigned long long cand = ((unsigned long long)(unsigned)mk << 32) | (unsigned)c;
            key = cand < key ? cand : key;
            if (!a.hist) continue;
            if constexpr (RUNS > 0) {
#pragma unroll
                for (int s = 0; s < RUNS; ++s) {
                    if (s >= a.S) break;
                    int bin = (mk - busy[s]) >> a.hist_shift;
                    bin = bin > a.hist_bins - 1 ? a.hist_bins - 1 : bin;
                    const bool same = bin == run_bin[s];
                    if (!same && run_len[s]) count_run(s, run_bin[s], run_len[s]);
                    run_len[s] = same ? run_len[s] + 1 : 1;
                    run_bin[s] = bin;
                }
            } else {
                for (int s = 0; s < a.S; ++s) {
                    const int tau_s = a.tfs ? a.tfs[(long long)s * a.K + k] + a.tbs[(long long)s * a.K + k] : a.t_f[s] + a.t_b[s];
                    int b = (mk - a.M * tau_s) >> a.hist_shift;
                    b = b > a.hist_bins - 1 ? a.hist_bins - 1 : b;
                    if (lds_hist) hist_count(hist_lds_scan + s * a.hist_bins, b, lane);
                    else hist_count(a.hist + s * a.hist_bins, b, lane);
                }
            }
        }
    }
    if constexpr (RUNS > 0) {
        if (a.hist && kvalid) {
#pragma unroll
            for (int s = 0; s < RUNS; ++s)
                if (s < a.S && run_len[s]) count_run(s, run_bin[s], run_len[s]);
        }
    }
    if (key != kNoKey) atomicMin(&a.keys[k], key);
    if (lds_hist) {
        __syncthreads();
        for (int i = threadIdx.x; i < a.S * a.hist_bins; i += kBlock) {
            const unsigned cnt = hist_lds_scan[i];
            if (cnt) atomicAdd(&a.hist[i], (unsigned long long)cnt);
        }
    }
}

// key = makespan << 32 | candidate: the minimum key is the smallest makespan, ties to the
// lowest index.  Bubbles of the winner: makespan - M (t_f + t_b) per stage.
__global__ __launch_bounds__(kBlock) void k_best_finalize(KArgs a) {
    const long long k = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (k >= a.K) return;
    const unsigned long long key = a.keys[k];
    const bool none = key == kNoKey;
    const int mk = none ? INT32_MAX : (int)(key >> 32);
    a.best_idx[k] = none ? -1 : (int)(unsigned)key;
    a.best_makespan[k] = mk;
    if (a.best_bubble)
        for (int s = 0; s < a.S; ++s)
            a.best_bubble[k * a.S + s] =
                none ? INT32_MAX
                     : mk - a.M * (a.tfs ? a.tfs[(long long)s * a.K + k] + a.tbs[(long long)s * a.K + k] : a.t_f[s] + a.t_b[s]);
}

// ---------------------------------------------------------------------------------------
// General kernel: one lane per pair, 64 consecutive candidates of one scenario per
// wavefront.  Plain form of the Section 3.1 recurrence:
//   start F(s,m) = max(last[s], fin F(s-1,m) + c_fwd[s-1]),  fin = start + t_f[s]
//   start B(s,m) = max(last[s], fin B(s+1,m) + c_bwd[s]),    fin = start + t_b[s]
// State per lane in global scratch, laid out [index][thread] so that lanes coalesce:
//   last[S], w'[S], fwd[M] (finish time of micro-batch m's latest forward).
template <bool BEST>
__global__ __launch_bounds__(kBlock) void k_resolve_general(KArgs a) {
    const int S = a.S, M = a.M;
    const long long NT = (long long)gridDim.x * kBlock;
    const long long tid = (long long)blockIdx.x * kBlock + threadIdx.x;
    const int lane = threadIdx.x & 63;
    int *last = a.scratch + tid;
    int *wl = a.scratch + (long long)S * NT + tid;
    int *fwd = a.scratch + 2ll * S * NT + tid;
    if (!a.general_all) {      // only the candidates the on-chip kernels left over: often none
        int mine = 0;
        for (int cls = a.cls_hi + 1; cls <= kNumRingClasses; ++cls) mine += a.status[16 + cls];
        if (mine == 0) return;
    }
    const long long ctiles = (a.C + 63) / 64;
    const long long ntiles = a.pair_div ? ctiles : a.K * ctiles;
    const long long nwaves = NT >> 6;
    for (long long tile = tid >> 6; tile < ntiles; tile += nwaves) {
        const long long c = (tile % ctiles) * 64 + lane;
        // paired mode (the guided search): every candidate has its own scenario
        const long long k = a.pair_div ? (c < a.C ? c / a.pair_div : 0) : tile / ctiles;
        const long long kin = k % a.Kin;             // scenario in the input arrays
        const int link_up = (int)(k / a.Kin) - 1;    // link whose forward delay this copy raises, or -1
        bool run = false;
        if (c < a.C) {
            const int flag = a.cand_flag[c];
            const int cls = a.cand_class[c];
            run = BEST ? (flag == ADAPTRA_FLAG_FEASIBLE) : !(flag & ADAPTRA_FLAG_DEADLOCK);
            if (!a.general_all && cls <= a.cls_hi) run = false;   // the on-chip kernels' share
        }
        unsigned long long key = kNoKey;
        if (run) {
            for (int s = 0; s < S; ++s) {
                wl[s * NT] = clampw(a.w[(long long)s * a.C + c], M);
                last[s * NT] = 0;
            }
            const int w0 = wl[0];
            for (int r = -w0; r < M; ++r) {
                for (int s = 0; s < S; ++s) {                    // forward sweep
                    const int m = wl[s * NT] + r;
                    if (m >= 0 && m < M) {
                        const int arrive = s == 0 ? 0 : fwd[m * NT] + a.cf[(long long)(s - 1) * a.Kin + kin] + (s - 1 == link_up ? a.sens_delta : 0);
                        const int fin = imax(last[s * NT], arrive) + (a.tfs ? a.tfs[(long long)s * a.Kin + kin] : a.t_f[s]);
                        last[s * NT] = fin;
                        fwd[m * NT] = fin;
                    }
                }
                if (r >= 0) {                                    // backward sweep
                    int carry = 0;
                    for (int s = S - 1; s >= 0; --s) {
                        const int arrive = s == S - 1 ? 0 : carry + a.cb[(long long)s * a.Kin + kin];
                        const int fin = imax(last[s * NT], arrive) + (a.tbs ? a.tbs[(long long)s * a.Kin + kin] : a.t_b[s]);
                        last[s * NT] = fin;
                        carry = fin;
                    }
                }
            }
            int mk = 0;
            for (int s = 0; s < S; ++s) mk = imax(mk, last[s * NT]);
            if (BEST) {
                key = ((unsigned long long)(unsigned)mk << 32) | (unsigned)c;
                if (a.hist) {
                    for (int s = 0; s < S; ++s) {
                        const int tau_s = a.tfs ? a.tfs[(long long)s * a.Kin + kin] + a.tbs[(long long)s * a.Kin + kin] : a.t_f[s] + a.t_b[s];
                        int b = (mk - M * tau_s) >> a.hist_shift;
                        b = b > a.hist_bins - 1 ? a.hist_bins - 1 : b;
                        atomicAdd(&a.hist[s * a.hist_bins + b], 1ull);
                    }
                }
            } else {
                a.mk_t[c * a.K + k] = mk;        // transposed and completed by k_eval_epilogue
            }
        }
        if (BEST) {
            if (a.pair_div) {
                if (key != kNoKey) atomicMin(&a.keys[k], key);
            } else {
                key = wave_min_u64(key);
                if (lane == 0 && key != kNoKey) atomicMin(&a.keys[k], key);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Candidate-lanes kernel: lane = candidate, like the general kernel, but with the state on
// chip, for the problems the hot kernel's mapping does not fit: fewer scenarios than would
// fill its lanes, and the guided search's paired form (a scenario per candidate).
//   last[S]              VGPRs (the stage loops are unrolled: static indices)
//   c_fwd, c_bwd         VGPRs, 2 (S - 1) per lane (the scenario may differ per lane)
//   w                    S bytes packed into S / 4 VGPRs
//   fwd[m]               LDS ring [slot][lane], D slots per wavefront as in the hot kernel,
//                        slot = m mod D with a per-lane index (bank = lane: conflict-free)
// Plain form of the Section 3.1 recurrence (see the general kernel).  After the fill phase (taken
// stage by stage, see there) all lanes walk the rounds r = 0 .. M-1 together; a lane's forward
// step of stage s counts only if its micro-batch w[s] + r exists (a select, no divergence).  The write of a step that does not
// count lands in a slot no live micro-batch uses: slots of live micro-batches differ from it
// by less than D.  Ring reads follow the previous stage's write in program order, so a link
// with equal w needs no special case.  S is padded as in the hot kernel.
// AHEAD: the ring values are read three stages before their use, so
// that the LDS latency is not paid stage by stage (the plain form waits for each read right
// where it is issued; measured 1.3-1.6 times slower from 16 stages on, whatever the size of the
// launch).  The read of stage s
// then precedes the write of stage s-1, which targets the same slot exactly when the two stages
// share w (w is non-increasing, so no earlier stage of the round can have written it): in that
// case the value just computed is taken instead.  Two more instructions per stage and round,
// and registers for the values in flight.
template <int S, bool BEST, bool VT, bool AHEAD>
__global__ __launch_bounds__(kBlock, AHEAD || S >= 64 || (VT && S >= 16) ? 2 : (S >= 32 ? 4 : 6)) void k_resolve_cand_lanes(KArgs) {
    // The arguments are read through kargs() where they are needed (see there): kept in SGPRs
    // across the round loop they would crowd out the loop's own scalars.
    extern __shared__ int lds[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int D = kargs()->ring_slots, M = kargs()->M;
    int *const ring = lds + wv * D * 64 + lane;          // slot i of this lane at ring[i * 64]
    const long long ctiles = (kargs()->C + 63) / 64;
    const long long ntiles = kargs()->pair_div ? ctiles : kargs()->K * ctiles;
    const long long nwaves = (long long)gridDim.x * kWavesPerBlock;
    // Stage times come from the zero-padded table, re-read in blocks of 16 stages inside the
    // round loop (scalar loads, a cache hit each): kept for all stages they would take 2 S
    // SGPRs, more than there are at S = 32.
    constexpr int kTimesBlock = 16;
    typedef __attribute__((address_space(4))) int ConstInt;   // written by k_prepass, constant here
    for (long long tile = (long long)blockIdx.x * kWavesPerBlock + wv; tile < ntiles; tile += nwaves) {
        const long long c = (tile % ctiles) * 64 + lane;
        const long long k = kargs()->pair_div ? (c < kargs()->C ? c / kargs()->pair_div : 0) : tile / ctiles;
        const long long kin = k % kargs()->Kin;
        const int link_up = (int)(k / kargs()->Kin) - 1;
        bool run = false;
        if (c < kargs()->C) {
            const int flag = kargs()->cand_flag[c];
            const int cls = kargs()->cand_class[c];
            run = (BEST ? (flag == ADAPTRA_FLAG_FEASIBLE) : !(flag & ADAPTRA_FLAG_DEADLOCK)) &&
                  cls >= kargs()->cls_lo && cls <= kargs()->cls_hi;
        }
        if (__ballot(run) == 0ull) continue;
        // w of the lane's candidate, four stages per register; lanes that do not run get w = 0
        // (their ring indices must still stay inside the ring)
        unsigned wpk[(S + 3) / 4];
#pragma unroll
        for (int i = 0; i < (S + 3) / 4; ++i)
            wpk[i] = run ? *(const unsigned *)(kargs()->cand_wq + c * kargs()->wq_stride + 4 * i) : 0u;
        int cf[S > 1 ? S - 1 : 1], cb[S > 1 ? S - 1 : 1], last[S];
#pragma unroll
        for (int s = 0; s < S; ++s) last[s] = 0;
#pragma unroll
        for (int s = 0; s + 1 < S; ++s) {
            const bool real = s + 1 < kargs()->S;
            cf[s] = real ? kargs()->cf[(long long)s * kargs()->Kin + kin] + (s == link_up ? kargs()->sens_delta : 0) : 0;
            cb[s] = real ? kargs()->cb[(long long)s * kargs()->Kin + kin] : 0;
        }
        // Per-scenario stage times (VT): the lane's own t_f and t_b, 2 S more registers.
        int tfv[VT ? S : 1], tbv[VT ? S : 1];
        if constexpr (VT) {
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const bool real = s < kargs()->S;
                tfv[s] = real ? kargs()->tfs[(long long)s * kargs()->Kin + kin] : 0;
                tbv[s] = real ? kargs()->tbs[(long long)s * kargs()->Kin + kin] : 0;
            }
        }
        // The rounds before r = 1 hold only forwards up to the last one, and what those wait for
        // is there once the stage before has run its own (w is non-increasing): they are taken
        // stage by stage.  Stage s runs its micro-batches 0 .. w[s] back to back; micro-batch i
        // sits in slot i for every lane (no index wraps: w < D), a lane whose stage has fewer
        // warm-up forwards than another lane's keeps its state and puts back what it read.  No
        // per-lane slot arithmetic, no test for the micro-batch's existence beyond i <= w[s], no
        // special case for links without slack -- and no rounds in which only a few stages of a
        // few lanes have work.  (Four micro-batches per iteration with their ring values read
        // together measured slower: 64 against 52 ms on the guided search.)
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int ws = (int)((wpk[s / 4] >> (8 * (s % 4))) & 0xffu);
            int t_f_s;
            if constexpr (VT) t_f_s = tfv[s];
            else t_f_s = ((const ConstInt *)kargs()->tpad)[s];
            int *p = ring;
            int arrived = s > 0 ? *p : 0;
            for (int i = 0;; ++i) {
                const bool valid = i <= ws;              // implies i < D
                if (__ballot(valid) == 0ull) break;
                int arrived_next = 0;
                if (s > 0 && i + 1 < D) arrived_next = p[64];      // the next slot, read ahead
                const int fin = (s == 0 ? last[0] : imax(last[s], arrived + cf[s > 0 ? s - 1 : 0])) + t_f_s;
                last[s] = valid ? fin : last[s];
                if (s == 0) {
                    if (valid && S > 1) *p = fin;
                } else if (s < S - 1) {
                    *p = valid ? fin : arrived;
                }
                p += 64;
                arrived = arrived_next;
            }
        }
        int b = 0;                                       // the ring slot of micro-batch r (r mod D)
        for (int r = 0; r < M; ++r) {
            if (r == 0) {
                // round 0's forwards were the last of the fill phase
            } else if constexpr (AHEAD) {                // forward sweep, ring reads three stages ahead
                constexpr int kAhead = S - 1 < 3 ? S - 1 : 3;
                int *slot_of[S];
                int ahead[S];
                auto ring_slot = [&](int s) {
                    unsigned slot = ((wpk[s / 4] >> (8 * (s % 4))) & 0xffu) + (unsigned)b;
                    slot = slot < slot - (unsigned)D ? slot : slot - (unsigned)D;      // mod D (w < D, b < D)
                    return ring + slot * 64;
                };
#pragma unroll
                for (int s = 1; s <= kAhead; ++s) {
                    slot_of[s] = ring_slot(s);
                    ahead[s] = *slot_of[s];
                }
                int fin_before = 0;
#pragma unroll
                for (int h = 0; h < S; h += kTimesBlock) {
                    const ConstInt *tf = (const ConstInt *)kargs()->tpad + h;
#pragma unroll
                    for (int j = 0; j < kTimesBlock && h + j < S; ++j) {
                        const int s = h + j;
                        if (s >= 1 && s + kAhead < S) {
                            slot_of[s + kAhead] = ring_slot(s + kAhead);
                            ahead[s + kAhead] = *slot_of[s + kAhead];
                        }
                        const int ws = (int)((wpk[s / 4] >> (8 * (s % 4))) & 0xffu);
                        const bool valid = (unsigned)(ws + r) < (unsigned)M;
                        int t_f_s;
                        if constexpr (VT) t_f_s = tfv[s];
                        else t_f_s = tf[j];
                        int fin;
                        if (s == 0) {
                            slot_of[0] = ring_slot(0);
                            fin = last[0] + t_f_s;
                        } else {
                            // w does not change over the rounds, and up to 32 stages the compiler keeps
                            // the S lane masks of this comparison in scalar registers (one instruction
                            // less per stage and round); at 64 stages they would not fit, so there the
                            // comparison is made afresh each time.
                            unsigned w4_before = wpk[(s - 1) / 4];
                            if constexpr (S >= 64) asm volatile("" : "+v"(w4_before));
                            const int ws_before = (int)((w4_before >> (8 * ((s - 1) % 4))) & 0xffu);
                            const int arrived = ws == ws_before ? fin_before : ahead[s];
                            fin = imax(last[s], arrived + cf[s - 1]) + t_f_s;
                        }
                        last[s] = valid ? fin : last[s];
                        if (s < S - 1) *slot_of[s] = fin;
                        fin_before = fin;
                    }
                }
            } else {
#pragma unroll
            for (int h = 0; h < S; h += kTimesBlock) {   // forward sweep
                const ConstInt *tf = (const ConstInt *)kargs()->tpad + h;      // scalar loads             // load this block's times here, not before the loops
#pragma unroll
                for (int j = 0; j < kTimesBlock && h + j < S; ++j) {
                    const int s = h + j;
                    const int ws = (int)((wpk[s / 4] >> (8 * (s % 4))) & 0xffu);
                    const bool valid = (unsigned)(ws + r) < (unsigned)M;
                    unsigned slot = (unsigned)(ws + b);
                    slot = slot < slot - (unsigned)D ? slot : slot - (unsigned)D;      // mod D (w < D, b < D)
                    int *const p = ring + slot * 64;
                    int t_f_s;
                    if constexpr (VT) t_f_s = tfv[s];
                    else t_f_s = tf[j];
                    int fin;
                    if (s == 0) fin = last[0] + t_f_s;
                    else fin = imax(last[s], *p + cf[s - 1]) + t_f_s;
                    last[s] = valid ? fin : last[s];
                    if (s < S - 1) *p = fin;
                }
            }
            }
            if (r >= 0) {                                // backward sweep
                __builtin_amdgcn_s_setprio(kPrioBackward);
                int carry = 0;
#pragma unroll
                for (int h = (S - 1) / kTimesBlock * kTimesBlock; h >= 0; h -= kTimesBlock) {
                    const ConstInt *tb = (const ConstInt *)kargs()->tpad + 64 + h;
#pragma unroll
                    for (int j = kTimesBlock - 1; j >= 0; --j) {
                        const int s = h + j;
                        if (s > S - 1) continue;
                        int t_b_s;
                        if constexpr (VT) t_b_s = tbv[s];
                        else t_b_s = tb[j];
                        const int arrive = s == S - 1 ? 0 : carry + cb[s < S - 1 ? s : 0];
                        last[s] = imax(last[s], arrive) + t_b_s;
                        carry = last[s];
                    }
                }
            }
            __builtin_amdgcn_s_setprio(kPrioForward);
            b = b + 1 == D ? 0 : b + 1;
        }
        const int mk = last[0];                          // B(0, M-1) is the last op of all
        unsigned long long key = kNoKey;
        if (run) {
            if (BEST) {
                key = ((unsigned long long)(unsigned)mk << 32) | (unsigned)c;
                if (kargs()->hist) {
                    for (int s = 0; s < kargs()->S; ++s) {
                        const int tau_s = kargs()->tfs ? kargs()->tfs[(long long)s * kargs()->Kin + kin] + kargs()->tbs[(long long)s * kargs()->Kin + kin]
                                                : kargs()->t_f[s] + kargs()->t_b[s];
                        int bin = (mk - M * tau_s) >> kargs()->hist_shift;
                        bin = bin > kargs()->hist_bins - 1 ? kargs()->hist_bins - 1 : bin;
                        atomicAdd(&kargs()->hist[s * kargs()->hist_bins + bin], 1ull);
                    }
                }
            } else {
                kargs()->mk_t[c * kargs()->K + k] = mk;        // transposed and completed by k_eval_epilogue
            }
        }
        if (BEST) {
            if (kargs()->pair_div) {
                if (key != kNoKey) atomicMin(&kargs()->keys[k], key);
            } else {
                key = wave_min_u64(key);
                if (lane == 0 && key != kNoKey) atomicMin(&kargs()->keys[k], key);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Hot kernel: lane = scenario, the candidate (hence the whole op order, every ring index
// and every branch) is uniform across the wavefront and lives in SGPRs.
//
// Shifted times.  Let a[s] = sum_{j<=s} t_f[j] + sum_{l<s} c_fwd[l], the earliest possible
// finish of F(s,0).  Each stage keeps one register
//     L[s] = (finish of its last forward, or start of its last backward) - a[s].
// In these coordinates the dependency rules of Section 3.1 become
//     forward  after a forward :  L[s] = max(L[s] + t_f[s],           R[m])
//     forward  after a backward:  L[s] = max(L[s] + t_f[s] + t_b[s],  R[m])
//     backward after a forward :  L[s] = max(L[s],                    carry + q[s])
//     backward after a backward:  L[s] = max(L[s] + t_b[s],           carry + q[s])
// with R[m] the shifted finish of micro-batch m's forward on stage s-1 (read from, and
// written back to, LDS slot m mod D), carry = L[s+1] after its backward, and
//     q[s] = c_fwd[s] + c_bwd[s] + t_f[s+1] + t_b[s+1]      (one VGPR per link and lane).
// Forward delays and forward durations are folded into a[s], backward durations into the
// next op's addend, so the steady state costs two integer VALU ops per resolved op.
// At the end  makespan = finish of B(0, M-1) = L[0] + t_f[0] + t_b[0].
//
// LDS ring: at round r the forwards in flight between stages are micro-batches
// w[S-1] + r < m <= w[0] + r, one value each, so D >= w[0] + 1 slots of 64 lanes suffice;
// slot-major layout [slot][lane] keeps every access conflict-free.  The reads are software
// pipelined: each is issued several stages (or, for the first stages, a whole backward
// sweep) ahead of its use, so the LDS latency does not stall every stage.
//
// Blocks per CU: what the LDS rings allow.  With per-scenario stage times (VT) the S addends
// are per lane and the 32-stage size needs about 150 VGPRs; held to 128 it spills 32 of them,
// but only in the code between the three phases -- the loop over the steady rounds touches no
// scratch memory -- and four wavefronts per SIMD instead of three are worth 23 % (16 stages:
// six blocks instead of five, 6 %).
template <int S, bool BEST, bool VT>
__global__ __launch_bounds__(kBlock, S >= 32 ? ADAPTRA_WAVES32 : 6) void k_resolve_scen_lanes(KArgs) {
    // The arguments are read through kargs() where they are needed (see there), never
    // through the by-value parameter.
    extern __shared__ int lds[];
    constexpr int kPD = S - 1 < kPrefetchStages ? S - 1 : kPrefetchStages;
    const int lane = threadIdx.x & 63;
    const int wv = uni(threadIdx.x >> 6);
    const unsigned ring_bytes = (unsigned)kargs()->ring_slots * 256u;
    const unsigned bias = 0u - ring_bytes;                 // ring offsets live in [bias, 2^32)
    // LDS byte address of this lane's column of the wave's ring, plus ring_bytes (un-bias)
    const unsigned ring = (unsigned)(size_t)(lds_int *)lds + (unsigned)wv * ring_bytes + (unsigned)lane * 4u + ring_bytes;
    unsigned *const hist_lds = (unsigned *)((char *)lds + kWavesPerBlock * ring_bytes);
    // S is the kernel's stage count; a pipeline with fewer stages is padded at its end
    // with stages of zero duration behind links of zero delay and with w = 0.  Such a stage
    // finishes F(m) the moment the stage before it does and starts B(m) at once, so the last
    // real stage sees exactly its own rule (B after its own F) and no time changes.  The real
    // count is kargs()->S.
    const bool lds_hist = BEST && kargs()->hist && kargs()->hist_in_lds;
    if (lds_hist) {
        const int n = kargs()->S * kargs()->hist_bins;
        for (int i = threadIdx.x; i < n; i += kBlock) hist_lds[i] = 0;
        __syncthreads();
    }

    const long long task = (long long)blockIdx.x * kWavesPerBlock + wv;
    const int tile = (int)(task % kargs()->n_ktiles);
    const long long c0 = (task / kargs()->n_ktiles) * kargs()->chunk;
    if (c0 < kargs()->C) {
        const long long K = kargs()->K;
        const long long k = (long long)tile * 64 + lane;
        const bool kvalid = k < K;
        const long long kk = kvalid ? k : K - 1;
        const long long Kin = kargs()->Kin;
        const long long kin = kk % Kin;              // scenario in the input arrays
        const int link_up = (int)(kk / Kin) - 1;     // link whose delay this copy raises, or -1
        // t_f and t_b of the stages share one VGPR each (lane s holds stage s); the addend a
        // stage currently needs is kept in an SGPR (add_f below) and switched with v_readlane
        // when the stage changes phase.
        // With per-scenario stage times (VT: compute stragglers) every lane has its own t_f and
        // t_b; they are then re-read from memory at the phase switches and add_f is per lane.
        const int tf_lanes = VT || lane >= kargs()->S ? 0 : kargs()->t_f[lane];
        const int tb_lanes = VT || lane >= kargs()->S ? 0 : kargs()->t_b[lane];
#define ADAPTRA_TF(s) (VT ? ((s) < kargs()->S ? kargs()->tfs[(s) * kargs()->Kin + kin] : 0) : __builtin_amdgcn_readlane(tf_lanes, (s)))
#define ADAPTRA_TB(s) (VT ? ((s) < kargs()->S ? kargs()->tbs[(s) * kargs()->Kin + kin] : 0) : __builtin_amdgcn_readlane(tb_lanes, (s)))
        const int tau0 = VT ? kargs()->tfs[kin] + kargs()->tbs[kin] : uni(kargs()->t_f[0]) + uni(kargs()->t_b[0]);
        int q[S > 1 ? S - 1 : 1];
        {
            const int *cf = kargs()->cf, *cb = kargs()->cb;
#pragma unroll
            for (int s = 0; s + 1 < S; ++s) {
                if (s + 1 < kargs()->S) {
                    int tau_next;
                    if constexpr (VT) tau_next = kargs()->tfs[(s + 1) * Kin + kin] + kargs()->tbs[(s + 1) * Kin + kin];
                    else tau_next = uni(kargs()->t_f[s + 1]) + uni(kargs()->t_b[s + 1]);
                    q[s] = cf[s * Kin + kin] + cb[s * Kin + kin] + tau_next + (s == link_up ? kargs()->sens_delta : 0);
                } else {
                    q[s] = 0;
                }
            }
        }

        unsigned long long key = kNoKey;
        const long long c_left = kargs()->C - c0;
        const int chunk = kargs()->chunk;
        const int c_end = (int)(c_left < chunk ? c_left : chunk);
        // Direct output (evaluation, chunks of exactly 16 candidates, a single launch): the
        // makespans of the chunk are kept per lane and written at its end, 16 consecutive
        // candidates = 64 contiguous bytes per scenario and output plane, so that the separate
        // streaming pass over all pairs is not needed and the writes hide under the VALU work.
        int mk_chunk[kChunk];
#pragma unroll
        for (int j = 0; j < kChunk; ++j) mk_chunk[j] = INT32_MAX;    // dead candidates keep the sentinel
        __builtin_amdgcn_s_setprio(kPrioForward);
        for (int ci = 0; ci < c_end; ++ci) {
            const long long c = c0 + ci;
            {
                const int cls = uni(kargs()->cand_class[c]);
                if (cls < kargs()->cls_lo || cls > kargs()->cls_hi) continue;
                if (BEST && uni(kargs()->cand_flag[c]) != ADAPTRA_FLAG_FEASIBLE) continue;
            }
            // w of the candidate: lane s holds w[s] (fetched with v_readlane where a stage's
            // own value is needed).  zmask, bit s: stages s-1 and s share w (slack 0).
            const int wq_lanes = kargs()->cand_wq[c * kargs()->wq_stride + (lane < S ? lane : 0)];
            const int W = __builtin_amdgcn_readlane(wq_lanes, 0);
            const int M = kargs()->M;
            const int wq_prev = __shfl_up(wq_lanes, 1);   // all lanes take part: not under the &&
            const unsigned long long zmask = __ballot(lane >= 1 && lane < S && wq_prev == wq_lanes);
            int L[S], x[S];
            unsigned soff[S];     // biased ring offset of the stage's next forward micro-batch
            int add_f[S];         // what the stage's next op adds to L[s]: t_f while the pipeline
                                  // fills, t_f + t_b in steady state, t_b once out of forwards
#pragma unroll
            for (int s = 0; s < S; ++s) {
                L[s] = kNeg;
                x[s] = 0;
                soff[s] = bias;   // micro-batch 0 sits in slot 0
                add_f[s] = ADAPTRA_TF(s);
            }
            L[0] = -add_f[0];

// One forward step of stage s.  x[s] is the value micro-batch m got on stage s-1, read from
// ring slot m mod D some stages earlier; if the two stages have equal w that value is only
// being produced in this very round and comes from L[s-1] instead.  The result goes to slot
// m and the stage's offset moves on to slot m+1.
#define ADAPTRA_F_OP(s, e)                                                      \
    do {                                                                        \
        const unsigned slot = ring + soff[s];                                   \
        if constexpr ((s) == 0) {                                               \
            L[0] += (e);                                                        \
            soff[0] = ring_next(soff[0], bias);                                 \
        } else {                                                                \
            const int t = L[s] + (e);                                           \
            L[s] = imax(t, select_by_bit_and_advance<(s)>(zmask, x[s], L[(s) > 0 ? (s) - 1 : 0], \
                                                          soff[s], bias));      \
        }                                                                       \
        if constexpr ((s) < S - 1) *(lds_int *)slot = L[s];                     \
    } while (0)
// Reads run kPD stages ahead of their use: stage s issues the read of stage s+kPD ...
#define ADAPTRA_READ_AHEAD(s)                                                   \
    do {                                                                        \
        if constexpr ((s) + kPD <= S - 1)                                       \
            x[(s) + kPD <= S - 1 ? (s) + kPD : 0] =                             \
                *(lds_int *)(ring + soff[(s) + kPD <= S - 1 ? (s) + kPD : 0]);  \
    } while (0)
// ... and the reads of stages 1..kPD for the next round are issued at the end of the
// forward sweep, so that they complete under the backward sweep.
#define ADAPTRA_READ_NEXT_ROUND()                                               \
    stages_up<1, kPD + 1>(ADAPTRA_STAGE_LAMBDA(sj) {                            \
        constexpr int j = decltype(sj)::value;                                  \
        x[j] = *(lds_int *)(ring + soff[j]);                                    \
    })
#define ADAPTRA_B_SWEEP()                                                       \
    do {                                                                        \
        __builtin_amdgcn_s_setprio(kPrioBackward);                              \
        int carry = L[S - 1];                                                   \
        stages_down<S - 2, 0>(ADAPTRA_STAGE_LAMBDA(si) {                        \
            constexpr int s = decltype(si)::value;                              \
            L[s] = imax(L[s], carry + q[s]);                                    \
            carry = L[s];                                                       \
        });                                                                     \
        __builtin_amdgcn_s_setprio(kPrioForward);                               \
    } while (0)

            // warm-up rounds r = -W .. 0: forwards only, each after a forward; stage s takes part
            // once w[s] + r >= 0, i.e. with its micro-batches 0 .. w[s].
            // They are taken stage by stage rather than round by round: stage s runs its
            // w[s] + 1 forwards back to back.  Everything they wait for is there -- the stage
            // before has run at least as many (w is non-increasing) -- so a link without slack
            // needs no special case here, the ring is read four micro-batches at a time ahead of
            // their use, no stage is tested for having started, and the ring ends up exactly as
            // after the rounds (micro-batch m in slot m, left by the last stage that ran it; no
            // slot index wraps, since w[0] + 1 <= D).
            stages_up<0, S>(ADAPTRA_STAGE_LAMBDA(si) {
                constexpr int s = decltype(si)::value;
                const int n = __builtin_amdgcn_readlane(wq_lanes, s) + 1;
                unsigned at = ring + bias;                        // slot 0 of this lane
                int i = 0;
                for (; i + 4 <= n; i += 4) {
                    int from_before[4];
                    if constexpr (s > 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) from_before[j] = *(lds_int *)(at + 256u * j);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        L[s] += add_f[s];
                        if constexpr (s > 0) L[s] = imax(L[s], from_before[j]);
                        if constexpr (s < S - 1) *(lds_int *)(at + 256u * j) = L[s];
                    }
                    at += 1024u;
                }
                for (; i < n; ++i) {
                    L[s] += add_f[s];
                    if constexpr (s > 0) L[s] = imax(L[s], *(lds_int *)at);
                    if constexpr (s < S - 1) *(lds_int *)at = L[s];
                    at += 256u;
                }
                // the stage's next micro-batch: slot n, or slot 0 again if the ring has just n slots
                const unsigned next = bias + 256u * (unsigned)n;     // 0 = one past the last slot
                soff[s] = next == 0u ? bias : next;
            });
            ADAPTRA_READ_NEXT_ROUND();
            ADAPTRA_B_SWEEP();                    // B(s, 0): each after a forward
#pragma unroll
            for (int s = 0; s < S; ++s) add_f[s] += ADAPTRA_TB(s);
            // steady rounds r = 1 .. M-1-W: F after B, B after F on every stage
            for (int r = M - 1 - W; r > 0; --r) {
                stages_up<0, S>(ADAPTRA_STAGE_LAMBDA(si) {
                    constexpr int s = decltype(si)::value;
                    ADAPTRA_F_OP(s, add_f[s]);
                    ADAPTRA_READ_AHEAD(s);
                });
                ADAPTRA_READ_NEXT_ROUND();
                ADAPTRA_B_SWEEP();
            }
            // cool-down rounds r = M-W .. M-1: stage s is out of forwards once
            // w[s] + r > M-1, which holds for the stages 0 .. done-1.
            {
                int done = 0;
                for (int r = M - W; r <= M - 1; ++r) {
                    const int done_before = done;
                    while (done < S && __builtin_amdgcn_readlane(wq_lanes, done) + r > M - 1) ++done;
                    stages_up<0, S>(ADAPTRA_STAGE_LAMBDA(si) {
                        constexpr int s = decltype(si)::value;
                        if (s >= done) ADAPTRA_F_OP(s, add_f[s]);
                        ADAPTRA_READ_AHEAD(s);
                    });
                    ADAPTRA_READ_NEXT_ROUND();
                    if constexpr (!VT) {
                        // The stages out of forwards run B after B: their backward duration is
                        // added first (independent adds, the sweep over them ends at `done`),
                        // then the backward sweep is the steady one, without a test per stage.
                        stages_below<0, S>(done, ADAPTRA_STAGE_LAMBDA(si) {
                            constexpr int s = decltype(si)::value;
                            L[s] += ADAPTRA_TB(s);
                        });
                        ADAPTRA_B_SWEEP();
                        continue;
                    }
                    int carry = 0;
                    __builtin_amdgcn_s_setprio(kPrioBackward);
                    stages_down<S - 1, 0>(ADAPTRA_STAGE_LAMBDA(si) {
                        constexpr int s = decltype(si)::value;
                        int prev = L[s];
                        if (s < done) {                                   // B after B
                            if (s >= done_before) add_f[s] -= ADAPTRA_TF(s);
                            prev += add_f[s];
                        }
                        L[s] = (s == S - 1) ? prev : imax(prev, carry + q[s < S - 1 ? s : 0]);
                        carry = L[s];
                    });
                    __builtin_amdgcn_s_setprio(kPrioForward);
                }
            }
#undef ADAPTRA_F_OP
#undef ADAPTRA_READ_AHEAD
#undef ADAPTRA_READ_NEXT_ROUND
#undef ADAPTRA_B_SWEEP

            const int mk = L[0] + tau0;
            if (BEST) {
                if (kvalid) {
                    const unsigned long long cand = ((unsigned long long)(unsigned)mk << 32) | (unsigned)c;
                    key = cand < key ? cand : key;
                    if (kargs()->hist) {
                        const int bins = kargs()->hist_bins, shift = kargs()->hist_shift;
                        unsigned long long *const hist = kargs()->hist;
                        for (int s = 0; s < kargs()->S; ++s) {
                            const int tau_s = ADAPTRA_TF(s) + ADAPTRA_TB(s);
                            int b = (mk - M * tau_s) >> shift;
                            b = b > bins - 1 ? bins - 1 : b;
                            if (lds_hist) hist_count(hist_lds + s * bins, b, lane);
                            else hist_count(hist + s * bins, b, lane);
                        }
                    }
                }
            } else if (kvalid) {
                // candidate-major scratch: the 64 lanes write 256 contiguous bytes;
                // k_eval_epilogue transposes into out_makespan and adds bubbles and flags
                kargs()->mk_t[c * K + k] = mk;
            }
            if constexpr (!BEST) {
#pragma unroll
                for (int j = 0; j < kChunk; ++j)
                    if (j == ci) mk_chunk[j] = mk;           // uniform ci: a select per register
            }
        }
        if (BEST && kvalid && key != kNoKey) atomicMin(&kargs()->keys[k], key);
        if constexpr (!BEST) {
            if (kargs()->direct_out && kvalid) {
                const long long C = kargs()->C, P = C * K;
                const long long at = k * C + c0;                 // 16 candidates from here
                int4 *const mko = (int4 *)(kargs()->out_makespan + at);
#pragma unroll
                for (int v = 0; v < kChunk / 4; ++v)
                    mko[v] = make_int4(mk_chunk[4 * v], mk_chunk[4 * v + 1], mk_chunk[4 * v + 2], mk_chunk[4 * v + 3]);
                *(uint4 *)(kargs()->out_feasible + at) = *(const uint4 *)(kargs()->cand_flag + c0);
                if (kargs()->out_bubble) {
                    const int M = kargs()->M;
                    for (int s = 0; s < kargs()->S; ++s) {
                        const int busy = M * (ADAPTRA_TF(s) + ADAPTRA_TB(s));
                        int4 *const bo = (int4 *)(kargs()->out_bubble + (long long)s * P + at);
#pragma unroll
                        for (int v = 0; v < kChunk / 4; ++v) {
                            int b4[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int mkj = mk_chunk[4 * v + j];
                                b4[j] = mkj == INT32_MAX ? INT32_MAX : mkj - busy;
                            }
                            bo[v] = make_int4(b4[0], b4[1], b4[2], b4[3]);
                        }
                    }
                }
            }
        }
    }
    if (lds_hist) {
        __syncthreads();
        const int n = kargs()->S * kargs()->hist_bins;
        unsigned long long *const hist = kargs()->hist;
        for (int i = threadIdx.x; i < n; i += kBlock) {
            const unsigned cnt = hist_lds[i];
            if (cnt) atomicAdd(&hist[i], (unsigned long long)cnt);
        }
    }
}
#undef ADAPTRA_TF
#undef ADAPTRA_TB

// ---------------------------------------------------------------------------------------
// status[0] = number of negative entries, status[1] = max time, status[2] = max delay
__global__ __launch_bounds__(kBlock) void k_check_inputs(KArgs a) {
    const long long nw = (long long)a.S * a.C;
    const long long nc = (long long)(a.S - 1) * a.K;
    const long long nts = a.tfs ? (long long)a.S * a.K : 0;
    const long long n = nw + 2 * nc + 2 * a.S + 2 * nts;
    const long long stride = (long long)gridDim.x * kBlock;
    int neg = 0, maxt = 0, maxc = 0;
    for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        if (i < nw) {
            neg += a.w[i] < 0;
        } else if (i < nw + nc) {
            const int v = a.cf[i - nw];
            neg += v < 0;
            maxc = imax(maxc, v);
        } else if (i < nw + 2 * nc) {
            const int v = a.cb[i - nw - nc];
            neg += v < 0;
            maxc = imax(maxc, v);
        } else if (i < nw + 2 * nc + 2 * a.S) {
            const long long j = i - nw - 2 * nc;
            const int v = j < a.S ? a.t_f[j] : a.t_b[j - a.S];
            neg += v < 0;
            maxt = imax(maxt, v);
        } else {
            const long long j = i - nw - 2 * nc - 2 * a.S;
            const int v = j < nts ? a.tfs[j] : a.tbs[j - nts];
            neg += v < 0;
            maxt = imax(maxt, v);
        }
    }
    if (neg) atomicAdd(&a.status[0], neg);
    if (maxt) atomicMax(&a.status[1], maxt);
    if (maxc) atomicMax(&a.status[2], maxc);
}

__global__ void k_zero_status(KArgs a) {
    a.status[threadIdx.x] = 0;      // launched with 64 threads: all of status
}

// ---------------------------------------------------------------------------------------
// The paper's analytic planning, one thread per scenario (Section 4.2).
//   Algorithm 1 (initial planning, scenario independent; thread 0 only): x_0 = x_max, the
//     slack x_max - 1 spread over the S - 1 links as evenly as possible, x_{S-1} = 1.
//   Algorithm 2 (dynamic adaptation): x_{S-1} = 1, and from the last link backwards
//     Delta_i = min(M - 2S, max(ceil((t_f[i] + t_b[i] + c_fwd[i] + c_bwd[i]) / (t_f[i+1] + t_b[i+1])), 2)),
//     floored at 0 (Lemma 1), x_i = min(x_{i+1} + Delta_i, M); a zero denominator lets the clip decide.
//   Eq. (1) for the schedule w_cur: link i absorbs its delay iff
//     t_f[i] + t_b[i] + c_fwd[i] + c_bwd[i] <= (w_cur[i] - w_cur[i+1]) (t_f[i+1] + t_b[i+1]).
// Outputs are w = x - 1.
struct SeedArgs {
    int S, M, x_max;
    long long K;
    const int *t_f, *t_b, *cf, *cb, *w_cur, *tfs, *tbs;
    int *w_init, *w_adapted;
    unsigned char *not_absorbed;
};

__global__ __launch_bounds__(kBlock) void k_seed(SeedArgs a) {
    const long long k = (long long)blockIdx.x * kBlock + threadIdx.x;
    const int S = a.S;
    if (k == 0 && a.w_init) {
        int x = a.x_max;
        a.w_init[0] = x - 1;
        if (S > 1) {
            const int avg = (a.x_max - 1) / (S - 1), r = (a.x_max - 1) % (S - 1);
            for (int i = 1; i < S; ++i) {
                x -= (i <= r) ? avg + 1 : avg;
                a.w_init[i] = x - 1;
            }
        }
    }
    if (k >= a.K) return;
    auto tau = [&](int i) -> long long {       // t_f + t_b of stage i as this scenario sees it
        return a.tfs ? (long long)a.tfs[(long long)i * a.K + k] + a.tbs[(long long)i * a.K + k]
                     : (long long)a.t_f[i] + a.t_b[i];
    };
    // One pass over the links, last to first, serves both outputs: the delays are read once.
    int x = 1;
    if (a.w_adapted) a.w_adapted[(long long)(S - 1) * a.K + k] = 0;
    const int clip = a.M - 2 * S;
    long long tau_next = S > 1 ? tau(S - 1) : 0;
    for (int i = S - 2; i >= 0; --i) {
        const long long tau_i = tau(i);
        const long long num = tau_i + a.cf[(long long)i * a.K + k] + a.cb[(long long)i * a.K + k];
        const long long den = tau_next;
        if (a.w_adapted) {
            long long d = clip;
            if (den != 0) {
                // ceil(num / den); both are sums of non-negative int32 values, and whenever they fit
                // 32 bits (always, under adaptra_check_inputs' bound) a 32-bit division does
                const long long up = num + den - 1;
                long long ratio = ((unsigned long long)(up | den) >> 32) == 0 ? (long long)((unsigned)up / (unsigned)den) : up / den;
                if (ratio < 2) ratio = 2;
                if (ratio < d) d = ratio;
            }
            if (d < 0) d = 0;
            const long long nx = x + d;
            x = nx > a.M ? a.M : (int)nx;
            a.w_adapted[(long long)i * a.K + k] = x - 1;
        }
        if (a.not_absorbed) {
            const long long rhs = ((long long)a.w_cur[i] - a.w_cur[i + 1]) * den;
            a.not_absorbed[(long long)i * a.K + k] = num <= rhs ? 0 : 1;
        }
        tau_next = tau_i;
    }
}

// ---------------------------------------------------------------------------------------
// Measurement aid: sustained rate of the two integer VALU ops the recurrence is made of.
// Every lane runs 8 independent chains of  v = max(v + c, d)  (one v_add_u32, one
// v_max_i32 each), 8 x 2 x 32 ops per loop trip, so neither latency nor memory limits it.
__global__ __launch_bounds__(kBlock) void k_valu_probe(int iters, int c, int d, int *out) {
    int v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = threadIdx.x + j;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 32; ++u) {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = imax(v[j] + c, d + j);
        }
    }
    int r = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) r ^= v[j];
    if (r == 0x7fffffff) out[0] = r;          // practically never: keeps the chains alive
}

// ---------------------------------------------------------------------------------------
// Host side
thread_local int g_last_hip_error = 0;
int g_kernel_mode = 0;
hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;


// The hot kernel exists for 2, 4, 8, 16 and 32 stages; a pipeline with another stage count
// up to 32 runs in the next larger one, padded with stages that take no time (see the
// kernel).  0: no hot kernel (more than 32 stages).
int hot_kernel_stages(int S) {
    for (int p = 2; p <= 32; p *= 2)
        if (S <= p) return p;
    return 0;
}
// The candidate-lanes kernel has one size more: per-lane state in VGPRs (last, c_fwd, c_bwd:
// 3 S registers) still fits at 64 stages with two wavefronts per SIMD, which the scenario-lanes
// kernel's per-stage scalars (2 S SGPRs) do not.
int cand_kernel_stages(int S) {
    for (int p = 2; p <= 64; p *= 2)
        if (S <= p) return p;
    return 0;
}

struct Workspace {
    size_t off_flag, off_class, off_wq, off_keys, off_status, off_tpad, off_scratch, off_mkt, total;
    int wq_stride;
    long long general_threads;
};

// The general kernel keeps (2 S + M) ints per thread in scratch; bound the scratch to
// about 256 MiB by limiting the number of resident threads.
long long general_thread_count(int S, int M) {
    const long long per_thread = (2ll * S + M) * 4;
    long long nt = (256ll << 20) / per_thread;
    if (nt > 65536) nt = 65536;
    if (nt < 4096) nt = 4096;
    return nt / kBlock * kBlock;
}

bool plan_workspace(int S, int M, long long C, long long K, Workspace *ws, bool with_mkt = true) {
    if (S < 1 || S > ADAPTRA_MAX_STAGES || M < 1 || M > ADAPTRA_MAX_MICROBATCHES) return false;
    if (C < 1 || C > INT32_MAX || K < 1 || K > INT32_MAX) return false;
    ws->wq_stride = (cand_kernel_stages(S) + 3) & ~3;
    ws->general_threads = general_thread_count(S, M);
    size_t o = 0;
    ws->off_flag = o;    o += adaptra_detail::align256((size_t)C);
    ws->off_class = o;   o += adaptra_detail::align256((size_t)C);
    ws->off_wq = o;      o += adaptra_detail::align256((size_t)C * ws->wq_stride);
    ws->off_keys = o;    o += adaptra_detail::align256((size_t)K * 8);
    ws->off_status = o;  o += 256;
    ws->off_tpad = o;    o += 512;
    ws->off_scratch = o; o += adaptra_detail::align256((size_t)ws->general_threads * (2 * S + M) * 4);
    ws->off_mkt = o;     o += with_mkt ? adaptra_detail::align256((size_t)C * (size_t)K * 4) : 0;   // last: the search needs none
    ws->total = o;
    return true;
}


// Which of the two on-chip kernels runs (the general kernel takes what neither can: warm-ups
// deeper than the ring, per-scenario stage times at too many stages); from 33 to 64 stages only
// the candidate-lanes kernel has a size.  The scenario-lanes kernel spends 6 VALU ops per
// stage and round on 64 scenarios whether or not all 64 lanes carry one; the candidate-lanes
// kernel spends 15 (13 in its plain form) on 64 pairs.  Measured at 16 and 32 stages they cross
// at about 33 scenarios on 65 536 candidates and at about 48 on 8 192, where the scenario-lanes
// kernel works through one candidate per wavefront and its set-up per scenario is not spread
// over a chunk.  The candidate-lanes kernel is also the only one for the search's paired form.
// With per-scenario stage times it keeps 5 S values per lane in registers (two wavefronts per
// SIMD from 16 stages on) and has no 64-stage size; where it is missing the scenario-lanes
// kernel wins from 6 scenarios against the general one.
enum ResolveKernel { kScenarioLanes, kCandidateLanes, kGeneralOnly };
ResolveKernel choose_kernel(int S, long long K, long long C, bool stage_times, bool paired) {
    const bool scen_ok = hot_kernel_stages(S) != 0 && !paired;
    const bool cand_ok = cand_kernel_stages(S) != 0 && !(stage_times && cand_kernel_stages(S) >= 64);
    switch (g_kernel_mode) {
        case 1: return kGeneralOnly;
        case 2: return scen_ok ? kScenarioLanes : kGeneralOnly;
        case 3:
        case 4: return cand_ok ? kCandidateLanes : kGeneralOnly;
        default: break;
    }
    const long long scen_from = C >= 32768 ? 33 : 48;          // the measured crossover
    if (scen_ok && (K >= scen_from || (!cand_ok && K >= 6))) return kScenarioLanes;
    if (cand_ok) return kCandidateLanes;
    return kGeneralOnly;
}

int hip_fail(hipError_t e) { return adaptra_detail::hip_fail(e); }

#define ADAPTRA_LAUNCH_CHECK()                          \
    do {                                                \
        hipError_t e_ = hipGetLastError();              \
        if (e_ != hipSuccess) return hip_fail(e_);      \
    } while (0)

int grid_for(long long n, long long cap = 1 << 20) {
    long long g = (n + kBlock - 1) / kBlock;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

int validate_common(const adaptra_params_t *p, const adaptra_candidates_t *cd,
                    const adaptra_scenarios_t *sc, void *workspace, size_t workspace_bytes,
                    Workspace *ws, bool with_mkt = true) {
    if (!p || !cd || !sc) return ADAPTRA_EINVAL;
    if (!plan_workspace(p->S, p->M, cd->n, sc->n, ws, with_mkt)) return ADAPTRA_EINVAL;
    if (!p->t_f || !p->t_b || !cd->w) return ADAPTRA_EINVAL;
    if (p->S > 1 && (!sc->c_fwd || !sc->c_bwd)) return ADAPTRA_EINVAL;
    if ((sc->t_f == nullptr) != (sc->t_b == nullptr)) return ADAPTRA_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ws->total) return ADAPTRA_EWORKSPACE;
    return ADAPTRA_OK;
}

void fill_args(KArgs *a, const adaptra_params_t *p, const adaptra_candidates_t *cd,
               const adaptra_scenarios_t *sc, void *workspace, const Workspace &ws) {
    *a = KArgs{};
    a->S = p->S; a->M = p->M;
    a->t_f = p->t_f; a->t_b = p->t_b; a->mem_cap = p->mem_cap;
    a->C = cd->n; a->K = sc->n; a->Kin = sc->n;
    a->w = cd->w; a->cf = sc->c_fwd; a->cb = sc->c_bwd;
    a->tfs = sc->t_f; a->tbs = sc->t_b;
    char *base = (char *)workspace;
    a->cand_flag = (unsigned char *)(base + ws.off_flag);
    a->cand_class = (unsigned char *)(base + ws.off_class);
    a->cand_wq = (unsigned char *)(base + ws.off_wq);
    a->wq_stride = ws.wq_stride;
    a->keys = (unsigned long long *)(base + ws.off_keys);
    a->status = (int *)(base + ws.off_status);
    a->tpad = (int *)(base + ws.off_tpad);
    a->scratch = (int *)(base + ws.off_scratch);
    a->mk_t = (int *)(base + ws.off_mkt);
    a->n_ktiles = (int)((sc->n + 63) / 64);
    // A wavefront of the hot kernel works through `chunk` candidates in a row, which amortises
    // its per-scenario set-up; a small problem takes shorter chunks so that there are still
    // enough wavefronts (about two per SIMD slot) to fill the chip.
    {
        const long long want_waves = 8192;
        long long chunk = cd->n * a->n_ktiles / want_waves;
        a->chunk = (int)(chunk < 1 ? 1 : (chunk > kChunk ? kChunk : chunk));
    }
    a->n_chunks = (cd->n + a->chunk - 1) / a->chunk;
}

// The ring classes a launch covers.  With a bound on w one launch takes every class up to the
// bound's, with exactly the ring the bound needs; without, five launches with rings of 8, 16,
// 32, 64 and 128 slots share the classes (empty ones exit at once).
struct ClassRange {
    int lo, hi;
};
int ring_launches(int w_bound, int M, ClassRange out[5]) {
    if (w_bound >= 0) {
        const int wb = w_bound > M - 1 ? M - 1 : w_bound;
        int last = (wb + 8) / 8 - 1;
        if (last > kNumRingClasses - 1) last = kNumRingClasses - 1;
        out[0] = {0, last};
        return 1;
    }
    out[0] = {0, 0}; out[1] = {1, 1}; out[2] = {2, 3}; out[3] = {4, 7}; out[4] = {8, kNumRingClasses - 1};
    return 5;
}

template <int S, bool BEST, bool VT>
int launch_scen_lanes_one(KArgs a, int w_bound, hipStream_t st) {
    const long long tasks = a.n_chunks * a.n_ktiles;
    const long long blocks = (tasks + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > INT32_MAX) return ADAPTRA_EINVAL;
    ClassRange ranges[5];
    const int n_launches = ring_launches(w_bound, a.M, ranges);
    for (int i = 0; i < n_launches; ++i) {
        a.cls_lo = ranges[i].lo;
        a.cls_hi = ranges[i].hi;
        a.ring_slots = 8 * (a.cls_hi + 1);
        size_t lds = (size_t)kWavesPerBlock * a.ring_slots * 256;
        if (BEST && a.hist && a.hist_in_lds) lds += (size_t)a.S * a.hist_bins * 4;
        if (lds > 48 * 1024) {      // above the default dynamic-LDS limit: raise it for this kernel
            hipError_t e = hipFuncSetAttribute((const void *)k_resolve_scen_lanes<S, BEST, VT>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return hip_fail(e);
        }
        hipLaunchKernelGGL((k_resolve_scen_lanes<S, BEST, VT>), dim3((unsigned)blocks), dim3(kBlock), lds, st, a);
        ADAPTRA_LAUNCH_CHECK();
    }
    return ADAPTRA_OK;
}

template <int S, bool BEST>
int launch_scen_lanes_sized(const KArgs &a, int w_bound, hipStream_t st) {
    return a.tfs ? launch_scen_lanes_one<S, BEST, true>(a, w_bound, st) : launch_scen_lanes_one<S, BEST, false>(a, w_bound, st);
}

template <bool BEST>
int launch_scen_lanes(const KArgs &a, int w_bound, hipStream_t st) {
    switch (hot_kernel_stages(a.S)) {
        case 2: return launch_scen_lanes_sized<2, BEST>(a, w_bound, st);
        case 4: return launch_scen_lanes_sized<4, BEST>(a, w_bound, st);
        case 8: return launch_scen_lanes_sized<8, BEST>(a, w_bound, st);
        case 16: return launch_scen_lanes_sized<16, BEST>(a, w_bound, st);
        case 32: return launch_scen_lanes_sized<32, BEST>(a, w_bound, st);
        default: return ADAPTRA_EINVAL;
    }
}

template <int S, bool BEST, bool VT, bool AHEAD>
int launch_cand_lanes_one(KArgs a, int w_bound, hipStream_t st) {
    const long long ntiles = (a.pair_div ? 1 : a.K) * ((a.C + 63) / 64);
    long long blocks = (ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;            // the tiles are walked in a loop
    ClassRange ranges[5];
    const int n_launches = ring_launches(w_bound, a.M, ranges);
    for (int i = 0; i < n_launches; ++i) {
        a.cls_lo = ranges[i].lo;
        a.cls_hi = ranges[i].hi;
        a.ring_slots = 8 * (a.cls_hi + 1);
        const size_t lds = (size_t)kWavesPerBlock * a.ring_slots * 256;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)k_resolve_cand_lanes<S, BEST, VT, AHEAD>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return hip_fail(e);
        }
        hipLaunchKernelGGL((k_resolve_cand_lanes<S, BEST, VT, AHEAD>), dim3((unsigned)blocks), dim3(kBlock), lds, st, a);
        ADAPTRA_LAUNCH_CHECK();
    }
    return ADAPTRA_OK;
}

template <bool BEST>
int launch_cand_lanes(const KArgs &a, int w_bound, hipStream_t st) {
    // The read-ahead form wherever it exists (kernel mode 3 asks for the plain one).
    const bool ahead = g_kernel_mode != 3;
#define ADAPTRA_CASE(S_)                                                                         \
    case S_:                                                                                     \
        if constexpr (S_ < 64) {      /* 5 S per-lane registers: not at 64 stages */             \
            if (a.tfs) return ahead ? launch_cand_lanes_one<S_, BEST, true, true>(a, w_bound, st)  \
                                    : launch_cand_lanes_one<S_, BEST, true, false>(a, w_bound, st); \
        }                                                                                        \
        return ahead ? launch_cand_lanes_one<S_, BEST, false, true>(a, w_bound, st)              \
                     : launch_cand_lanes_one<S_, BEST, false, false>(a, w_bound, st);
    switch (cand_kernel_stages(a.S)) {
        ADAPTRA_CASE(2) ADAPTRA_CASE(4) ADAPTRA_CASE(8) ADAPTRA_CASE(16) ADAPTRA_CASE(32) ADAPTRA_CASE(64)
        default: return ADAPTRA_EINVAL;
    }
#undef ADAPTRA_CASE
}

template <bool BEST>
int launch_general(KArgs a, const Workspace &ws, bool all, hipStream_t st) {
    a.general_all = all ? 1 : 0;
    const long long ntiles = (a.pair_div ? 1 : a.K) * ((a.C + 63) / 64);
    long long threads = ntiles * 64;
    if (threads > ws.general_threads) threads = ws.general_threads;
    const int blocks = (int)((threads + kBlock - 1) / kBlock);
    hipLaunchKernelGGL((k_resolve_general<BEST>), dim3(blocks), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

int record_event(hipEvent_t ev, hipStream_t st) {
    if (!g_ev_before || !g_ev_after) return ADAPTRA_OK;
    hipError_t e = hipEventRecord(ev, st);
    return e == hipSuccess ? ADAPTRA_OK : hip_fail(e);
}

// The measurement events bracket the kernel that carries the load: the on-chip
// kernel when it is in use, else the general kernel.
// direct (evaluation only, may be null): set to the highest ring class whose candidates got
// their final outputs straight from the scenario-lanes kernel, or to -1 if the caller's
// epilogue has to produce all of them.  The kernel does so when one launch covers its
// candidates, every chunk holds exactly 16 of them and the output addresses allow 16-byte
// stores; the epilogue is then needed only for tiles with candidates left to the general kernel.
template <bool BEST>
int launch_resolve(KArgs a, const Workspace &ws, int w_bound, hipStream_t st, int *direct = nullptr) {
    int rc;
    if (direct) *direct = -1;
    const ResolveKernel which = choose_kernel(a.S, a.K, a.C, a.tfs != nullptr, a.pair_div != 0);
    if (which != kGeneralOnly) {
        const bool hot = which == kScenarioLanes;
        a.cls_hi = kNumRingClasses - 1;
        if (w_bound >= 0) {
            const int wb = w_bound > a.M - 1 ? a.M - 1 : w_bound;
            const int hi = (wb + 8) / 8 - 1;
            if (hi < a.cls_hi) a.cls_hi = hi;
        }
        const int general_from = a.cls_hi;               // classes above it go to the general kernel
        const auto aligned16 = [](const void *p) { return ((uintptr_t)p & 15) == 0; };
        if (!BEST && direct && hot && w_bound >= 0 && a.chunk == kChunk && a.C % kChunk == 0 && a.Kin == a.K &&
            aligned16(a.out_makespan) && aligned16(a.out_feasible) && aligned16(a.out_bubble)) {
            a.direct_out = 1;
            *direct = general_from;
        }
        if ((rc = record_event(g_ev_before, st))) return rc;
        if ((rc = hot ? launch_scen_lanes<BEST>(a, w_bound, st) : launch_cand_lanes<BEST>(a, w_bound, st))) return rc;
        if ((rc = record_event(g_ev_after, st))) return rc;
        a.cls_hi = general_from;
        return launch_general<BEST>(a, ws, false, st);   // too deep for the ring, or beyond w_bound
    }
    if ((rc = record_event(g_ev_before, st))) return rc;
    if ((rc = launch_general<BEST>(a, ws, true, st))) return rc;
    return record_event(g_ev_after, st);
}

}  // namespace

int adaptra_detail::hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return ADAPTRA_EHIP;
}

extern "C" {

size_t adaptra_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen) {
    Workspace ws;
    if (!params || !plan_workspace(params->S, params->M, n_cand, n_scen, &ws)) return 0;
    return ws.total;
}

size_t adaptra_best_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen) {
    Workspace ws;
    if (!params || !plan_workspace(params->S, params->M, n_cand, n_scen, &ws, false)) return 0;
    return ws.total;
}

int adaptra_check_inputs(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                         const adaptra_scenarios_t *scens,
                         void *workspace, size_t workspace_bytes, void *stream) {
    Workspace ws;
    int rc = validate_common(params, cands, scens, workspace, workspace_bytes, &ws);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    KArgs a;
    fill_args(&a, params, cands, scens, workspace, ws);
    hipLaunchKernelGGL(k_zero_status, dim3(1), dim3(64), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    const long long n = (long long)a.S * a.C + 2ll * (a.S - 1) * a.K + 2 * a.S + (a.tfs ? 2ll * a.S * a.K : 0);
    hipLaunchKernelGGL(k_check_inputs, dim3(grid_for(n, 4096)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    int status[4] = {0, 0, 0, 0};
    hipError_t e = hipMemcpyAsync(status, a.status, sizeof(status), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    if (status[0] != 0) return ADAPTRA_ERANGE;
    const long long bound = 2ll * a.M * a.S * ((long long)status[1] + (long long)status[2]);
    if (bound >= (1ll << 31)) return ADAPTRA_EOVERFLOW;
    return ADAPTRA_OK;
}

int adaptra_eval(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                 const adaptra_scenarios_t *scens,
                 int32_t *out_makespan, int32_t *out_bubble, uint8_t *out_feasible,
                 void *workspace, size_t workspace_bytes, void *stream) {
    Workspace ws;
    int rc = validate_common(params, cands, scens, workspace, workspace_bytes, &ws);
    if (rc) return rc;
    if (!out_makespan || !out_feasible) return ADAPTRA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    KArgs a;
    fill_args(&a, params, cands, scens, workspace, ws);
    a.out_makespan = out_makespan;
    a.out_bubble = out_bubble;
    a.out_feasible = out_feasible;
    hipLaunchKernelGGL(k_zero_status, dim3(1), dim3(64), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_prepass, dim3(grid_for(a.C, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    int direct = -1;
    rc = launch_resolve<false>(a, ws, cands->w_bound, st, &direct);
    if (rc) return rc;
    const long long tiles = ((a.C + 63) / 64) * ((a.K + 63) / 64);
    if (tiles > INT32_MAX) return ADAPTRA_EINVAL;
    if (direct >= 0) { a.direct_out = 1; a.cls_hi = direct; }
    hipLaunchKernelGGL(k_eval_epilogue, dim3((unsigned)tiles), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

int adaptra_eval_best(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                      const adaptra_scenarios_t *scens,
                      int32_t *out_makespan, int32_t *out_bubble, uint8_t *out_feasible,
                      int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                      uint64_t *out_hist,
                      void *workspace, size_t workspace_bytes, void *stream) {
    Workspace ws;
    int rc = validate_common(params, cands, scens, workspace, workspace_bytes, &ws);
    if (rc) return rc;
    if (!out_makespan || !out_feasible || !out_best_idx || !out_best_makespan) return ADAPTRA_EINVAL;
    if (params->hist_bins < 0 || params->hist_bins > 65536) return ADAPTRA_EINVAL;
    if (params->hist_bins > 0 && (!out_hist || params->hist_shift < 0 || params->hist_shift > 30))
        return ADAPTRA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    KArgs a;
    fill_args(&a, params, cands, scens, workspace, ws);
    a.out_makespan = out_makespan;
    a.out_bubble = out_bubble;
    a.out_feasible = out_feasible;
    a.best_idx = out_best_idx;
    a.best_makespan = out_best_makespan;
    a.best_bubble = out_best_bubble;
    a.hist = params->hist_bins > 0 ? (unsigned long long *)out_hist : nullptr;
    a.hist_bins = params->hist_bins;
    a.hist_shift = params->hist_shift;
    a.hist_in_lds = (size_t)a.S * a.hist_bins * 4 <= (size_t)kMaxLdsHistBytes;
    hipLaunchKernelGGL(k_zero_status, dim3(1), dim3(64), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_prepass, dim3(grid_for(a.C, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_best_init, dim3(grid_for(a.K + (long long)a.S * a.hist_bins, 4096)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    // the evaluation: the resolve kernels must not see the search's outputs (they would search too)
    KArgs e = a;
    e.hist = nullptr;
    int direct = -1;
    rc = launch_resolve<false>(e, ws, cands->w_bound, st, &direct);
    if (rc) return rc;
    const long long tiles = ((a.C + 63) / 64) * ((a.K + 63) / 64);
    if (tiles > INT32_MAX) return ADAPTRA_EINVAL;
    e = a;
    if (direct >= 0) { e.direct_out = 1; e.cls_hi = direct; }
    hipLaunchKernelGGL(k_eval_epilogue, dim3((unsigned)tiles), dim3(kBlock), 0, st, e);
    ADAPTRA_LAUNCH_CHECK();
    // the search, over the makespans just computed
    const long long tasks = ((a.K + 63) / 64) * ((a.C + 63) / 64);
    const size_t lds = a.hist && a.hist_in_lds ? (size_t)a.S * a.hist_bins * 4 : 0;
    if (a.hist && a.S <= 16)
        hipLaunchKernelGGL(k_best_from_eval<16>, dim3((unsigned)((tasks + kWavesPerBlock - 1) / kWavesPerBlock)), dim3(kBlock),
                           lds, st, a);
    else
        hipLaunchKernelGGL(k_best_from_eval<0>, dim3((unsigned)((tasks + kWavesPerBlock - 1) / kWavesPerBlock)), dim3(kBlock),
                           lds, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_best_finalize, dim3(grid_for(a.K, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

size_t adaptra_sensitivity_workspace_bytes(const adaptra_params_t *params, int64_t n_cand, int64_t n_scen) {
    Workspace ws;
    if (!params || n_scen < 1 || n_scen > INT32_MAX / ADAPTRA_MAX_STAGES) return 0;
    if (!plan_workspace(params->S, params->M, n_cand, n_scen * params->S, &ws)) return 0;
    return ws.total;
}

int adaptra_sensitivity(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                        const adaptra_scenarios_t *scens, int32_t delta,
                        int32_t *out_makespan, uint8_t *out_feasible, int32_t *out_sens,
                        void *workspace, size_t workspace_bytes, void *stream) {
    if (!params || !cands || !scens) return ADAPTRA_EINVAL;
    if (delta < 1 || scens->n < 1 || scens->n > INT32_MAX / ADAPTRA_MAX_STAGES) return ADAPTRA_EINVAL;
    if (params->S > 1 && !out_sens) return ADAPTRA_EINVAL;
    // The same machinery as adaptra_eval on a scenario axis of S blocks of n: the base
    // scenarios, then one block per link with that link's delay raised.
    adaptra_scenarios_t wide = *scens;
    wide.n = scens->n * params->S;
    Workspace ws;
    int rc = validate_common(params, cands, &wide, workspace, workspace_bytes, &ws);
    if (rc) return rc;
    if (cands->n * scens->n > INT32_MAX) return ADAPTRA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    KArgs a;
    fill_args(&a, params, cands, &wide, workspace, ws);
    a.Kin = scens->n;
    a.sens_delta = delta;
    a.out_makespan = out_makespan;
    a.out_feasible = out_feasible;
    a.out_bubble = out_sens;
    hipLaunchKernelGGL(k_zero_status, dim3(1), dim3(64), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_prepass, dim3(grid_for(a.C, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    rc = launch_resolve<false>(a, ws, cands->w_bound, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_sens_epilogue, dim3(grid_for(a.C * a.Kin, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

int adaptra_best(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                 const adaptra_scenarios_t *scens,
                 int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                 uint64_t *out_hist,
                 void *workspace, size_t workspace_bytes, void *stream) {
    return adaptra_detail::best(params, cands, scens, 0, out_best_idx, out_best_makespan, out_best_bubble,
                                out_hist, workspace, workspace_bytes, stream);
}

}  // extern "C"

// adaptra_best proper.  pair_div > 0 (the guided search): candidate c belongs to scenario
// c / pair_div and is evaluated under that scenario only, by the general kernel (its lanes
// carry candidates, so each may have a scenario of its own).
int adaptra_detail::best(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                         const adaptra_scenarios_t *scens, int pair_div,
                         int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                         uint64_t *out_hist,
                         void *workspace, size_t workspace_bytes, void *stream) {
    Workspace ws;
    int rc = validate_common(params, cands, scens, workspace, workspace_bytes, &ws, false);
    if (rc) return rc;
    if (!out_best_idx || !out_best_makespan) return ADAPTRA_EINVAL;
    if (params->hist_bins < 0 || params->hist_bins > 65536) return ADAPTRA_EINVAL;
    if (params->hist_bins > 0 && (!out_hist || params->hist_shift < 0 || params->hist_shift > 30))
        return ADAPTRA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    KArgs a;
    fill_args(&a, params, cands, scens, workspace, ws);
    a.best_idx = out_best_idx;
    a.best_makespan = out_best_makespan;
    a.best_bubble = out_best_bubble;
    a.hist = params->hist_bins > 0 ? (unsigned long long *)out_hist : nullptr;
    a.hist_bins = params->hist_bins;
    a.hist_shift = params->hist_shift;
    a.hist_in_lds = (size_t)a.S * a.hist_bins * 4 <= (size_t)kMaxLdsHistBytes;
    if (pair_div < 0 || (pair_div > 0 && (cands->n + pair_div - 1) / pair_div > scens->n)) return ADAPTRA_EINVAL;
    a.pair_div = pair_div;
    hipLaunchKernelGGL(k_zero_status, dim3(1), dim3(64), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_prepass, dim3(grid_for(a.C, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_best_init, dim3(grid_for(a.K + (long long)a.S * a.hist_bins, 4096)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    rc = launch_resolve<true>(a, ws, cands->w_bound, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_best_finalize, dim3(grid_for(a.K, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

extern "C" {

int adaptra_seed(const adaptra_params_t *params, const adaptra_scenarios_t *scens, int32_t x_max,
                 const int32_t *w_current, int32_t *out_w_init, int32_t *out_w_adapted,
                 uint8_t *out_not_absorbed, void *stream) {
    if (!params || !scens) return ADAPTRA_EINVAL;
    const int S = params->S, M = params->M;
    if (S < 1 || S > ADAPTRA_MAX_STAGES || M < 1 || M > ADAPTRA_MAX_MICROBATCHES) return ADAPTRA_EINVAL;
    if (scens->n < 1 || scens->n > INT32_MAX || !params->t_f || !params->t_b) return ADAPTRA_EINVAL;
    if (S > 1 && (!scens->c_fwd || !scens->c_bwd)) return ADAPTRA_EINVAL;
    if ((scens->t_f == nullptr) != (scens->t_b == nullptr)) return ADAPTRA_EINVAL;
    if (out_w_init && x_max < 1) return ADAPTRA_EINVAL;
    if (out_not_absorbed && !w_current) return ADAPTRA_EINVAL;
    if (!out_w_init && !out_w_adapted && !out_not_absorbed) return ADAPTRA_EINVAL;
    SeedArgs a;
    a.S = S; a.M = M; a.x_max = x_max; a.K = scens->n;
    a.t_f = params->t_f; a.t_b = params->t_b; a.cf = scens->c_fwd; a.cb = scens->c_bwd;
    a.tfs = scens->t_f; a.tbs = scens->t_b;
    a.w_cur = w_current; a.w_init = out_w_init; a.w_adapted = out_w_adapted; a.not_absorbed = out_not_absorbed;
    hipLaunchKernelGGL(k_seed, dim3(grid_for(a.K, INT32_MAX)), dim3(kBlock), 0, (hipStream_t)stream, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

int adaptra_set_kernel_mode(int mode) {
    if (mode < 0 || mode > 4) return -1;
    const int prev = g_kernel_mode;
    g_kernel_mode = mode;
    return prev;
}

int adaptra_set_resolve_events(void *before, void *after) {
    g_ev_before = (hipEvent_t)before;
    g_ev_after = (hipEvent_t)after;
    return ADAPTRA_OK;
}

int adaptra_valu_probe(int32_t blocks, int32_t iters, int32_t *scratch, void *stream, int64_t *lane_ops) {
    if (blocks < 1 || iters < 1 || !scratch) return ADAPTRA_EINVAL;
    hipLaunchKernelGGL(k_valu_probe, dim3(blocks), dim3(kBlock), 0, (hipStream_t)stream, iters, 1, -5, scratch);
    ADAPTRA_LAUNCH_CHECK();
    if (lane_ops) *lane_ops = (int64_t)blocks * kBlock * (int64_t)iters * 32 * 8 * 2;
    return ADAPTRA_OK;
}

int adaptra_last_hip_error(void) { return g_last_hip_error; }

int adaptra_version(void) { return 1; }

}  // extern "C"

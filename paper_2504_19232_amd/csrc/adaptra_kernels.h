// adaptra_kernels.h -- the two on-chip recurrence kernels of the evaluation path (gfx950), their
// shared device helpers and their launchers.  Internal: included by adaptra.hip (the rest of the
// path and the C ABI) and by one translation unit per kernel size (adaptra_size.inc), so that the
// sizes compile side by side.
//
// Model and notation follow the Adaptra paper: S stages, M micro-batches, w[s] warm-up
// forwards of stage s (the paper's x_s = w[s] + 1), link delays c_fwd / c_bwd, the
// dependency rules of Section 3.1 and the stage order of Sections 4.1 / 4.3.  Everything
// is int32 microseconds; there is no floating point on this path.
//
// Order of evaluation used by both kernels: with w non-increasing over stages (Lemma 1) the
// rounds r = -w[0] .. M-1, each a forward sweep s = 0..S-1 over F(s, w[s] + r) followed (r >= 0)
// by a backward sweep s = S-1..0 over B(s, r), visit every op after all of its predecessors and
// every stage's ops in that stage's own order.
#ifndef ADAPTRA_KERNELS_H
#define ADAPTRA_KERNELS_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "adaptra.h"
#include "adaptra_internal.h"

namespace adaptra_detail {

constexpr int kNeg = -(1 << 30);          // "no earlier op": below every shifted time
constexpr int kChunk = 16;                 // candidates one wavefront works through, at most; the direct
                                           // output copies a chunk's flags as ONE 16-byte word
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = 64 * kWavesPerBlock;
constexpr int kClassDead = 255;           // deadlocked: never resolved
constexpr int kClassDeep = 254;           // warm-up depth beyond the LDS ring: general kernel
constexpr int kNumRingClasses = 16;       // ring of 8 * (class + 1) slots: up to 128 slots = 32 KiB per wavefront
constexpr int kMaxLdsHistBytes = 16384;
// Wavefront priorities inside the hot kernel (s_setprio): a wavefront in a forward sweep -- LDS
// traffic and independent instructions -- goes ahead of one in a backward sweep, whose
// instructions all wait on each other and fill the gaps just as well.  Measured on configuration
// 3: 49.3 -> 47.2 ms; any two different levels do, the other way round costs 2 ms.
constexpr int kPrioForward = 2, kPrioBackward = 0;
constexpr int kDrainBlock = 4;   // stages per copy of the cool-down round (see the hot kernel)
constexpr int kPrefetchStages = 4;        // ring reads run this many stages ahead of their use
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
    int *status;                           // [0..3] input check, [16..32] candidates per ring class, [48] entries of live_list
    int *live_list;                        // search only: the feasible candidates an on-chip kernel can take, in any order
    const int *gate;                       // guided search only: when set and *gate == 0 (nothing moved in the round
                                           // before) every kernel of the call exits at once
    Neighbourhood moves;                   // guided search only: moves.point set = the candidates are derived, `w` is not read
    int *mk_t;                             // eval: makespan, candidate-major [C][K]
    int *tpad;                             // t_f at [0..63], t_b at [64..127], zero beyond stage S-1
    int kernel_mode;                       // host side only: the kernel selection this call runs under
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
// The value continues in a register chosen here (an empty asm statement that "rewrites" it).
__device__ __forceinline__ void pin_vector(int &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin_scalar(unsigned &v) { asm volatile("" : "+s"(v)); }
__device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }

// Move j of the guided search's neighbourhood: j = 0 keeps the point; otherwise (j - 1) / 2
// numbers the stage range [lo, hi] and the parity of j - 1 picks -1 (even) or +1 (odd).
__device__ __forceinline__ void neighbourhood_move(int nb, int S, int j, int *lo, int *hi, int *sign) {
    if (j == 0) { *lo = 0; *hi = -1; *sign = 0; return; }
    int r = (j - 1) >> 1;
    *sign = ((j - 1) & 1) ? 1 : -1;
    if (nb == 0) { *lo = 0; *hi = r; return; }
    int a = 0;
    while (r >= S - a) { r -= S - a; ++a; }      // ranges are numbered a = 0.., b = a..S-1
    *lo = a; *hi = a + r;
}
// Where a candidate's warm-up vector comes from: w[s] = base[s * stride] + (lo <= s <= hi ?
// sign : 0), not yet clamped -- an array column, or a scenario's point and a move.
struct WSource {
    const int *base;
    long long stride;
    int lo, hi, sign;
    bool rest;                             // the scenario is at rest: w = (0, 1, 0, ...), which Lemma 1 rules out
};
__device__ __forceinline__ WSource w_source(const KArgs &a, long long c) {
    WSource src;
    if (a.moves.point) {
        const long long k = c / a.moves.per_point;
        src.base = a.moves.point + k;
        src.stride = a.moves.K;
        src.rest = a.moves.active && !a.moves.active[k];
        neighbourhood_move(a.moves.nb, a.S, (int)(c % a.moves.per_point), &src.lo, &src.hi, &src.sign);
    } else {
        src.base = a.w + c;
        src.stride = a.C;
        src.lo = 0; src.hi = -1; src.sign = 0;
        src.rest = false;
    }
    return src;
}
__device__ __forceinline__ int w_at(const WSource &src, int s) {
    if (src.rest) return s == 1;
    return src.base[(long long)s * src.stride] + (s >= src.lo && s <= src.hi ? src.sign : 0);
}
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
//   - returns bit `kBit` of the 64-bit mask set ? b : a.  One SALU op spreads the bit over a
//     scalar register pair (a signed one-bit field extract), one VALU op selects on that pair.
//     The pair is an ordinary one, not vcc: in a dense stream a v_cndmask_b32 on a vcc that
//     the scalar unit wrote issues at a fifth of the plain rate on this chip, on an ordinary
//     pair at the plain rate (the probes of adaptra_probe.hip); spaced out as in this kernel
//     the two forms measured the same.  A branch around a move measured slower, hoisted lane
//     masks would need two SGPRs per stage.
//   - advances the stage's ring offset `t` by one slot (see ring_next).
template <int kBit>
__device__ __forceinline__ int select_by_bit_and_advance(unsigned long long mask, int a, int b,
                                                         unsigned &t, unsigned bias) {
    int o;
    unsigned long long lanes;
    asm("s_bfe_i64 %2, %3, %4\n\tv_cndmask_b32_e64 %0, %5, %6, %2\n\t"
        "s_add_u32 %1, %1, 0x100\n\ts_cmov_b32 %1, %7"
        : "=v"(o), "+s"(t), "=&s"(lanes) : "s"(mask), "n"(kBit | (1 << 16)), "v"(a), "v"(b), "s"(bias) : "scc");
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
// kBegin, kBegin + kStep, ... below kEnd
template <int kBegin, int kEnd, int kStep, class F>
__device__ __forceinline__ void stage_blocks_up(F &&f) {
    if constexpr (kBegin < kEnd) {
        f(StageIndex<kBegin>{});
        stage_blocks_up<kBegin + kStep, kEnd, kStep>(f);
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
// A wavefront-uniform value held in a vector register on purpose: v_add_u32 with two vector
// operands can issue at twice the rate of the same add with a scalar operand on this chip (see
// adaptra_probe.hip), so the addends of the recurrence's steady loop live in VGPRs -- where there
// is room: at 32 stages the vector form takes all 128 registers and spills 11 values (outside
// the steady loop) for no gain (40.06 against 40.12 ms on configuration 3), so the addends stay
// scalar there; at 8 and 16 stages the vector form is 1-2 % ahead.
// (Per-lane addends -- per-scenario stage times -- pass through the same empty statement: it
// also keeps the compiler from re-deriving them from memory inside the loops.)
template <int S, bool VT>
__device__ __forceinline__ int in_vgpr(int v) {
    if constexpr (S < 32 || VT) asm("" : "+v"(v));
    return v;
}
__device__ __forceinline__ int clampw(int w, int M) { return w < 0 ? 0 : (w > M - 1 ? M - 1 : w); }
// Byte `k` of `word` plus a wavefront-uniform number, as ONE instruction (an add that selects the
// byte of its operand).  Written out because the compiler, given two loops that use the bytes of
// the round-invariant packed w, unpacks all S of them into registers of their own ahead of the
// loops (32 registers at 32 stages, a wavefront per SIMD less).
__device__ __forceinline__ unsigned byte_plus(unsigned word, int k, int uniform) {
    unsigned r;
    switch (k) {
    case 0: asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(r) : "v"(word), "s"(uniform)); break;
    case 1: asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(r) : "v"(word), "s"(uniform)); break;
    case 2: asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(r) : "v"(word), "s"(uniform)); break;
    default: asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD" : "=v"(r) : "v"(word), "s"(uniform)); break;
    }
    return r;
}

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


// The scenario-lanes kernel exists for 2, 4, 8, 12, 16, 24 and 32 stages; a pipeline with
// another stage count up to 32 runs in the next larger one, padded with stages that take no
// time (see the kernel).  0: no such kernel (more than 32 stages).
inline int hot_kernel_stages(int S) {
    for (int p : {2, 4, 8, 12, 16, 24, 32})
        if (S <= p) return p;
    return 0;
}
// The candidate-lanes kernel has two sizes more: per-lane state in VGPRs (last, c_fwd, c_bwd:
// 3 S registers) still fits at 48 and 64 stages with two wavefronts per SIMD, which the
// scenario-lanes kernel's per-stage scalars (2 S SGPRs) do not.
inline int cand_kernel_stages(int S) {
    for (int p : {2, 4, 8, 12, 16, 24, 32, 48, 64})
        if (S <= p) return p;
    return 0;
}
// With per-scenario stage times the candidate-lanes kernel keeps 5 S values per lane: up to 32 stages.
constexpr int kCandLanesStageTimesMax = 32;

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
__global__ __launch_bounds__(kBlock, S >= 48 || (VT && S >= 16) ? 2 : (S >= 24 ? 4 : (AHEAD ? 4 : 6))) void k_resolve_cand_lanes(KArgs) {
    // The arguments are read through kargs() where they are needed (see there): kept in SGPRs
    // across the round loop they would crowd out the loop's own scalars.
    extern __shared__ int lds[];
    if (kargs()->gate && *kargs()->gate == 0) return;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int D = kargs()->ring_slots, M = kargs()->M;
    int *const ring = lds + wv * D * 64 + lane;          // slot i of this lane at ring[i * 64]
    // The search (BEST) walks the pre-pass's list of feasible candidates instead of the candidate
    // axis itself, 64 list entries per tile: a tile costs the same however many of its lanes carry
    // a pair, and among all candidates the feasible ones can be few (the guided search's pools hold
    // every neighbour of a point, most of which break Lemma 1 or a memory cap).  The order of the
    // list is arbitrary; the result -- a minimum over (makespan, candidate) keys -- is not.
    const long long n_cand = BEST ? (long long)uni(kargs()->status[48]) : kargs()->C;
    const long long ctiles = (n_cand + 63) / 64;
    const long long ntiles = kargs()->pair_div ? ctiles : kargs()->K * ctiles;
    const long long nwaves = (long long)gridDim.x * kWavesPerBlock;
    // Stage times come from the zero-padded table, re-read in blocks of 16 stages inside the
    // round loop (scalar loads, a cache hit each): kept for all stages they would take 2 S
    // SGPRs, more than there are at S = 32.
    constexpr int kTimesBlock = 16;
    typedef __attribute__((address_space(4))) int ConstInt;   // written by k_prepass, constant here
    for (long long tile = (long long)blockIdx.x * kWavesPerBlock + wv; tile < ntiles; tile += nwaves) {
        const long long at = (tile % ctiles) * 64 + lane;
        const bool have = at < n_cand;
        long long c = at;
        if constexpr (BEST) c = have ? kargs()->live_list[at] : 0;
        const long long k = kargs()->pair_div ? (have ? c / kargs()->pair_div : 0) : tile / ctiles;
        const long long kin = k % kargs()->Kin;
        const int link_up = (int)(k / kargs()->Kin) - 1;
        bool run = false;
        if (have) {
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
        int r_all;                                       // last round in which every stage of every lane has a forward
        {                                                // (worked out here, before the state below occupies the registers)
            int wmax = 0;
#pragma unroll
            for (int s = 0; s < S; ++s) wmax = imax(wmax, (int)((wpk[s / 4] >> (8 * (s % 4))) & 0xffu));
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) wmax = imax(wmax, __shfl_xor(wmax, off));
            r_all = uni(M - 1 - wmax);
        }
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
        // One round.  kTest: the forward step of a stage counts only if its micro-batch exists,
        // w[s] + r < M; the rounds in which that holds for every stage of every lane of the
        // wavefront (the long middle of the schedule) run a copy without the test, three vector
        // instructions per stage and round less.
        auto one_round = [&](int r, auto test_tag) {
            constexpr bool kTest = decltype(test_tag)::value;
            if (r == 0) {
                // round 0's forwards were the last of the fill phase
            } else if constexpr (AHEAD) {                // forward sweep, ring reads three stages ahead
                constexpr int kAhead = S - 1 < 3 ? S - 1 : 3;
                int *slot_of[S];
                int ahead[S];
                auto ring_slot = [&](int s) {
                    unsigned slot = byte_plus(wpk[s / 4], s % 4, b);
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
                        const bool valid = kTest && byte_plus(wpk[s / 4], s % 4, r) < (unsigned)M;
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
                        if constexpr (kTest) last[s] = valid ? fin : last[s];
                        else last[s] = fin;
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
                    const bool valid = kTest && byte_plus(wpk[s / 4], s % 4, r) < (unsigned)M;
                    unsigned slot = byte_plus(wpk[s / 4], s % 4, b);
                    slot = slot < slot - (unsigned)D ? slot : slot - (unsigned)D;      // mod D (w < D, b < D)
                    int *const p = ring + slot * 64;
                    int t_f_s;
                    if constexpr (VT) t_f_s = tfv[s];
                    else t_f_s = tf[j];
                    int fin;
                    if (s == 0) fin = last[0] + t_f_s;
                    else fin = imax(last[s], *p + cf[s - 1]) + t_f_s;
                    if constexpr (kTest) last[s] = valid ? fin : last[s];
                        else last[s] = fin;
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
        };
        one_round(0, std::true_type{});
        int r = 1;
        for (; r <= r_all; ++r) one_round(r, std::false_type{});
        for (; r < M; ++r) one_round(r, std::true_type{});
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
__global__ __launch_bounds__(kBlock, S >= 32 ? 4 : (S >= 24 ? 5 : 6)) void k_resolve_scen_lanes(KArgs) {
    // The arguments are read through kargs() where they are needed (see there), never
    // through the by-value parameter.
    extern __shared__ int lds[];
    if (kargs()->gate && *kargs()->gate == 0) return;
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
    // The search (BEST) walks the pre-pass's list of feasible candidates, as the candidate-lanes
    // kernel does: a wavefront's chunk then holds candidates that all run, however few of the
    // candidate axis are feasible (3 901 of 65 536 on the benchmarked workload: by index, most
    // chunks held one or none and the wavefronts' work was set-up).  The list may be much shorter
    // than the axis the grid was sized for, so the chunk is chosen here: about 8 192 wavefronts'
    // worth of work as on the host, never so short that the grid's tasks would not cover the list.
    const long long n_cand = BEST && kargs()->live_list ? (long long)uni(kargs()->status[48]) : kargs()->C;
    int chunk_here = kargs()->chunk;
    if (BEST && kargs()->live_list) {
        long long ch = n_cand * kargs()->n_ktiles / 8192;
        const long long need = (n_cand * kargs()->chunk + kargs()->C - 1) / kargs()->C;
        ch = ch < need ? need : ch;
        chunk_here = uni((int)(ch < 1 ? 1 : (ch > kChunk ? kChunk : ch)));
    }
    const long long c0 = (task / kargs()->n_ktiles) * chunk_here;
    if (c0 < n_cand) {
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
        const long long c_left = n_cand - c0;
        const int chunk = chunk_here;
        const int c_end = (int)(c_left < chunk ? c_left : chunk);
        // Direct output (evaluation, chunks of exactly 16 candidates, a single launch): the
        // makespans of the chunk are kept per lane and written at its end, 16 consecutive
        // candidates = 64 contiguous bytes per scenario and output plane, so that the separate
        // streaming pass over all pairs is not needed and the writes hide under the VALU work.
        __builtin_amdgcn_s_setprio(kPrioForward);
        for (int ci = 0; ci < c_end; ++ci) {
            const long long c = BEST && kargs()->live_list ? (long long)uni(kargs()->live_list[c0 + ci]) : c0 + ci;
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
            unsigned slot_first[kPD > 1 ? kPD : 1];   // ring addresses of stages 1..kPD-1 for the coming round
            int add_f[S];         // what the stage's next op adds to L[s]: t_f while the pipeline
                                  // fills, t_f + t_b in steady state, t_b once out of forwards
#pragma unroll
            for (int s = 0; s < S; ++s) {
                L[s] = kNeg;
                x[s] = 0;
                soff[s] = bias;   // micro-batch 0 sits in slot 0
                add_f[s] = in_vgpr<S, VT>(ADAPTRA_TF(s));
            }
            L[0] = -add_f[0];

// One forward step of stage s.  x[s] is the value micro-batch m got on stage s-1, read from
// ring slot m mod D some stages earlier; if the two stages have equal w that value is only
// being produced in this very round and comes from L[s-1] instead.  The result goes to slot
// m and the stage's offset moves on to slot m+1.
#define ADAPTRA_F_OP(s, e)                                                      \
    do {                                                                        \
        unsigned slot;                                                          \
        if constexpr ((s) >= 1 && (s) < kPD) slot = slot_first[(s) < kPD ? (s) : 0]; \
        else slot = ring + soff[s];                                             \
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
// ... and the reads of stages 1..kPD-1, which no stage of their own round can issue that far
// ahead, are issued at the end of the forward sweep before, so that they complete under the
// backward sweep.  Their addresses are the ones those stages write to in the next round
// (slot_first: kept, not computed again).
#define ADAPTRA_READ_NEXT_ROUND()                                               \
    stages_up<1, kPD>(ADAPTRA_STAGE_LAMBDA(sj) {                                \
        constexpr int j = decltype(sj)::value;                                  \
        slot_first[j] = ring + soff[j];                                         \
        x[j] = *(lds_int *)slot_first[j];                                       \
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
            for (int s = 0; s < S; ++s) add_f[s] = in_vgpr<S, VT>(add_f[s] + ADAPTRA_TB(s));
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
            // w[s] + r > M-1, which holds for the stages 0 .. done-1 (w is non-increasing), and
            // `done` only grows.  The rounds are taken by one copy of the round's code per block
            // of kDrainBlock stages: the copy for the block [D0, D1) runs while `done` lies in
            // it.  In that copy the stages below D0 have no forward step, no test, and no ring
            // read issued on their behalf; the stages from D1 on run the steady forward step
            // untested; only the block's own stages are tested.  The finished stages' backward
            // durations are added ahead of the steady backward sweep (independent adds).
            {
                int done = 0, r = M - W;
                int converted = 0;     // VT: stages whose addend has been switched to t_b alone
                stage_blocks_up<0, S, kDrainBlock>(ADAPTRA_STAGE_LAMBDA(bi) {
                    constexpr int D0 = decltype(bi)::value;
                    constexpr int D1 = D0 + kDrainBlock < S ? D0 + kDrainBlock : S;
                    // The state enters each copy's loop through a register of the loop's own
                    // choosing: without this the compiler reconciles the registers of the copy
                    // before with this loop's on the loop's BACK edge, S vector moves per round.
                    stages_up<0, S>(ADAPTRA_STAGE_LAMBDA(si) {
                        constexpr int s = decltype(si)::value;
                        pin_vector(L[s]);
                        pin_scalar(soff[s]);
                    });
                    for (; r <= M - 1; ++r) {
                        // (counted with one ballot over the lanes that hold w; a scalar loop over the
                        // stages measured 0.3 % slower, 1 % with per-scenario stage times)
                        static_assert(S <= 32, "the stages' lanes are counted in the low half of the ballot");
                        done = __builtin_popcount((unsigned)__ballot(wq_lanes + r > M - 1) & (S >= 32 ? ~0u : (1u << (S & 31)) - 1u));
                        done = uni(done);      // said again for the compiler, which otherwise loses it across the copies
                        if constexpr (VT) {
                            // per-lane addends: a stage that has just run out of forwards keeps t_b alone
                            converted = uni(converted);
                            stages_up<D0, D1>(ADAPTRA_STAGE_LAMBDA(si) {
                                constexpr int s = decltype(si)::value;
                                if (s >= converted && s < done) add_f[s] = in_vgpr<S, VT>(add_f[s] - ADAPTRA_TF(s));
                            });
                            converted = done < D1 ? done : D1;
                        }
                        if (D1 < S && done >= D1) break;      // the next block's copy takes this round
                        stages_up<0, S>(ADAPTRA_STAGE_LAMBDA(si) {
                            constexpr int s = decltype(si)::value;
                            if constexpr (s >= D1) {
                                ADAPTRA_F_OP(s, add_f[s]);
                            } else if constexpr (s >= D0) {
                                if (s >= done) ADAPTRA_F_OP(s, add_f[s]);
                            }
                            if constexpr (s + kPD >= D0) ADAPTRA_READ_AHEAD(s);
                        });
                        stages_up<(D0 > 1 ? D0 : 1), kPD>(ADAPTRA_STAGE_LAMBDA(sj) {      // next round's first reads
                            constexpr int j = decltype(sj)::value;
                            slot_first[j] = ring + soff[j];
                            x[j] = *(lds_int *)slot_first[j];
                        });
                        stages_up<0, D0>(ADAPTRA_STAGE_LAMBDA(si) {
                            constexpr int s = decltype(si)::value;
                            if constexpr (VT) L[s] += add_f[s];
                            else L[s] += ADAPTRA_TB(s);
                        });
                        stages_up<D0, D1>(ADAPTRA_STAGE_LAMBDA(si) {
                            constexpr int s = decltype(si)::value;
                            if (s < done) {
                                if constexpr (VT) L[s] += add_f[s];
                                else L[s] += ADAPTRA_TB(s);
                            }
                        });
                        ADAPTRA_B_SWEEP();
                    }
                });
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
        }
        if (BEST && kvalid && key != kNoKey) atomicMin(&kargs()->keys[k], key);
        if constexpr (!BEST) {
            if (kargs()->direct_out && kvalid) {
                // The chunk's makespans come back from the candidate-major scratch this wavefront
                // has just written (its own stores, in program order; 256 contiguous bytes per
                // candidate), four candidates at a time: kept in registers across the candidate
                // loop they would cost 16 VGPRs there, where the recurrence needs them.
                const long long C = kargs()->C, P = C * K;
                const long long at = k * C + c0;                 // 16 candidates from here
                static_assert(kChunk == 16, "a chunk's flag bytes are copied as one uint4");
                *(uint4 *)(kargs()->out_feasible + at) = *(const uint4 *)(kargs()->cand_flag + c0);
                const int M = kargs()->M;
                // all loads first: a load issued behind the stores below would have to wait for
                // them (memory operations of a wavefront are counted off in order)
                int mk16[kChunk];
#pragma unroll
                for (int j = 0; j < kChunk; ++j) {
                    // a deadlocked candidate was never resolved: sentinel.  (One left to the
                    // general kernel has no makespan yet either; its tile is redone by the
                    // epilogue, so anything may be written here.)
                    const bool dead = uni(kargs()->cand_flag[c0 + j]) & ADAPTRA_FLAG_DEADLOCK;
                    mk16[j] = dead ? INT32_MAX : kargs()->mk_t[(c0 + j) * K + k];
                }
#pragma unroll
                for (int v = 0; v < kChunk / 4; ++v)
                    ((int4 *)(kargs()->out_makespan + at))[v] = make_int4(mk16[4 * v], mk16[4 * v + 1], mk16[4 * v + 2], mk16[4 * v + 3]);
                if (kargs()->out_bubble) {
                    for (int s = 0; s < kargs()->S; ++s) {
                        const int busy = M * (ADAPTRA_TF(s) + ADAPTRA_TB(s));
                        int4 *const bo = (int4 *)(kargs()->out_bubble + (long long)s * P + at);
#pragma unroll
                        for (int v = 0; v < kChunk / 4; ++v) {
                            int b4[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int mkj = mk16[4 * v + j];
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


// The ring classes a launch covers.  With a bound on w one launch takes every class up to the
// bound's, with exactly the ring the bound needs; without, five launches with rings of 8, 16,
// 32, 64 and 128 slots share the classes (empty ones exit at once).
struct ClassRange {
    int lo, hi;
};
inline int ring_launches(int w_bound, int M, ClassRange out[5]) {
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

// Dynamic LDS above the default limit of 48 KiB has to be allowed per kernel; `allowed` (one
// per kernel instantiation and device) remembers the largest size already granted.
constexpr int kLdsDevices = 64;
struct LdsAllowed {
    std::atomic<size_t> bytes[kLdsDevices];
};
inline bool lds_needs_grant(size_t lds, const LdsAllowed &allowed, int *dev) {
    if (lds <= 48 * 1024) return false;
    if (hipGetDevice(dev) != hipSuccess) *dev = -1;
    return !(*dev >= 0 && *dev < kLdsDevices && allowed.bytes[*dev].load(std::memory_order_relaxed) >= lds);
}
inline void lds_granted(size_t lds, LdsAllowed *allowed, int dev) {
    if (dev >= 0 && dev < kLdsDevices) allowed->bytes[dev].store(lds, std::memory_order_relaxed);
}
#define ADAPTRA_ALLOW_LDS(kernel, lds)                                                                        \
    do {                                                                                                      \
        int dev_;                                                                                             \
        if (lds_needs_grant((lds), lds_allowed, &dev_)) {                                                     \
            hipError_t e_ = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(lds)); \
            if (e_ != hipSuccess) return hip_fail(e_);                                                        \
            lds_granted((lds), &lds_allowed, dev_);                                                           \
        }                                                                                                     \
    } while (0)

template <int S, bool BEST, bool VT>
int launch_scen_lanes_one(KArgs a, int w_bound, hipStream_t st) {
    static LdsAllowed lds_allowed;
    const long long tasks = a.n_chunks * a.n_ktiles;
    const long long blocks = (tasks + kWavesPerBlock - 1) / kWavesPerBlock;      // grids_fit() has bounded it
    ClassRange ranges[5];
    const int n_launches = ring_launches(w_bound, a.M, ranges);
    for (int i = 0; i < n_launches; ++i) {
        a.cls_lo = ranges[i].lo;
        a.cls_hi = ranges[i].hi;
        a.ring_slots = 8 * (a.cls_hi + 1);
        size_t lds = (size_t)kWavesPerBlock * a.ring_slots * 256;
        if (BEST && a.hist && a.hist_in_lds) lds += (size_t)a.S * a.hist_bins * 4;
        // above the default dynamic-LDS limit: raise it for this kernel, once per size asked for
        // (the call costs tens of microseconds, the guided search launches hundreds of times)
        ADAPTRA_ALLOW_LDS((k_resolve_scen_lanes<S, BEST, VT>), lds);
        hipLaunchKernelGGL((k_resolve_scen_lanes<S, BEST, VT>), dim3((unsigned)blocks), dim3(kBlock), lds, st, a);
        ADAPTRA_CHECK_LAUNCH();
    }
    return ADAPTRA_OK;
}

template <int S, bool BEST, bool VT, bool AHEAD>
int launch_cand_lanes_one(KArgs a, int w_bound, hipStream_t st) {
    static LdsAllowed lds_allowed;
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
        ADAPTRA_ALLOW_LDS((k_resolve_cand_lanes<S, BEST, VT, AHEAD>), lds);
        hipLaunchKernelGGL((k_resolve_cand_lanes<S, BEST, VT, AHEAD>), dim3((unsigned)blocks), dim3(kBlock), lds, st, a);
        ADAPTRA_CHECK_LAUNCH();
    }
    return ADAPTRA_OK;
}


// One translation unit per size defines these two (adaptra_size.inc): the launch of the
// scenario-lanes kernel (search or evaluation; per-scenario stage times iff a.tfs) and of the
// candidate-lanes kernel (plain or read-ahead form) at `stages` stages.
#define ADAPTRA_DECLARE_SIZE(stages)                                                                    \
    int launch_scen_lanes_##stages(bool best, const KArgs &a, int w_bound, hipStream_t st);             \
    int launch_cand_lanes_##stages(bool best, bool ahead, const KArgs &a, int w_bound, hipStream_t st);
ADAPTRA_DECLARE_SIZE(2) ADAPTRA_DECLARE_SIZE(4) ADAPTRA_DECLARE_SIZE(8) ADAPTRA_DECLARE_SIZE(12) ADAPTRA_DECLARE_SIZE(16)
ADAPTRA_DECLARE_SIZE(24) ADAPTRA_DECLARE_SIZE(32) ADAPTRA_DECLARE_SIZE(48) ADAPTRA_DECLARE_SIZE(64)
#undef ADAPTRA_DECLARE_SIZE

}  // namespace adaptra_detail

#endif  // ADAPTRA_KERNELS_H

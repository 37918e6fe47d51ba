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

#include <atomic>

#include "adaptra.h"
#include "adaptra_internal.h"
#include "adaptra_kernels.h"
#include "adaptra_testing.h"

// Scratch of adaptra_best_static, the entry point for callers that cannot allocate: one copy per
// GPU the library runs on, held until the process ends.  Host code never uses this name as an
// address (it is a host-side stand-in): the device address comes from hipGetSymbolAddress, once
// per device (static_scratch below).
constexpr size_t kStaticScratchBytes = (size_t)ADAPTRA_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using namespace adaptra_detail;

// ---------------------------------------------------------------------------------------
// Per candidate, independent of the scenario: w' = clamp(w, 0, M-1); deadlock iff some
// w'[s] < w'[s+1] (Lemma 1); memory cap exceeded iff some w'[s] + 1 > mem_cap[s]
// (Algorithm 1, x_max).  Also packs w' into bytes for the hot kernel and bins the
// candidate by the ring depth it needs, w'[0] + 1 slots.
__global__ __launch_bounds__(kBlock) void k_prepass(KArgs a) {
    if (a.gate && *a.gate == 0) return;
    __shared__ int class_count[kNumRingClasses + 1];
    if (threadIdx.x <= kNumRingClasses) class_count[threadIdx.x] = 0;
    if (blockIdx.x == 0 && threadIdx.x < 128) {             // stage times padded with zeros (candidate-lanes kernel)
        const int i = threadIdx.x & 63;
        a.tpad[threadIdx.x] = i < a.S ? (threadIdx.x < 64 ? a.t_f[i] : a.t_b[i]) : 0;
    }
    __syncthreads();
    long long c = (long long)blockIdx.x * kBlock + threadIdx.x;
    bool listed = false;
    if (c < a.C) {
    const int S = a.S, M = a.M;
    bool dead = false, mem = false;
    int prev = INT32_MAX, w0 = 0;
    // One pass over the stages, sixteen at a time (all their loads issued before the first is
    // used): the Lemma 1 and memory tests, and w as bytes for the ring kernels (wq_stride is a
    // multiple of 4; bytes past S are the padding stages of the kernel size the pipeline runs
    // in, w = 0).  The bytes of a candidate no ring kernel takes are never read.
    const WSource src = w_source(a, c);
    unsigned *const q = (unsigned *)(a.cand_wq + c * a.wq_stride);
    for (int s0 = 0; s0 < a.wq_stride; s0 += 16) {
        int wv[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) wv[j] = s0 + j < S ? clampw(w_at(src, s0 + j), M) : 0;
        unsigned packed[4] = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int s = s0 + j, ws = wv[j];
            if (s < S) {
                if (s == 0) w0 = ws;
                if (prev < ws) dead = true;
                if (a.mem_cap && ws + 1 > a.mem_cap[s]) mem = true;
                prev = ws;
            }
            packed[j / 4] |= (unsigned)(ws & 0xff) << (8 * (j % 4));
        }
        if (s0 + 16 <= a.wq_stride && (a.wq_stride & 15) == 0) {
            *(uint4 *)(q + s0 / 4) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (s0 + 4 * v < a.wq_stride) q[s0 / 4 + v] = packed[v];
        }
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
    listed = flag == ADAPTRA_FLAG_FEASIBLE && cls < kNumRingClasses;
    }
    // The feasible candidates that an on-chip kernel can take, as a list for the search of the
    // candidate-lanes kernel: one atomic per wavefront reserves its entries' places.
    if (a.live_list) {
        const unsigned long long votes = __ballot(listed);
        if (votes) {
            const int lane = threadIdx.x & 63;
            int base = 0;
            if (lane == __ffsll((long long)votes) - 1) base = atomicAdd(&a.status[48], __popcll(votes));
            base = __builtin_amdgcn_readlane(base, __ffsll((long long)votes) - 1);
            if (listed) a.live_list[base + __popcll(votes & ((1ull << lane) - 1ull))] = (int)c;
        }
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
    if (a.gate && *a.gate == 0) return;
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
    if (a.gate && *a.gate == 0) return;
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
    if (a.gate && *a.gate == 0) return;
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
            const WSource src = w_source(a, c);
            for (int s = 0; s < S; ++s) {
                wl[s * NT] = clampw(w_at(src, s), M);
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
    if (a.gate && *a.gate == 0) return;
    a.status[threadIdx.x] = 0;      // launched with 64 threads: all of status
}

// ---------------------------------------------------------------------------------------
// The paper's analytic planning, one thread per scenario (Section 4.2).
//   Algorithm 1 (initial planning, scenario independent; the first S threads): x_0 = x_max, the
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

// V consecutive scenarios per thread (1 or 4).  With 4 every access of a lane is 16 bytes (4 for
// the flags), so a wavefront's load or store covers 1 KiB of one row: the kernel walks 2(S-1)
// input rows and 2S-1 output rows at once, each K ints from the next, i.e. every access of a
// wavefront is to another page than the one before, and four times the bytes per access is a
// quarter of the address translations per byte.
template <int V>
struct SeedVec { int v[V]; };
template <int V>
__device__ __forceinline__ SeedVec<V> seed_load(const int *p) {
    SeedVec<V> r;
    if (V % 4 == 0) {
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
            const int4 t = reinterpret_cast<const int4 *>(p)[q];
            r.v[(4 * q) % V] = t.x; r.v[(4 * q + 1) % V] = t.y; r.v[(4 * q + 2) % V] = t.z; r.v[(4 * q + 3) % V] = t.w;
        }
    } else if (V == 2) {
        const int2 t = *reinterpret_cast<const int2 *>(p);
        r.v[0] = t.x; r.v[1 % V] = t.y;
    } else {
        r.v[0] = *p;
    }
    return r;
}
template <int V>
__device__ __forceinline__ void seed_store(int *p, const SeedVec<V> &r) {
    if (V % 4 == 0) {
#pragma unroll
        for (int q = 0; q < V / 4; ++q)
            reinterpret_cast<int4 *>(p)[q] = make_int4(r.v[(4 * q) % V], r.v[(4 * q + 1) % V], r.v[(4 * q + 2) % V], r.v[(4 * q + 3) % V]);
    } else if (V == 2) {
        *reinterpret_cast<int2 *>(p) = make_int2(r.v[0], r.v[1 % V]);
    } else {
        *p = r.v[0];
    }
}

// ceil(num / den), exact wherever it is below `clip`, some value >= clip otherwise (also for den
// = 0); 3 <= clip <= 2^15, num < 2^34.  Algorithm 2 only ever uses the ratio through min(., clip),
// so a single-precision estimate is enough to be within one of floor(num / den) in the range that
// matters (relative error below 2^-21, i.e. below 2^-6 up to clip + 1), and two exact products
// decide between the three values the ceiling can then have.  No integer division, no branch.
__device__ __forceinline__ int seed_ceil_ratio(unsigned long long num, unsigned den, int clip) {
    const float nf = fmaf((float)(unsigned)(num >> 32), 4294967296.f, (float)(unsigned)num);
    const float estimate = nf * __builtin_amdgcn_rcpf((float)den);      // inf or NaN for den = 0: fminf then gives clip
    const unsigned c = (unsigned)fminf(estimate, (float)clip);          // floor, at most clip
    const unsigned long long below = (unsigned long long)c * den;       // c - 1 < num / den < c + 2
    return (int)c + (num > below ? 1 : 0) + (num > below + den ? 1 : 0);
}

template <int V>
__global__ __launch_bounds__(kBlock) void k_seed(SeedArgs a) {
    const long long thread = (long long)blockIdx.x * kBlock + threadIdx.x;
    const long long k = thread * V;
    const int S = a.S;
    // Algorithm 1: the x_max - 1 units of slack go to the S - 1 links in equal shares, the
    // links nearest stage 0 taking the units left over; stage s holds x_max minus the slack of
    // the s links above it.  One thread per stage.
    if (thread < S && a.w_init) {
        const int s = (int)thread;
        int x = a.x_max;
        if (S > 1) {
            const int share = (a.x_max - 1) / (S - 1), left_over = (a.x_max - 1) % (S - 1);
            x -= s * share + (s < left_over ? s : left_over);
        }
        a.w_init[s] = x - 1;
    }
    if (k >= a.K) return;                       // V divides K when V > 1: a thread's scenarios all exist
    const long long K = a.K;
    // t_f + t_b of stage i as each of this thread's scenarios sees it (two non-negative int32: 32 bits unsigned)
    auto tau = [&](int i, unsigned (&out)[V]) {
        if (a.tfs) {
            const SeedVec<V> f = seed_load<V>(a.tfs + (long long)i * K + k), b = seed_load<V>(a.tbs + (long long)i * K + k);
#pragma unroll
            for (int v = 0; v < V; ++v) out[v] = (unsigned)f.v[v] + (unsigned)b.v[v];
        } else {
            const unsigned t = (unsigned)a.t_f[i] + (unsigned)a.t_b[i];
#pragma unroll
            for (int v = 0; v < V; ++v) out[v] = t;
        }
    };
    // One pass over the links, last to first, serves both outputs, so the delays are read once
    // (a link's slack needs the one below it only through the running sum x).
    const int *__restrict__ const cf = a.cf + k, *__restrict__ const cb = a.cb + k;
    int *__restrict__ const w_adapted = a.w_adapted ? a.w_adapted + k : nullptr;
    unsigned char *__restrict__ const not_absorbed = a.not_absorbed ? a.not_absorbed + k : nullptr;
    SeedVec<V> x;
#pragma unroll
    for (int v = 0; v < V; ++v) x.v[v] = 0;     // w = x - 1 of the last stage
    if (w_adapted) seed_store<V>(w_adapted + (long long)(S - 1) * K, x);
#pragma unroll
    for (int v = 0; v < V; ++v) x.v[v] = 1;
    const int clip = a.M - 2 * S;               // at most 2^15 (the limit on M)
    unsigned tau_next[V];
    if (S > 1) tau(S - 1, tau_next);
    for (int i = S - 2; i >= 0; --i) {
        unsigned tau_i[V];
        tau(i, tau_i);
        const SeedVec<V> f = seed_load<V>(cf + (long long)i * K), b = seed_load<V>(cb + (long long)i * K);
        // Eq. (1) with the current schedule's slack, which may be anything a difference of two int32 can be
        const long long slack_cur = not_absorbed ? (long long)a.w_cur[i] - a.w_cur[i + 1] : 0;
        const unsigned slack_abs = (unsigned)(slack_cur < 0 ? -slack_cur : slack_cur);
        unsigned long long flags = 0;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const unsigned den = tau_next[v];
            const unsigned long long num = (unsigned long long)tau_i[v] + ((unsigned)f.v[v] + (unsigned)b.v[v]);
            if (w_adapted) {
                int d = clip;                   // a ratio of at least 2 never gets below a clip of 2 or less
                if (clip > 2) {
                    const int ratio = seed_ceil_ratio(num, den, clip);
                    d = ratio < 2 ? 2 : (ratio < clip ? ratio : clip);
                }
                if (d < 0) d = 0;
                const int nx = x.v[v] + d;
                x.v[v] = nx > a.M ? a.M : nx;
            }
            if (not_absorbed) {
                // num <= slack_cur * den; with a negative slack the product is negative unless den = 0
                const bool absorbed = slack_cur >= 0 ? num <= (unsigned long long)slack_abs * den : (num | den) == 0;
                flags |= (absorbed ? 0ull : 1ull) << (8 * v);
            }
            tau_next[v] = tau_i[v];
        }
        if (w_adapted) {
            SeedVec<V> w;
#pragma unroll
            for (int v = 0; v < V; ++v) w.v[v] = x.v[v] - 1;
            seed_store<V>(w_adapted + (long long)i * K, w);
        }
        if (not_absorbed) {
            // little-endian: byte v = scenario k + v
            if (V == 8) *reinterpret_cast<unsigned long long *>(not_absorbed + (long long)i * K) = flags;
            else if (V == 4) *reinterpret_cast<unsigned *>(not_absorbed + (long long)i * K) = (unsigned)flags;
            else if (V == 2) *reinterpret_cast<unsigned short *>(not_absorbed + (long long)i * K) = (unsigned short)flags;
            else not_absorbed[(long long)i * K] = (unsigned char)flags;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Host side
thread_local int g_last_hip_error = 0;
// Test and measurement switches (adaptra_testing.h).  The kernel mode is one atomic word that
// every call reads once, when it fills its arguments; the timing events belong to the thread
// that set them.
std::atomic<int> g_kernel_mode{0};
thread_local hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;


struct Workspace {
    size_t off_flag, off_class, off_wq, off_live, off_keys, off_status, off_tpad, off_scratch, off_mkt, total;
    int wq_stride;
    long long general_threads;
};

// The general kernel keeps (2 S + M) ints per thread in scratch; bound the scratch to
// about 256 MiB by limiting the number of resident threads.  small: the 16 MiB that
// adaptra_best_static's fixed scratch sets aside for it (at least one block of threads; its
// size limits keep that inside the 16 MiB).
long long general_thread_count(int S, int M, bool small) {
    const long long per_thread = (2ll * S + M) * 4;
    long long nt = ((small ? 16ll : 256ll) << 20) / per_thread;
    if (nt > 65536) nt = 65536;
    if (nt < (small ? kBlock : 4096)) nt = small ? kBlock : 4096;
    return nt / kBlock * kBlock;
}

bool plan_workspace(int S, int M, long long C, long long K, Workspace *ws, bool with_mkt = true, bool small = false) {
    if (S < 1 || S > ADAPTRA_MAX_STAGES || M < 1 || M > ADAPTRA_MAX_MICROBATCHES) return false;
    if (C < 1 || C > INT32_MAX || K < 1 || K > INT32_MAX) return false;
    ws->wq_stride = (cand_kernel_stages(S) + 3) & ~3;
    ws->general_threads = general_thread_count(S, M, small);
    size_t o = 0;
    ws->off_flag = o;    o += adaptra_detail::align256((size_t)C);
    ws->off_class = o;   o += adaptra_detail::align256((size_t)C);
    ws->off_wq = o;      o += adaptra_detail::align256((size_t)C * ws->wq_stride);
    ws->off_live = o;    o += adaptra_detail::align256((size_t)C * 4);
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
ResolveKernel choose_kernel(int mode, int S, long long K, long long C, bool stage_times, bool paired) {
    const bool scen_ok = hot_kernel_stages(S) != 0 && !paired;
    const bool cand_ok = cand_kernel_stages(S) != 0 && !(stage_times && cand_kernel_stages(S) > kCandLanesStageTimesMax);
    switch (mode) {
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
                    Workspace *ws, bool with_mkt = true, bool small = false, bool derived = false) {
    if (!p || !cd || !sc) return ADAPTRA_EINVAL;
    if (!plan_workspace(p->S, p->M, cd->n, sc->n, ws, with_mkt, small)) return ADAPTRA_EINVAL;
    if (!p->t_f || !p->t_b || (!cd->w && !derived)) return ADAPTRA_EINVAL;
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
    a->live_list = nullptr;                // adaptra_best sets it: only the search walks the list
    a->gate = nullptr;
    a->tpad = (int *)(base + ws.off_tpad);
    a->scratch = (int *)(base + ws.off_scratch);
    a->mk_t = (int *)(base + ws.off_mkt);
    a->n_ktiles = (int)((sc->n + 63) / 64);
    a->kernel_mode = g_kernel_mode.load(std::memory_order_relaxed);
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

// Every grid of the evaluation path that grows with the problem, checked before the first
// launch, so that ADAPTRA_EINVAL always means that nothing was enqueued: the 64 x 64 tiles of
// the epilogue and of the search over an evaluation (only where an evaluation is written out),
// and the scenario-lanes kernel's blocks (never used in the paired form, whose kernels walk
// their tiles in a loop).
bool grids_fit(const KArgs &a, bool writes_evaluation) {
    const long long tiles = ((a.C + 63) / 64) * ((a.K + 63) / 64);
    const long long hot_blocks = a.pair_div ? 0 : (a.n_chunks * a.n_ktiles + kWavesPerBlock - 1) / kWavesPerBlock;
    return (!writes_evaluation || tiles <= INT32_MAX) && hot_blocks <= INT32_MAX;
}

template <bool BEST>
int launch_scen_lanes(const KArgs &a, int w_bound, hipStream_t st) {
    switch (hot_kernel_stages(a.S)) {
#define ADAPTRA_CASE(S_) case S_: return launch_scen_lanes_##S_(BEST, a, w_bound, st);
        ADAPTRA_CASE(2) ADAPTRA_CASE(4) ADAPTRA_CASE(8) ADAPTRA_CASE(12) ADAPTRA_CASE(16) ADAPTRA_CASE(24) ADAPTRA_CASE(32)
#undef ADAPTRA_CASE
        default: return ADAPTRA_EINVAL;
    }
}

template <bool BEST>
int launch_cand_lanes(const KArgs &a, int w_bound, hipStream_t st) {
    // The read-ahead form wherever it exists (kernel mode 3 asks for the plain one).
    const bool ahead = a.kernel_mode != 3;
    switch (cand_kernel_stages(a.S)) {
#define ADAPTRA_CASE(S_) case S_: return launch_cand_lanes_##S_(BEST, ahead, a, w_bound, st);
        ADAPTRA_CASE(2) ADAPTRA_CASE(4) ADAPTRA_CASE(8) ADAPTRA_CASE(12) ADAPTRA_CASE(16) ADAPTRA_CASE(24) ADAPTRA_CASE(32)
        ADAPTRA_CASE(48) ADAPTRA_CASE(64)
#undef ADAPTRA_CASE
        default: return ADAPTRA_EINVAL;
    }
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
    const ResolveKernel which = choose_kernel(a.kernel_mode, a.S, a.K, a.C, a.tfs != nullptr, a.pair_div != 0);
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

// Device address of the current GPU's copy of `scratch`.  Looked up on the first call on each
// device, with that device current, and kept: every GPU holds its own copy of the array at its
// own address.  (Two threads racing through the first call store the same value.)
constexpr int kMaxDevices = 64;
std::atomic<void *> g_static_scratch[kMaxDevices];
int static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return ADAPTRA_EINVAL;
    void *ptr = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr || ((uintptr_t)ptr & 255)) return ADAPTRA_EWORKSPACE;
        g_static_scratch[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return ADAPTRA_OK;
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
    if (!grids_fit(a, true)) return ADAPTRA_EINVAL;
    hipLaunchKernelGGL(k_zero_status, dim3(1), dim3(64), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_prepass, dim3(grid_for(a.C, INT32_MAX)), dim3(kBlock), 0, st, a);
    ADAPTRA_LAUNCH_CHECK();
    int direct = -1;
    rc = launch_resolve<false>(a, ws, cands->w_bound, st, &direct);
    if (rc) return rc;
    const long long tiles = ((a.C + 63) / 64) * ((a.K + 63) / 64);
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
    if (!grids_fit(a, true)) return ADAPTRA_EINVAL;
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
    if (!grids_fit(a, true)) return ADAPTRA_EINVAL;
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

int adaptra_best_static(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                        const adaptra_scenarios_t *scens,
                        int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                        uint64_t *out_hist, void *stream) {
    if (!params || !cands || !scens) return ADAPTRA_EINVAL;
    if (cands->n > ADAPTRA_STATIC_MAX_CANDIDATES || scens->n > ADAPTRA_STATIC_MAX_SCENARIOS ||
        params->M > ADAPTRA_STATIC_MAX_MICROBATCHES)
        return ADAPTRA_ELIMIT;
    void *ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc) return rc;
    // Every kernel takes the workspace through its arguments, exactly as in adaptra_best; what
    // must start at zero (status words, search keys, histogram) is cleared by the kernels of
    // the call itself, so the previous call's contents do not matter.
    return adaptra_detail::best(params, cands, scens, 0, out_best_idx, out_best_makespan, out_best_bubble,
                                out_hist, ptr, kStaticScratchBytes, stream, true);
}


}  // extern "C"

// adaptra_best proper.  pair_div > 0 (the guided search): candidate c belongs to scenario
// c / pair_div and is evaluated under that scenario only, by the general kernel (its lanes
// carry candidates, so each may have a scenario of its own).
int adaptra_detail::best(const adaptra_params_t *params, const adaptra_candidates_t *cands,
                         const adaptra_scenarios_t *scens, int pair_div,
                         int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
                         uint64_t *out_hist,
                         void *workspace, size_t workspace_bytes, void *stream, bool small_scratch, const int *gate,
                         const Neighbourhood *moves) {
    Workspace ws;
    int rc = validate_common(params, cands, scens, workspace, workspace_bytes, &ws, false, small_scratch, moves != nullptr);
    if (rc) return rc;
    if (moves && (!moves->point || moves->per_point < 1 || moves->K * moves->per_point < cands->n)) return ADAPTRA_EINVAL;
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
    a.live_list = (int *)((char *)workspace + ws.off_live);
    a.gate = gate;
    if (moves) a.moves = *moves;
    if (!grids_fit(a, false)) return ADAPTRA_EINVAL;
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
    // four scenarios per thread where every row then starts on a 16-byte boundary (4 for the flags)
    const uintptr_t align16 = (uintptr_t)a.cf | (uintptr_t)a.cb | (uintptr_t)a.tfs | (uintptr_t)a.tbs | (uintptr_t)a.w_adapted;
    if (a.K % 4 == 0 && (align16 & 15) == 0 && ((uintptr_t)a.not_absorbed & 3) == 0)
        hipLaunchKernelGGL((k_seed<4>), dim3(grid_for(a.K / 4, INT32_MAX)), dim3(kBlock), 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((k_seed<1>), dim3(grid_for(a.K, INT32_MAX)), dim3(kBlock), 0, (hipStream_t)stream, a);
    ADAPTRA_LAUNCH_CHECK();
    return ADAPTRA_OK;
}

int adaptra_set_kernel_mode(int mode) {
    if (mode < 0 || mode > 4) return -1;
    return g_kernel_mode.exchange(mode, std::memory_order_relaxed);
}

int adaptra_set_resolve_events(void *before, void *after) {
    g_ev_before = (hipEvent_t)before;
    g_ev_after = (hipEvent_t)after;
    return ADAPTRA_OK;
}

int adaptra_last_hip_error(void) { return g_last_hip_error; }

int adaptra_version(void) { return 1; }

}  // extern "C"

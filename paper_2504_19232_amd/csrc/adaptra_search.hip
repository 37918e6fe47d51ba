// adaptra_search.hip -- guided search over warm-up vectors for gfx950 (MI355X).
//
// A neighbourhood descent over the slacks Delta_i = w_i - w_{i+1} (the coordinates of the
// paper's Section 4.2 planning) for schedule spaces too large to enumerate.  Every scenario
// descends on its own; the work of a round is one batched evaluation of the analytical model
// (Section 3.1) over all scenarios' neighbourhoods at once -- the search of adaptra_best in
// its paired form, candidate c under scenario c / (moves + 1) -- so the kernels here only
// set up and move the points.
//
//   k_search_init      every scenario's point = w_start clamped, makespan = INT32_MAX
//   k_search_advance   a scenario adopts its best pool entry iff strictly better
//
// The pool -- entry k * (moves + 1) + j = the point of scenario k after move j, clamped -- is
// never written out: the evaluation's pre-pass derives each entry from the points (S x K ints,
// cached) where it would otherwise read the candidate array, and k_search_advance derives the
// winning entry once more.  Stored, the pool of a round was S x K x (moves + 1) ints written
// and read back (138 MB each way at 32 stages and 1024 scenarios).
//
// The host only needs to know when nothing moves any more, so it enqueues kRoundsPerCheck rounds
// at a time and reads the per-round move counts back once per batch: every kernel of a round
// (this file's and the evaluation's) exits at once when the round before it moved nothing.
//
// A scenario that did not move in a round is at rest for good: its pool, hence its best entry,
// would be the same in every later round.  Its pool entries then read as a vector that Lemma 1
// rules out (w_0 < w_1), which the evaluation flags in its pre-pass and never resolves, so the
// rounds get cheaper as the scenarios settle.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"
#include "adaptra_kernels.h"

namespace {

using adaptra_detail::blocks_for;
using adaptra_detail::hip_fail;
using adaptra_detail::kThreadsPerBlock;

struct SearchArgs {
    int S, M, nb, n_moves;
    long long K, C;               // scenarios; pool entries = K * (n_moves + 1)
    const int *w_start;
    int *cur_w, *cur_mk;          // [S][K], [K]: the outputs double as the state
    int *counters;                // [1] largest w[0] any point has had, [kMovedAt + i] scenarios that moved in round i of the batch
    const int *gate;              // the round before's move count, or null (first round of a batch): 0 = skip this round
    int *moved;                   // this round's move count
    int *active;                  // [K] 1 while the scenario is still moving
    const int *best_idx, *best_mk;
};

constexpr int kRoundsPerCheck = 8;      // rounds enqueued between two host read-backs
constexpr int kMovedAt = 8;             // counters[kMovedAt .. kMovedAt + kRoundsPerCheck)

__device__ __forceinline__ int clamp_w(int w, int M) { return w < 0 ? 0 : (w > M - 1 ? M - 1 : w); }

__global__ void k_search_init(SearchArgs a) {
    const long long k = (long long)blockIdx.x * kThreadsPerBlock + threadIdx.x;
    if (k >= a.K) return;
    for (int s = 0; s < a.S; ++s) a.cur_w[(long long)s * a.K + k] = clamp_w(a.w_start[s], a.M);
    a.cur_mk[k] = INT32_MAX;
    a.active[k] = 1;
}

__global__ void k_search_clear_moved(SearchArgs a) {
    if (threadIdx.x < kRoundsPerCheck) a.counters[kMovedAt + threadIdx.x] = 0;
}

__global__ void k_search_advance(SearchArgs a) {
    if (a.gate && *a.gate == 0) return;
    const long long k = (long long)blockIdx.x * kThreadsPerBlock + threadIdx.x;
    if (k >= a.K) return;
    const int bi = a.best_idx[k];
    if (bi >= 0 && a.best_mk[k] < a.cur_mk[k]) {
        int lo, hi, sign;                               // entry bi is this scenario's point after move bi mod (moves + 1)
        adaptra_detail::neighbourhood_move(a.nb, a.S, bi % (a.n_moves + 1), &lo, &hi, &sign);
        for (int s = 0; s < a.S; ++s) {
            int *const w = &a.cur_w[(long long)s * a.K + k];
            *w = clamp_w(*w + (s >= lo && s <= hi ? sign : 0), a.M);
        }
        a.cur_mk[k] = a.best_mk[k];
        atomicAdd(a.moved, 1);
        atomicMax(&a.counters[1], a.cur_w[k]);           // w is non-increasing over the stages of a feasible point
    } else {
        a.active[k] = 0;
    }
}


struct SearchPlan {
    int n_moves;
    long long c_max;
    size_t off_counters, off_active, off_best_idx, off_best_mk, off_best_ws, best_ws_bytes, total;
};

bool plan_search(const adaptra_params_t *p, long long K, int nb, SearchPlan *pl) {
    if (!p || p->S < 1 || p->S > ADAPTRA_MAX_STAGES || p->M < 1 || p->M > ADAPTRA_MAX_MICROBATCHES) return false;
    if (K < 1 || K > INT32_MAX || (nb != 0 && nb != 1)) return false;
    pl->n_moves = nb == 0 ? 2 * p->S : p->S * (p->S + 1);
    pl->c_max = K * (pl->n_moves + 1);
    if (pl->c_max > INT32_MAX) return false;
    pl->best_ws_bytes = adaptra_best_workspace_bytes(p, pl->c_max, K);
    if (pl->best_ws_bytes == 0) return false;
    size_t o = 0;
    pl->off_counters = o; o += 256;
    pl->off_active = o;   o += adaptra_detail::align256((size_t)K * 4);
    pl->off_best_idx = o; o += adaptra_detail::align256((size_t)K * 4);
    pl->off_best_mk = o;  o += adaptra_detail::align256((size_t)K * 4);
    pl->off_best_ws = o;  o += adaptra_detail::align256(pl->best_ws_bytes);
    pl->total = o;
    return true;
}

}  // namespace

extern "C" {

size_t adaptra_search_workspace_bytes(const adaptra_params_t *params, int64_t n_scen, int32_t neighbourhood) {
    SearchPlan pl;
    return plan_search(params, n_scen, neighbourhood, &pl) ? pl.total : 0;
}

int adaptra_search(const adaptra_params_t *params, const adaptra_scenarios_t *scens,
                   const int32_t *w_start, int32_t neighbourhood, int32_t max_iters,
                   int32_t *out_w, int32_t *out_makespan, int32_t *out_rounds, int64_t *out_evaluated,
                   void *workspace, size_t workspace_bytes, void *stream) {
    if (!params || !scens || !w_start || !out_w || !out_makespan || max_iters < 1) return ADAPTRA_EINVAL;
    SearchPlan pl;
    if (!plan_search(params, scens->n, neighbourhood, &pl)) return ADAPTRA_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < pl.total) return ADAPTRA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)workspace;
    SearchArgs a{};
    a.S = params->S; a.M = params->M; a.nb = neighbourhood; a.n_moves = pl.n_moves;
    a.K = scens->n;
    a.w_start = w_start;
    a.cur_w = out_w; a.cur_mk = out_makespan;
    a.counters = (int *)(base + pl.off_counters);
    a.active = (int *)(base + pl.off_active);
    a.C = pl.c_max;
    // resting scenarios can be marked where a vector with w_0 < w_1 exists: a stage 1, and M > 1
    const bool skip_resting = a.S > 1 && a.M > 1;
    const adaptra_detail::Neighbourhood moves{out_w, skip_resting ? a.active : nullptr, a.K, pl.n_moves + 1, neighbourhood};
    int *best_idx = (int *)(base + pl.off_best_idx), *best_mk = (int *)(base + pl.off_best_mk);
    a.best_idx = best_idx; a.best_mk = best_mk;
    adaptra_params_t bp = *params;
    bp.hist_bins = 0; bp.hist_shift = 0;
    const int kblocks = blocks_for(a.K, INT32_MAX);
    // An upper bound on every w in the pool lets the evaluation run as a single launch with the
    // smallest ring that fits: the largest w[0] any point has had (kept on the device, read
    // back with the round's move count), plus one for the move.
    int w_top = 0;
    {
        int w_host[ADAPTRA_MAX_STAGES];
        hipError_t e = hipMemcpyAsync(w_host, w_start, sizeof(int) * a.S, hipMemcpyDeviceToHost, st);
        if (e != hipSuccess) return hip_fail(e);
        if ((e = hipStreamSynchronize(st)) != hipSuccess) return hip_fail(e);
        for (int s = 0; s < a.S; ++s) {
            const int w = w_host[s] < 0 ? 0 : (w_host[s] > a.M - 1 ? a.M - 1 : w_host[s]);
            w_top = w > w_top ? w : w_top;
        }
    }

    hipLaunchKernelGGL(k_search_init, dim3(kblocks), dim3(kThreadsPerBlock), 0, st, a);
    ADAPTRA_CHECK_LAUNCH();
    {
        hipError_t e = hipMemcpyAsync(a.counters + 1, &w_top, sizeof(int), hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return hip_fail(e);
        if ((e = hipStreamSynchronize(st)) != hipSuccess) return hip_fail(e);     // w_top is on this stack
    }
    int rounds = 0;
    long long evaluated = 0, still_moving = a.K;
    for (bool settled = false; !settled && rounds < max_iters;) {
        const int n = max_iters - rounds < kRoundsPerCheck ? max_iters - rounds : kRoundsPerCheck;
        hipLaunchKernelGGL(k_search_clear_moved, dim3(1), dim3(64), 0, st, a);
        ADAPTRA_CHECK_LAUNCH();
        for (int i = 0; i < n; ++i) {
            a.gate = i == 0 ? nullptr : a.counters + kMovedAt + i - 1;
            a.moved = a.counters + kMovedAt + i;
            // steps 1 and 2: every scenario's point and its neighbours, each under its own scenario,
            // and the best entry per scenario.  No w in the pool exceeds the largest w[0] any point
            // had at the last read-back by more than one per round since.
            const long long top = (long long)w_top + i + 1;
            const adaptra_candidates_t pool{a.C, nullptr, (int32_t)(top > a.M - 1 ? a.M - 1 : top)};
            int rc = adaptra_detail::best(&bp, &pool, scens, pl.n_moves + 1, best_idx, best_mk, nullptr, nullptr,
                                          base + pl.off_best_ws, pl.best_ws_bytes, stream, false, a.gate, &moves);
            if (rc) return rc;
            // step 3: move
            hipLaunchKernelGGL(k_search_advance, dim3(kblocks), dim3(kThreadsPerBlock), 0, st, a);
            ADAPTRA_CHECK_LAUNCH();
        }
        int back[kMovedAt + kRoundsPerCheck] = {};
        hipError_t e = hipMemcpyAsync(back, a.counters, sizeof(back), hipMemcpyDeviceToHost, st);
        if (e != hipSuccess) return hip_fail(e);
        if ((e = hipStreamSynchronize(st)) != hipSuccess) return hip_fail(e);
        w_top = back[1];
        for (int i = 0; i < n && !settled; ++i) {         // rounds behind one that moved nothing were skipped
            ++rounds;
            evaluated += (skip_resting ? still_moving : a.K) * (pl.n_moves + 1);
            still_moving = back[kMovedAt + i];
            settled = still_moving == 0;
        }
    }
    if (out_rounds) *out_rounds = rounds;
    if (out_evaluated) *out_evaluated = evaluated;
    return ADAPTRA_OK;
}

}  // extern "C"

// adaptra_internal.h -- host-side helpers shared by the library's source files (not part of
// the C ABI).
#ifndef ADAPTRA_INTERNAL_H
#define ADAPTRA_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "adaptra.h"

namespace adaptra_detail {

constexpr int kThreadsPerBlock = 256;

// Records the hipError_t for adaptra_last_hip_error and returns ADAPTRA_EHIP.
int hip_fail(hipError_t e);

// Candidates that are not stored but derived: candidate c is the point of scenario
// c / per_point after move c % per_point of the guided search's neighbourhood (see
// neighbourhood_move), or -- for a scenario whose `active` word is 0 -- a vector that Lemma 1
// rules out, which no kernel ever resolves.  point == nullptr: the candidates are an array.
struct Neighbourhood {
    const int *point;             // DEVICE [S][K]
    const int *active;            // DEVICE [K] or null (every scenario active)
    long long K;
    int per_point;                // moves + 1
    int nb;                       // 0: prefix ranges, 1: all ranges
};

// adaptra_best with more arguments: pair_div > 0 evaluates candidate c under scenario
// c / pair_div only (0: every candidate under every scenario); small_scratch plans the
// workspace with the general kernel's share held to 16 MiB (adaptra_best_static); gate, a
// DEVICE int, makes every kernel of the call exit at once when it is 0 at that time (the guided
// search enqueues several rounds between two host read-backs); moves, when set, replaces
// cands->w (which is then not read and may be null).
int best(const adaptra_params_t *params, const adaptra_candidates_t *cands, const adaptra_scenarios_t *scens,
         int pair_div, int32_t *out_best_idx, int32_t *out_best_makespan, int32_t *out_best_bubble,
         uint64_t *out_hist, void *workspace, size_t workspace_bytes, void *stream, bool small_scratch = false,
         const int *gate = nullptr, const Neighbourhood *moves = nullptr);

// Workspace sections start on 256-byte boundaries.
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline int blocks_for(long long n, long long cap) {
    long long g = (n + kThreadsPerBlock - 1) / kThreadsPerBlock;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace adaptra_detail

#define ADAPTRA_CHECK_LAUNCH()                                             \
    do {                                                                   \
        hipError_t e_ = hipGetLastError();                                 \
        if (e_ != hipSuccess) return adaptra_detail::hip_fail(e_);         \
    } while (0)

#endif  // ADAPTRA_INTERNAL_H

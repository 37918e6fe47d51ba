// Drives the HOST code of every entry point of the library -- argument checks, workspace
// planning, kernel choice, launch shapes -- over seeded problem sizes, in a build with
// -fsanitize=address,undefined in which every HIP call is a stub that succeeds
// (tests/hip_launch_stub.h).  Device pointers are made-up addresses; host code never
// dereferences them.  Prints a checksum; tests/test_host_sanitizers.py builds and runs it.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "adaptra.h"
#include "adaptra_testing.h"

static uint64_t state = 0x9e3779b97f4a7c15ull;
static int64_t draw(int64_t lo, int64_t hi) {          // xorshift64, inclusive range
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return lo + (int64_t)(state % (uint64_t)(hi - lo + 1));
}
#define EXPECT(cond)                                                             \
    do {                                                                         \
        if (!(cond)) { fprintf(stderr, "line %d: %s failed\n", __LINE__, #cond); exit(1); } \
    } while (0)

int main() {
    int32_t *const dev = (int32_t *)(uintptr_t)0x7000000000ull;      // "device" addresses, never read here
    void *const ws = (void *)(uintptr_t)0x7100000000ull;             // 256-byte aligned
    uint64_t sum = 0;
    for (int mode = 0; mode <= 4; ++mode) {
        EXPECT(adaptra_set_kernel_mode(mode) >= 0);
        for (int rep = 0; rep < 400; ++rep) {
            adaptra_params_t p = {};
            p.S = (int32_t)draw(1, 64);
            p.M = (int32_t)(rep % 7 == 0 ? draw(1, 32768) : draw(1, 300));
            p.t_f = dev; p.t_b = dev; p.mem_cap = rep % 3 ? dev : nullptr;
            p.hist_bins = rep % 4 == 0 ? (int32_t)draw(1, 400) : 0;
            p.hist_shift = (int32_t)draw(0, 30);
            adaptra_candidates_t c = {rep % 11 == 0 ? draw(1, 2147483647) : draw(1, 200000), dev, rep % 2 ? (int32_t)draw(0, 400) : -1};
            adaptra_scenarios_t s = {rep % 13 == 0 ? draw(1, 3000000) : draw(1, 5000), dev, dev, rep % 5 == 0 ? dev : nullptr, rep % 5 == 0 ? dev : nullptr};
            const size_t need = adaptra_workspace_bytes(&p, c.n, s.n), need_best = adaptra_best_workspace_bytes(&p, c.n, s.n);
            EXPECT(need > 0 && need % 256 == 0 && need_best > 0 && need_best <= need);
            sum += need;
            uint64_t *hist = p.hist_bins ? (uint64_t *)dev : nullptr;
            int rc = adaptra_eval(&p, &c, &s, dev, rep % 2 ? dev : nullptr, (uint8_t *)dev, ws, need, nullptr);
            EXPECT(rc == ADAPTRA_OK || rc == ADAPTRA_EINVAL);            // EINVAL: more tiles than a grid holds
            sum += (uint64_t)rc;
            rc = adaptra_best(&p, &c, &s, dev, dev, dev, hist, ws, need_best, nullptr);
            EXPECT(rc == ADAPTRA_OK || rc == ADAPTRA_EINVAL);
            rc = adaptra_eval_best(&p, &c, &s, dev, dev, (uint8_t *)dev, dev, dev, dev, hist, ws, need, nullptr);
            EXPECT(rc == ADAPTRA_OK || rc == ADAPTRA_EINVAL);
            EXPECT(adaptra_eval(&p, &c, &s, dev, dev, (uint8_t *)dev, ws, need - 1, nullptr) == ADAPTRA_EWORKSPACE);
            EXPECT(adaptra_best(&p, &c, &s, dev, dev, dev, hist, (char *)ws + 8, need_best, nullptr) == ADAPTRA_EWORKSPACE);
            EXPECT(adaptra_check_inputs(&p, &c, &s, ws, need, nullptr) == ADAPTRA_OK);   // the stubbed read-back is all zeros
            rc = adaptra_best_static(&p, &c, &s, dev, dev, dev, hist, nullptr);
            const bool within = c.n <= ADAPTRA_STATIC_MAX_CANDIDATES && s.n <= ADAPTRA_STATIC_MAX_SCENARIOS && p.M <= ADAPTRA_STATIC_MAX_MICROBATCHES;
            EXPECT(within ? rc == ADAPTRA_OK : rc == ADAPTRA_ELIMIT);
            EXPECT(adaptra_seed(&p, &s, (int32_t)draw(1, 100), dev, dev, dev, (uint8_t *)dev, nullptr) == ADAPTRA_OK);
            if (c.n <= 4096 && s.n <= 4096) {
                const size_t sens = adaptra_sensitivity_workspace_bytes(&p, c.n, s.n);
                EXPECT(sens > 0);
                rc = adaptra_sensitivity(&p, &c, &s, 1, dev, (uint8_t *)dev, dev, ws, sens, nullptr);
                EXPECT(rc == ADAPTRA_OK);
                EXPECT(adaptra_sensitivity(&p, &c, &s, 0, dev, (uint8_t *)dev, dev, ws, sens, nullptr) == ADAPTRA_EINVAL);
            }
            for (int nb = 0; nb <= 1; ++nb) {
                const size_t srch = adaptra_search_workspace_bytes(&p, s.n, nb);
                if (srch == 0) continue;                              // pool beyond 2^31 - 1 entries
                int32_t rounds = -1; int64_t evaluated = -1;
                rc = adaptra_search(&p, &s, dev, nb, 5, dev, dev, &rounds, &evaluated, ws, srch, nullptr);
                if (rc != ADAPTRA_OK || rounds != 1 || evaluated <= 0)
                    fprintf(stderr, "search: rc %d rounds %d evaluated %lld S %d M %d K %lld nb %d\n", rc, rounds, (long long)evaluated, p.S, p.M, (long long)s.n, nb);
                EXPECT(rc == ADAPTRA_OK && rounds == 1 && evaluated > 0);     // the stubbed read-back says nothing moved
                EXPECT(adaptra_search(&p, &s, dev, nb, 5, dev, dev, nullptr, nullptr, ws, srch - 256, nullptr) == ADAPTRA_EWORKSPACE);
                sum += srch;
            }
            const size_t zb = adaptra_zb_workspace_bytes(&p, c.n, s.n);
            if (zb) {
                for (int64_t plan = -1; plan <= 0; ++plan) {
                    rc = adaptra_zb_eval(&p, dev, &c, &s, plan, dev, rep % 2 ? dev : nullptr, ws, zb, nullptr);
                    EXPECT(rc == ADAPTRA_OK);
                }
                EXPECT(adaptra_zb_check_inputs(&p, dev, &c, &s, ws, zb, nullptr) == ADAPTRA_OK);
                EXPECT(adaptra_zb_eval(&p, dev, &c, &s, s.n, dev, dev, ws, zb, nullptr) == ADAPTRA_EINVAL);
                sum += zb;
            }
        }
    }
    // out-of-range sizes
    adaptra_params_t bad = {};
    bad.S = 65; bad.M = 8;
    EXPECT(adaptra_workspace_bytes(&bad, 10, 10) == 0 && adaptra_zb_workspace_bytes(&bad, 10, 10) == 0);
    bad.S = 8; bad.M = 32769;
    EXPECT(adaptra_workspace_bytes(&bad, 10, 10) == 0 && adaptra_search_workspace_bytes(&bad, 10, 0) == 0);
    int64_t n = 0;
    for (int mix = -1; mix <= ADAPTRA_PROBE_MIXES; ++mix)
        EXPECT(adaptra_valu_probe(mix, 4, 2, dev, nullptr, &n) == (mix < 0 || mix >= ADAPTRA_PROBE_MIXES ? ADAPTRA_EINVAL : ADAPTRA_OK));
    EXPECT(adaptra_set_kernel_mode(0) >= 0 && adaptra_set_kernel_mode(9) == -1);
    printf("checksum %llu\n", (unsigned long long)sum);
    return 0;
}

/*
 * Drives the C oracle (both simulators) over small seeded inputs, for a build with
 * -fsanitize=address,undefined: heap errors, leaks of the simulator state and undefined
 * integer behaviour in the test infrastructure itself would otherwise go unnoticed.
 * Prints a checksum; tests/test_oracle_sanitizers.py builds and runs it.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t adaptra_oracle_eval(int S, int M, const int32_t *t_f, const int32_t *t_b, const int32_t *mem_cap,
                            int64_t n_cand, const int32_t *w, int64_t n_scen, const int32_t *c_fwd,
                            const int32_t *c_bwd, int64_t n_pairs, const int64_t *pair_cand,
                            const int64_t *pair_scen, int32_t *out_makespan, int32_t *out_bubble,
                            uint8_t *out_flag, int32_t *out_peak, int n_threads);
int adaptra_oracle_timeline(int S, int M, const int32_t *t_f, const int32_t *t_b, const int32_t *w,
                            const int32_t *cf, const int32_t *cb, int64_t *start_f, int64_t *fin_f,
                            int64_t *start_b, int64_t *fin_b, int64_t *idle, int32_t *peak, int64_t *makespan);
int64_t adaptra_oracle_zb(int S, int N, int mode, const int32_t *tF, const int32_t *tB, const int32_t *tW,
                          const int32_t *x, const int32_t *in_order, const int32_t *cf, const int32_t *cb,
                          int32_t *out_order, int64_t *out_start, int64_t *out_fin, int64_t *out_idle);
int64_t adaptra_oracle_zb_batch(int S, int N, const int32_t *tF, const int32_t *tB, const int32_t *tW,
                                int64_t n_cand, const int32_t *x, int64_t n_scen, const int32_t *cf,
                                const int32_t *cb, int32_t *out_makespan, int32_t *out_idle);

static uint64_t state = 88172645463325252ull;
static int32_t draw(int32_t lo, int32_t hi) {          /* xorshift64, inclusive range */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return lo + (int32_t)(state % (uint64_t)(hi - lo + 1));
}
static int32_t *ints(int64_t n) { return (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1)); }

int main(void) {
    uint64_t sum = 0;
    for (int trial = 0; trial < 60; ++trial) {
        const int S = draw(1, 9), M = draw(1, 12), C = draw(1, 20), K = draw(1, 6), L = S - 1;
        int32_t *t_f = ints(S), *t_b = ints(S), *t_w = ints(S), *cap = ints(S), *w = ints((int64_t)S * C), *x = ints((int64_t)S * C);
        int32_t *cf = ints((int64_t)L * K), *cb = ints((int64_t)L * K);
        for (int i = 0; i < S; ++i) { t_f[i] = draw(1, 300); t_b[i] = draw(1, 500); t_w[i] = draw(0, 200); cap[i] = draw(1, 2 * S + 2); }
        for (int64_t i = 0; i < (int64_t)S * C; ++i) { w[i] = draw(-1, M + 2); x[i] = (w[i] < 0 ? 0 : (w[i] > M - 1 ? M - 1 : w[i])) + 1; }
        for (int64_t i = 0; i < (int64_t)L * K; ++i) { cf[i] = draw(0, 4000); cb[i] = draw(0, 4000); }
        const int64_t P = (int64_t)C * K;
        int32_t *mk = ints(P), *bub = ints(S * P), *peak = ints(S * P);
        uint8_t *flag = (uint8_t *)malloc((size_t)P);
        if (adaptra_oracle_eval(S, M, t_f, t_b, trial % 2 ? cap : NULL, C, w, K, cf, cb, P, NULL, NULL, mk, bub, flag, peak,
                                1 + trial % 3) < 0) return 2;
        for (int64_t p = 0; p < P; ++p) sum += (uint64_t)mk[p] + flag[p];
        /* one timeline and one ZeroBubble generate-then-replay per trial */
        int64_t *sf = malloc(sizeof(int64_t) * S * M), *ff = malloc(sizeof(int64_t) * S * M), *sb = malloc(sizeof(int64_t) * S * M),
                *fb = malloc(sizeof(int64_t) * S * M), *idle = malloc(sizeof(int64_t) * S), span = 0;
        int32_t *pk = ints(S), *w0 = ints(S), *x0 = ints(S), *cf0 = ints(L), *cb0 = ints(L);
        for (int i = 0; i < S; ++i) { w0[i] = w[(int64_t)i * C]; x0[i] = x[(int64_t)i * C]; }
        for (int i = 0; i < L; ++i) { cf0[i] = cf[(int64_t)i * K]; cb0[i] = cb[(int64_t)i * K]; }
        if (adaptra_oracle_timeline(S, M, t_f, t_b, w0, cf0, cb0, sf, ff, sb, fb, idle, pk, &span) < 0) return 3;
        sum += (uint64_t)span;
        int32_t *order = ints(3 * S * M);
        int64_t *zs = malloc(sizeof(int64_t) * 3 * S * M), *zf = malloc(sizeof(int64_t) * 3 * S * M), *zi = malloc(sizeof(int64_t) * S);
        const int64_t gen = adaptra_oracle_zb(S, M, 0, t_f, t_b, t_w, x0, NULL, cf0, cb0, order, zs, zf, zi);
        const int64_t rep = adaptra_oracle_zb(S, M, 1, t_f, t_b, t_w, NULL, order, cf0, cb0, NULL, zs, zf, zi);
        if (gen != rep) return 4;                       /* a plan replayed under its own delays */
        sum += (uint64_t)gen;
        int32_t *zmk = ints(P), *zidle = ints(S * P);
        if (adaptra_oracle_zb_batch(S, M, t_f, t_b, t_w, C, x, K, cf, cb, zmk, zidle) != 0) return 5;
        for (int64_t p = 0; p < P; ++p) sum += (uint64_t)zmk[p];
        free(t_f); free(t_b); free(t_w); free(cap); free(w); free(x); free(cf); free(cb); free(mk); free(bub); free(peak);
        free(flag); free(sf); free(ff); free(sb); free(fb); free(idle); free(pk); free(w0); free(x0); free(cf0); free(cb0);
        free(order); free(zs); free(zf); free(zi); free(zmk); free(zidle);
    }
    printf("checksum %llu\n", (unsigned long long)sum);
    return 0;
}

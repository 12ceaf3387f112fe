/* Runs the two C flow solvers of the CPU checker under the sanitizers on small seeded instances (uniform and
 * tie-heavy rewards, tight, slack and short capacity, per-token k with zeros) and checks that they agree where both
 * apply.  The literal graph solves every case; the contracted form needs room for every token's k. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int mcmf_literal_kc(const int64_t *q, int T, int E, const int *kvec, const int *caps, uint8_t *P, int64_t *flow,
                    int64_t *total, int64_t *n_arcs);
int mcmf_contracted_kc(const int64_t *q, int T, int E, const int *kvec, const int *caps, uint8_t *P, int64_t *prices,
                       int64_t *flow, int64_t *total, int64_t *n_paths, int64_t *n_hops);

static uint64_t state = 88172645463325252ull;
static uint32_t rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (uint32_t)(state >> 11);
}

int main(void)
{
    int cases = 0;
    for (int rep = 0; rep < 60; ++rep) {
        const int T = 1 + (int)(rnd() % 40), E = 1 + (int)(rnd() % 9);
        const int kmax = 1 + (int)(rnd() % (unsigned)E);
        const int ties = rep % 3 == 0;
        int64_t *q = malloc(sizeof(int64_t) * (size_t)T * E);
        int *kvec = malloc(sizeof(int) * (size_t)T), *caps = malloc(sizeof(int) * (size_t)E);
        uint8_t *P1 = malloc((size_t)T * E), *P2 = malloc((size_t)T * E);
        int64_t *prices = malloc(sizeof(int64_t) * (size_t)E);
        if (!q || !kvec || !caps || !P1 || !P2 || !prices) return 2;
        for (int i = 0; i < T * E; ++i) q[i] = ties ? (int64_t)(rnd() % 4) : (int64_t)(rnd() % 2000000) - 500000;
        long long demand = 0, room = 0;
        for (int i = 0; i < T; ++i) {
            kvec[i] = rep % 2 ? kmax : (int)(rnd() % (unsigned)(kmax + 1));
            demand += kvec[i];
        }
        for (int j = 0; j < E; ++j) {
            caps[j] = (int)(rnd() % (unsigned)(2 * T * kmax / E + 2));
            room += caps[j] < T ? caps[j] : T;
        }
        int64_t f1 = 0, t1 = 0, arcs = 0, f2 = 0, t2 = 0, np = 0, nh = 0;
        if (mcmf_literal_kc(q, T, E, kvec, caps, P1, &f1, &t1, &arcs) != 0) return 3;
        if (arcs != (int64_t)T + E + (int64_t)T * E) return 4;           /* Table 1: n + e + n*e arcs */
        if (demand <= room) {
            const int rc = mcmf_contracted_kc(q, T, E, kvec, caps, P2, prices, &f2, &t2, &np, &nh);
            if (rc == 0 && (f1 != f2 || t1 != t2)) {
                fprintf(stderr, "case %d: literal (%lld, %lld) != contracted (%lld, %lld)\n", rep, (long long)f1,
                        (long long)t1, (long long)f2, (long long)t2);
                return 5;
            }
            if (rc == 0) ++cases;
        }
        free(q); free(kvec); free(caps); free(P1); free(P2); free(prices);
    }
    printf("flow solvers under sanitizers: ok (%d cases compared)\n", cases);
    return cases > 10 ? 0 : 6;
}

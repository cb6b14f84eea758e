/*
 * The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer.
 *
 * Built by tests/test_oracle_sanitized.py together with the two files of
 * oracle/ (all three compiled with -fsanitize=address,undefined and
 * -fno-sanitize-recover), so that an out-of-bounds access, a use after free, a
 * signed overflow or a bad shift anywhere in the checker ends the program with
 * a report.  It replays a file of cases (a stream of int32 written by the test):
 *
 *   n_cases, then per case:
 *     variant (0 joint, 1 vertical), queue_model, profile_form,
 *     S, c_max, n_batch, batch_sizes[n_batch], r_max, tick, slo_max, N,
 *     enumerate (1: compare every instance with the exhaustive enumeration),
 *     expect (1: expected outputs follow the inputs),
 *     coef[N][S][cs], lambda[N], slo[N], r_fixed[N][S] (vertical only),
 *     and, if expect: status[N], cost[N], ticks[N], cfg[N][S][3].
 *
 * Every case goes through the candidate tables and the solve; vertical cases
 * also through the solve with fallback, joint ones through the stability test
 * (predicted rate = rate + 7) and the solve with every model pinned to one core.
 * Exit status 0 and "sanitized ok" when nothing disagrees.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int themis_oracle_set_model(int32_t, int32_t);
int themis_bruteforce_set_model(int32_t, int32_t);
int themis_oracle_candidates(int32_t, int32_t, int32_t, const int32_t *, int32_t, int32_t, int32_t,
                             int32_t, const int32_t *, const int32_t *, const int32_t *,
                             const int32_t *, int32_t, int32_t, int32_t *, int32_t *, int32_t *);
int themis_oracle_solve_ex(int32_t, int32_t, int32_t, const int32_t *, int32_t, int32_t, int32_t,
                           int32_t, const int32_t *, const int32_t *, const int32_t *,
                           const int32_t *, const int32_t *, int32_t, int32_t, int32_t *,
                           int32_t *, int32_t *, int32_t *);
int themis_oracle_vertical_fallback(int32_t, int32_t, int32_t, const int32_t *, int32_t, int32_t,
                                    int32_t, int32_t, const int32_t *, const int32_t *,
                                    const int32_t *, const int32_t *, int32_t, int32_t, int32_t *,
                                    int32_t *, int32_t *, int32_t *, int32_t *, int32_t *,
                                    int32_t *, int32_t *, int32_t *);
int themis_oracle_stability(int32_t, int32_t, int32_t, const int32_t *, int32_t, int32_t, int32_t,
                            int32_t, const int32_t *, const int32_t *, const int32_t *,
                            const int32_t *, const int32_t *, int32_t, int32_t, int32_t *,
                            int32_t *, int32_t *, int32_t *, int32_t *);
int themis_bruteforce_ex(int32_t, int32_t, int32_t, const int32_t *, int32_t, int32_t,
                         const int32_t *, int32_t, int32_t, const int32_t *, const int32_t *,
                         int32_t *, int32_t *, int32_t *, int64_t *);

static int32_t *take(int32_t **at, const int32_t *end, size_t n)
{
    int32_t *p = *at;
    if ((size_t)(end - p) < n) {
        fprintf(stderr, "case file truncated\n");
        exit(3);
    }
    *at = p + n;
    return p;
}

/* exact-size heap copies, so that a read one past an array is seen */
static int32_t *dup32(const int32_t *src, size_t n)
{
    int32_t *p = (int32_t *)malloc(n ? n * sizeof *p : 1);
    if (!p) exit(4);
    if (n) memcpy(p, src, n * sizeof *p);
    return p;
}

static int32_t *new32(size_t n)
{
    int32_t *p = (int32_t *)calloc(n ? n : 1, sizeof *p);
    if (!p) exit(4);
    return p;
}

int main(int argc, char **argv)
{
    FILE *f;
    long bytes;
    int32_t *buf, *at, *end;
    int n_cases, cs_i, failures = 0;
    long n_inst_total = 0, n_enum = 0;
    if (argc != 2) return 2;
    f = fopen(argv[1], "rb");
    if (!f) return 2;
    fseek(f, 0, SEEK_END);
    bytes = ftell(f);
    fseek(f, 0, SEEK_SET);
    buf = (int32_t *)malloc((size_t)bytes + 4);
    if (!buf || fread(buf, 1, (size_t)bytes, f) != (size_t)bytes) return 2;
    fclose(f);
    at = buf;
    end = buf + bytes / 4;
    n_cases = *take(&at, end, 1);
    for (cs_i = 0; cs_i < n_cases; ++cs_i) {
        const int32_t *h = take(&at, end, 6);
        const int variant = h[0], qm = h[1], pf = h[2], S = h[3], c_max = h[4], nb = h[5];
        const int cs = pf ? 6 : 5, K = c_max * nb;
        int32_t *bs = dup32(take(&at, end, (size_t)nb), (size_t)nb);
        const int32_t *g = take(&at, end, 6);
        const int r_max = g[0], tick = g[1], slo_max = g[2], N = g[3], enumerate = g[4],
                  expect = g[5];
        int32_t *coef = dup32(take(&at, end, (size_t)N * S * cs), (size_t)N * S * cs);
        int32_t *lam = dup32(take(&at, end, (size_t)N), (size_t)N);
        int32_t *slo = dup32(take(&at, end, (size_t)N), (size_t)N);
        int32_t *rf = variant ? dup32(take(&at, end, (size_t)N * S), (size_t)N * S) : NULL;
        int32_t *status = new32((size_t)N), *cost = new32((size_t)N), *ticks = new32((size_t)N);
        int32_t *cfg = new32((size_t)N * S * 3);
        int32_t *lt_t = new32((size_t)N * S * K), *co_t = new32((size_t)N * S * K),
                *r_t = new32((size_t)N * S * K);
        int i, x;
        if (themis_oracle_set_model(qm, pf) || themis_bruteforce_set_model(qm, pf)) return 5;
        if (themis_oracle_candidates(S, c_max, nb, bs, r_max, tick, slo_max, 0, coef, lam, slo, rf,
                                     0, N, lt_t, co_t, r_t))
            return 5;
        if (themis_oracle_solve_ex(S, c_max, nb, bs, r_max, tick, slo_max, 0, coef, lam, slo, rf,
                                   NULL, 0, N, status, cost, ticks, cfg))
            return 5;
        n_inst_total += N;
        if (expect) {
            const int32_t *e_st = take(&at, end, (size_t)N), *e_co = take(&at, end, (size_t)N),
                          *e_tk = take(&at, end, (size_t)N),
                          *e_cfg = take(&at, end, (size_t)N * S * 3);
            for (i = 0; i < N; ++i)
                if (status[i] != e_st[i] || cost[i] != e_co[i] || ticks[i] != e_tk[i] ||
                    memcmp(cfg + (size_t)i * S * 3, e_cfg + (size_t)i * S * 3,
                           sizeof(int32_t) * (size_t)S * 3)) {
                    if (failures++ < 10)
                        fprintf(stderr, "case %d instance %d: differs from the expected values\n",
                                cs_i, i);
                }
        }
        if (enumerate)
            for (i = 0; i < N; ++i) {
                int32_t b_cost = 0, b_ticks = 0;
                int32_t *b_cfg = new32((size_t)S * 3);
                int64_t visited = 0;
                int rc;
                if (status[i] == 2) {  /* invalid input: nothing to enumerate */
                    free(b_cfg);
                    continue;
                }
                rc = themis_bruteforce_ex(S, c_max, nb, bs, r_max, tick, coef + (size_t)i * S * cs,
                                          lam[i], slo[i], rf ? rf + (size_t)i * S : NULL, NULL,
                                          &b_cost, &b_ticks, b_cfg, &visited);
                ++n_enum;
                if (rc != status[i] || b_cost != cost[i] || b_ticks != ticks[i] ||
                    memcmp(b_cfg, cfg + (size_t)i * S * 3, sizeof(int32_t) * (size_t)S * 3)) {
                    if (failures++ < 10)
                        fprintf(stderr, "case %d instance %d: solve and enumeration differ\n", cs_i,
                                i);
                }
                free(b_cfg);
            }
        if (variant) {
            int32_t *lv = new32((size_t)N), *st_h = new32((size_t)N), *co_h = new32((size_t)N),
                    *tk_h = new32((size_t)N), *cfg_h = new32((size_t)N * S * 3);
            if (themis_oracle_vertical_fallback(S, c_max, nb, bs, r_max, tick, slo_max, 0, coef, lam,
                                                slo, rf, 0, N, status, cost, ticks, cfg, lv, st_h,
                                                co_h, tk_h, cfg_h))
                return 5;
            for (i = 0; i < N; ++i)
                if (lv[i] < 0 || lv[i] > lam[i]) ++failures;
            free(lv), free(st_h), free(co_h), free(tk_h), free(cfg_h);
        } else {
            int32_t *pred = new32((size_t)N), *stable = new32((size_t)N);
            int32_t *one = new32((size_t)N * S);
            for (i = 0; i < N; ++i) pred[i] = lam[i] + 7;
            for (x = 0; x < N * S; ++x) one[x] = 1;
            if (themis_oracle_stability(S, c_max, nb, bs, r_max, tick, slo_max, 0, coef, lam, pred,
                                        slo, NULL, 0, N, stable, status, cost, ticks, cfg))
                return 5;
            if (themis_oracle_solve_ex(S, c_max, nb, bs, r_max, tick, slo_max, 0, coef, lam, slo,
                                       NULL, one, 0, N, status, cost, ticks, cfg))
                return 5;
            free(pred), free(stable), free(one);
        }
        free(bs), free(coef), free(lam), free(slo), free(rf);
        free(status), free(cost), free(ticks), free(cfg), free(lt_t), free(co_t), free(r_t);
    }
    free(buf);
    if (failures) {
        fprintf(stderr, "%d disagreements\n", failures);
        return 1;
    }
    printf("sanitized ok: %d cases, %ld instances, %ld enumerated\n", n_cases, n_inst_total, n_enum);
    return 0;
}

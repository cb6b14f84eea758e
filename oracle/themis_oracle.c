/*
 * CPU checker for the batched autoscaling solve -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C.  Nothing in the product path may call this
 * file; it exists so that tests and the benchmark's CPU-baseline leg have an
 * independent answer to compare the GPU library with.  It shares no source,
 * header, table or helper with the GPU code.
 *
 * What it computes (per instance = one pipeline at one arrival rate):
 * the integer program of Section 4.3 (Eq. 6)
 *
 *     minimise   sum_s n_s * c_s
 *     subject to sum_s l_s(b_s,c_s) + q_s(b_s) <= SLO          (Eq. 5)
 *                lambda <= h_s(b_s,c_s) * n_s   for every s
 *                b_s, c_s, n_s positive integers
 *
 * solved the way Section 4.4 solves it: a dynamic program that adds the
 * pipeline's models one at a time and, for every latency budget on a grid,
 * splits the budget between the current model and the rest (Algorithm 1 for
 * the vertical case where n_s is given, Algorithm 2 for the derived instance
 * count; the joint solve is Algorithm 1's (c,b) loop with Algorithm 2's
 * instance count folded into each candidate).  Like the paper's tables, the
 * DP here is over EXACT latency sums: g[s][t] is the least total cores of
 * models s..S-1 whose latencies add up to exactly t grid ticks (the paper's
 * dp[][] reachability flag is "g < INF", its best[][][0] is g).  The answer
 * scan walks the budgets upward and only accepts a strictly smaller total,
 * which yields least cost first and least latency second, as in the scan
 * that follows Algorithm 1's main loop.
 *
 * Readings where the paper is silent or garbled:
 *   - integer stand-in for the fitted profile of Eq. 1:
 *       proc(c,b) = ceil((a + k*b + q*b*b) / min(c,p)) + o   microseconds
 *     (epsilon->a, gamma->k, eta->o, plus the quadratic batch term Section 4.1
 *     mentions and a core cap p for the parallelism limit);
 *   - throughput h = b / proc, constraint non-strict as in Eq. 6, so the
 *     derived instance count is n = ceil(lambda*proc / (b*1e6)), never
 *     the floor printed in Algorithm 2 (a floor would break the constraint);
 *   - the candidate filter in both listings is read as "skip when the
 *     throughput is insufficient or the latency exceeds the budget", which is
 *     what the prose after Algorithm 1 says;
 *   - queueing delay: the batch-fill wait of Eq. 4, (b-1)/lambda, taken per
 *     replica (each of the n replicas sees lambda/n):
 *       queue = ceil((b-1) * 1e6 * n / lambda)   microseconds;
 *   - every rounding is upward; a stage's latency is put on the grid by
 *     lt = ceil((proc+queue)/tick) and the budget is T = floor(SLO/tick);
 *   - ties: least cost, then least total ticks, then the lexicographically
 *     smallest ((c,b,n) of model 0, (c,b,n) of model 1, ...).  Running the
 *     recurrence over suffixes and rebuilding forward from model 0, taking
 *     the first (c ascending, then b ascending) candidate that attains the
 *     optimum at each step, realises that order.
 *
 * Parity pins (tests/test_oracle_pins.py): exhaustive enumeration of Eq. 6
 * in oracle/themis_bruteforce.c on tiny pipelines, a hand-worked example,
 * the separable closed form under a loose SLO, monotonicity and refinement
 * invariants, and a forward recurrence over sparse sets of prefix sums.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_INF ((int64_t)1 << 60)

/*
 * Model options, process-wide (set them before calling, never while another
 * thread is inside this file).
 *   queue model   0  batch-fill wait per replica, ceil((b-1)*1e6*n/lambda)
 *                    (the default reading described above)
 *                 1  Eq. 4 as printed: one queue per model,
 *                    ceil((b-1)*1e6/lambda), independent of n
 *                 2  Eq. 3: max( (b-1)/lambda , l(b,c) - (n*b+1)/lambda ),
 *                    first term as in 1, second rounded up as
 *                    proc - floor((n*b+1)*1e6/lambda)
 *   profile form  0  five coefficients (a,k,q,p,o)
 *                 1  six (a,k,q,p,o,d): Eq. 1's term delta*b, which does not
 *                    shrink with the cores, is added: proc += d*b
 */
static int g_queue_model = 0;
static int g_profile_form = 0;

int themis_oracle_set_model(int32_t queue_model, int32_t profile_form)
{
    if (queue_model < 0 || queue_model > 2 || profile_form < 0 || profile_form > 1) return -1;
    g_queue_model = queue_model;
    g_profile_form = profile_form;
    return 0;
}

static int coef_stride(void) { return g_profile_form ? 6 : 5; }

static int64_t ceildiv64(int64_t x, int64_t d) { return (x + d - 1) / d; }

/* One candidate (c, b) of one model: Section 4.4, the "calculate l, q, h" step. */
typedef struct {
    int feasible;
    int64_t r;      /* instances n_s                        */
    int64_t lt;     /* latency in grid ticks                */
    int64_t cost;   /* n_s * c_s                            */
    int64_t lat_us; /* proc + queue, microseconds           */
} orc_cand;

static orc_cand eval_candidate(const int32_t *cf, int64_t lambda, int64_t T,
                               int64_t tick, int64_t c, int64_t b,
                               int64_t r_max, int64_t r_given /* <=0: derive */)
{
    orc_cand out;
    int64_t a = cf[0], k = cf[1], q = cf[2], p = cf[3], o = cf[4];
    int64_t d = g_profile_form ? cf[5] : 0;
    int64_t div = c < p ? c : p;
    int64_t proc = ceildiv64(a + k * b + q * b * b, div) + d * b + o;
    int64_t r;
    memset(&out, 0, sizeof out);
    if (r_given <= 0) {
        /* least n with lambda <= n * b / proc  (per second = 1e6 us) */
        r = ceildiv64(lambda * proc, b * 1000000);
        if (r < 1) r = 1;
        if (r > r_max) return out;
    } else {
        r = r_given;
        if (lambda * proc > r * b * 1000000) return out;
    }
    {
        int64_t queue, lat;
        if (g_queue_model == 0) {
            queue = ceildiv64((b - 1) * 1000000 * r, lambda);
        } else {
            queue = ceildiv64((b - 1) * 1000000, lambda);
            if (g_queue_model == 2) {
                /* all n instances busy: wait for one to finish */
                int64_t busy = proc - ((r * b + 1) * 1000000) / lambda;
                if (busy > queue) queue = busy;
            }
        }
        lat = proc + queue;
        int64_t lt = ceildiv64(lat, tick);
        if (lt > T) return out;
        out.feasible = 1;
        out.r = r;
        out.lt = lt;
        out.cost = r * c;
        out.lat_us = lat;
    }
    return out;
}

/*
 * Input ranges an instance must respect (an interface rule, not the paper's):
 * 1 <= lambda <= 2^20, 0 <= SLO <= slo_max, 0 <= a,k,q,d <= 2^20,
 * 1 <= o <= 2^20, p >= 1, and 1 <= given instances <= r_max.  They keep every
 * product below 2^63 for batch sizes up to 1024 and make every stage latency
 * at least one microsecond.
 */
#define ORC_VAL_MAX (1 << 20)

static int instance_valid(int64_t lambda, int64_t slo, int64_t slo_max,
                          const int32_t *cf, int S,
                          const int32_t *rfix, int64_t r_max)
{
    int s, j, cs = coef_stride();
    if (lambda < 1 || lambda > ORC_VAL_MAX || slo < 0 || slo > slo_max) return 0;
    for (s = 0; s < S; ++s) {
        for (j = 0; j < 3; ++j)
            if (cf[cs * s + j] < 0 || cf[cs * s + j] > ORC_VAL_MAX) return 0;
        if (cf[cs * s + 3] < 1) return 0;
        if (cf[cs * s + 4] < 1 || cf[cs * s + 4] > ORC_VAL_MAX) return 0;
        if (cs == 6 && (cf[cs * s + 5] < 0 || cf[cs * s + 5] > ORC_VAL_MAX)) return 0;
        if (rfix && (rfix[s] < 1 || rfix[s] > r_max)) return 0;
    }
    return 1;
}

/*
 * Candidate tables of instances [i0, i1): lt/cost/r are [i1-i0][S][K] with
 * K = c_max*n_batch and index (c-1)*n_batch + j; infeasible entries hold -1.
 * r_fixed == NULL selects the joint evaluation.
 */
int themis_oracle_candidates(int32_t n_stage, int32_t c_max, int32_t n_batch,
                             const int32_t *batch_sizes, int32_t r_max,
                             int32_t tick_us, int32_t slo_max_us, int32_t coef_shared,
                             const int32_t *coef, const int32_t *lambda,
                             const int32_t *slo_us, const int32_t *r_fixed,
                             int32_t i0, int32_t i1,
                             int32_t *lt_out, int32_t *cost_out, int32_t *r_out)
{
    int S = n_stage, K = c_max * n_batch;
    int i, s, c, j;
    for (i = i0; i < i1; ++i) {
        const int32_t *cf = coef_shared ? coef : coef + (size_t)i * S * coef_stride();
        const int32_t *rf = r_fixed ? r_fixed + (size_t)i * S : NULL;
        int ok = instance_valid(lambda[i], slo_us[i], slo_max_us, cf, S, rf, r_max);
        int64_t T = ok ? slo_us[i] / tick_us : 0;
        for (s = 0; s < S; ++s)
            for (c = 1; c <= c_max; ++c)
                for (j = 0; j < n_batch; ++j) {
                    size_t at = ((size_t)(i - i0) * S + s) * K + (size_t)(c - 1) * n_batch + j;
                    orc_cand cd;
                    memset(&cd, 0, sizeof cd);
                    if (ok)
                        cd = eval_candidate(cf + coef_stride() * s, lambda[i], T, tick_us, c,
                                            batch_sizes[j], r_max, rf ? rf[s] : 0);
                    lt_out[at] = cd.feasible ? (int32_t)cd.lt : -1;
                    cost_out[at] = cd.feasible ? (int32_t)cd.cost : -1;
                    r_out[at] = cd.feasible ? (int32_t)cd.r : -1;
                }
    }
    return 0;
}

/* Scratch that solve_one() grows as needed and the caller frees. */
typedef struct {
    orc_cand *cand;
    size_t cand_cap;
    int64_t *g;
    size_t g_cap;
} orc_scratch;

static void scratch_free(orc_scratch *w)
{
    free(w->cand);
    free(w->g);
    w->cand = NULL;
    w->g = NULL;
    w->cand_cap = w->g_cap = 0;
}

/*
 * One instance at arrival rate `lambda`.  rf != NULL: replicas given per model
 * (vertical).  cfix != NULL: cores given per model, each in 1..c_max or the
 * instance is invalid (only candidates with c == cfix[s] are considered; used for the horizontal remainder of
 * Algorithm 1's fallback).  Writes status (0 solved, 1 none, 2 invalid),
 * cost, ticks, cfg[S][3].  Returns <0 on an internal error.
 */
static int solve_one(int S, int c_max, int n_batch, const int32_t *batch_sizes, int r_max,
                     int tick_us, int slo_max_us, const int32_t *cf, int64_t lambda,
                     int64_t slo, const int32_t *rf, const int32_t *cfix, orc_scratch *w,
                     int32_t *status, int32_t *cost, int32_t *ticks, int32_t *o_cfg)
{
    int K = c_max * n_batch;
    int s, k;
    int64_t T, t, best_cost, best_t;
    size_t row;
    orc_cand *cand;
    int64_t *g;

    *status = 1;
    *cost = -1;
    *ticks = -1;
    memset(o_cfg, 0, sizeof(int32_t) * S * 3);
    if (!instance_valid(lambda, slo, slo_max_us, cf, S, rf, r_max)) {
        *status = 2;
        return 0;
    }
    if (cfix)                          /* given cores must be allocatable */
        for (s = 0; s < S; ++s)
            if (cfix[s] < 1 || cfix[s] > c_max) {
                *status = 2;
                return 0;
            }
    T = slo / tick_us;
    row = (size_t)T + 1;
    if ((size_t)S * K > w->cand_cap) {
        free(w->cand);
        w->cand_cap = (size_t)S * K;
        w->cand = (orc_cand *)malloc(sizeof(orc_cand) * w->cand_cap);
        if (!w->cand) return -1;
    }
    if ((size_t)(S + 1) * row > w->g_cap) {
        free(w->g);
        w->g_cap = (size_t)(S + 1) * row;
        w->g = (int64_t *)malloc(sizeof(int64_t) * w->g_cap);
        if (!w->g) return -1;
    }
    cand = w->cand;
    g = w->g;

    /* the candidates of every model, in (c ascending, b ascending) order */
    for (s = 0; s < S; ++s)
        for (k = 0; k < K; ++k) {
            int c = k / n_batch + 1;
            orc_cand cd = eval_candidate(cf + coef_stride() * s, lambda, T, tick_us, c,
                                         batch_sizes[k % n_batch], r_max, rf ? rf[s] : 0);
            if (cfix && c != cfix[s]) cd.feasible = 0;
            cand[(size_t)s * K + k] = cd;
        }

    /* no models left: only the empty split (zero latency) is reachable */
    for (t = 0; t <= T; ++t) g[(size_t)S * row + t] = ORC_INF;
    g[(size_t)S * row + 0] = 0;

    /* add models one at a time; split budget t between model s and the rest */
    for (s = S - 1; s >= 0; --s)
        for (t = 0; t <= T; ++t) {
            int64_t m = ORC_INF;
            for (k = 0; k < K; ++k) {
                const orc_cand *cd = &cand[(size_t)s * K + k];
                int64_t rest;
                if (!cd->feasible || cd->lt > t) continue;
                rest = g[(size_t)(s + 1) * row + (t - cd->lt)];
                if (rest >= ORC_INF) continue;
                if (cd->cost + rest < m) m = cd->cost + rest;
            }
            g[(size_t)s * row + t] = m;
        }

    /* answer scan: budgets upward, strictly smaller total replaces */
    best_cost = ORC_INF;
    best_t = -1;
    for (t = 0; t <= T; ++t)
        if (g[t] < best_cost) { best_cost = g[t]; best_t = t; }
    if (best_t < 0) return 0;

    /* rebuild forward; first candidate in (c,b) order that attains g */
    t = best_t;
    for (s = 0; s < S; ++s) {
        int found = 0;
        for (k = 0; k < K && !found; ++k) {
            const orc_cand *cd = &cand[(size_t)s * K + k];
            int64_t rest;
            if (!cd->feasible || cd->lt > t) continue;
            rest = g[(size_t)(s + 1) * row + (t - cd->lt)];
            if (rest >= ORC_INF) continue;
            if (cd->cost + rest == g[(size_t)s * row + t]) {
                o_cfg[3 * s + 0] = k / n_batch + 1;
                o_cfg[3 * s + 1] = batch_sizes[k % n_batch];
                o_cfg[3 * s + 2] = (int32_t)cd->r;
                t -= cd->lt;
                found = 1;
            }
        }
        if (!found) return -2;
    }
    if (t != 0) return -3;
    *status = 0;
    *cost = (int32_t)best_cost;
    *ticks = (int32_t)best_t;
    return 0;
}

/*
 * Solve instances [i0, i1).  Outputs are indexed from i0:
 *   status 0 solved, 1 no configuration meets the SLO, 2 invalid input;
 *   cost = total cores, ticks = total latency on the grid (both -1 unless
 *   solved); cfg[.][s] = (c, b, n) per model (zeros unless solved).
 * c_fixed (may be NULL): int32 [N][S], cores pinned per model.
 */
int themis_oracle_solve_ex(int32_t n_stage, int32_t c_max, int32_t n_batch,
                           const int32_t *batch_sizes, int32_t r_max,
                           int32_t tick_us, int32_t slo_max_us, int32_t coef_shared,
                           const int32_t *coef, const int32_t *lambda,
                           const int32_t *slo_us, const int32_t *r_fixed,
                           const int32_t *c_fixed, int32_t i0, int32_t i1,
                           int32_t *status, int32_t *cost, int32_t *ticks, int32_t *cfg)
{
    int S = n_stage, i, rc = 0;
    orc_scratch w = {0};
    for (i = i0; i < i1 && rc == 0; ++i) {
        const int32_t *cf = coef_shared ? coef : coef + (size_t)i * S * coef_stride();
        rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                       lambda[i], slo_us[i], r_fixed ? r_fixed + (size_t)i * S : NULL,
                       c_fixed ? c_fixed + (size_t)i * S : NULL, &w, status + (i - i0),
                       cost + (i - i0), ticks + (i - i0), cfg + (size_t)(i - i0) * S * 3);
    }
    scratch_free(&w);
    return rc;
}

int themis_oracle_solve(int32_t n_stage, int32_t c_max, int32_t n_batch,
                        const int32_t *batch_sizes, int32_t r_max,
                        int32_t tick_us, int32_t slo_max_us, int32_t coef_shared,
                        const int32_t *coef, const int32_t *lambda,
                        const int32_t *slo_us, const int32_t *r_fixed,
                        int32_t i0, int32_t i1,
                        int32_t *status, int32_t *cost, int32_t *ticks, int32_t *cfg)
{
    return themis_oracle_solve_ex(n_stage, c_max, n_batch, batch_sizes, r_max, tick_us,
                                  slo_max_us, coef_shared, coef, lambda, slo_us, r_fixed, NULL,
                                  i0, i1, status, cost, ticks, cfg);
}

/*
 * Algorithm 1 with its fallback (Section 4.4): solve the vertical problem at
 * lambda; if there is no solution, binary-search the largest arrival rate the
 * given replicas can absorb, keep the vertical configuration at that rate, and
 * serve the remaining lambda - lambda_v by NEW instances found with the
 * horizontal dynamic program (Algorithm 2: choose instance count and batch),
 * each model keeping the core allocation of the vertical configuration.
 *
 * Readings where the listing is garbled: the midpoint is (left+right)/2, and a
 * FEASIBLE midpoint raises `left` (the printed midpoint formula and branches
 * would not search).  left starts at 1 and right at lambda, the loop runs while
 * right - left > 1, and the configuration returned is the one at `left`; if
 * even that is infeasible the instance has no solution (lambda_v = 0).
 * Feasibility is not monotone in lambda (a higher rate fills batches faster),
 * so the search is a heuristic; this checker follows its steps literally.
 *
 * Outputs per instance, indexed from i0:
 *   status/cost/ticks/cfg   the vertical part (at lambda_v); status 1 if none
 *   lambda_v                rate absorbed by the given replicas (lambda if the
 *                           vertical solve succeeded outright, 0 if none)
 *   status_h/cost_h/ticks_h/cfg_h  the new instances for lambda - lambda_v:
 *                           status_h 0 with cost 0, ticks 0 and zero cfg when
 *                           nothing remains; 1 when the remainder cannot be
 *                           served within the SLO and r_max; 2 when there is
 *                           no vertical part to pin the cores to.
 */
int themis_oracle_vertical_fallback(int32_t n_stage, int32_t c_max, int32_t n_batch,
                                    const int32_t *batch_sizes, int32_t r_max,
                                    int32_t tick_us, int32_t slo_max_us, int32_t coef_shared,
                                    const int32_t *coef, const int32_t *lambda,
                                    const int32_t *slo_us, const int32_t *r_fixed,
                                    int32_t i0, int32_t i1,
                                    int32_t *status, int32_t *cost, int32_t *ticks, int32_t *cfg,
                                    int32_t *lambda_v,
                                    int32_t *status_h, int32_t *cost_h, int32_t *ticks_h,
                                    int32_t *cfg_h)
{
    int S = n_stage, i, s, rc = 0;
    orc_scratch w = {0};
    int32_t *cfix = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
    if (!cfix) return -1;
    for (i = i0; i < i1 && rc == 0; ++i) {
        const int32_t *cf = coef_shared ? coef : coef + (size_t)i * S * coef_stride();
        const int32_t *rf = r_fixed + (size_t)i * S;
        int32_t *st = status + (i - i0), *co = cost + (i - i0), *tk = ticks + (i - i0);
        int32_t *cg = cfg + (size_t)(i - i0) * S * 3;
        int32_t *sth = status_h + (i - i0), *coh = cost_h + (i - i0), *tkh = ticks_h + (i - i0);
        int32_t *cgh = cfg_h + (size_t)(i - i0) * S * 3;
        int64_t left, right;

        lambda_v[i - i0] = 0;
        *sth = 2;
        *coh = -1;
        *tkh = -1;
        memset(cgh, 0, sizeof(int32_t) * S * 3);

        rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                       lambda[i], slo_us[i], rf, NULL, &w, st, co, tk, cg);
        if (rc) break;
        if (*st == 2) continue;                 /* invalid input */
        if (*st == 0) {                         /* vertical scaling alone suffices */
            lambda_v[i - i0] = lambda[i];
            *sth = 0;
            *coh = 0;
            *tkh = 0;
            continue;
        }
        /* binary search on the workload */
        left = 1;
        right = lambda[i];
        while (right - left > 1 && rc == 0) {
            int64_t mid = (left + right) / 2;
            rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                           mid, slo_us[i], rf, NULL, &w, st, co, tk, cg);
            if (*st == 0) left = mid; else right = mid;
        }
        if (rc) break;
        rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                       left, slo_us[i], rf, NULL, &w, st, co, tk, cg);
        if (rc) break;
        if (*st != 0) continue;                 /* not even one request per second */
        lambda_v[i - i0] = (int32_t)left;
        if (left == lambda[i]) {                /* only when lambda == 1 */
            *sth = 0;
            *coh = 0;
            *tkh = 0;
            continue;
        }
        /* new instances for the rest, cores as in the vertical configuration */
        for (s = 0; s < S; ++s) cfix[s] = cg[3 * s + 0];
        rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                       lambda[i] - left, slo_us[i], NULL, cfix, &w, sth, coh, tkh, cgh);
    }
    free(cfix);
    scratch_free(&w);
    return rc;
}

/*
 * The workload-stability test of Section 5.1.3 ("When"): run the horizontal
 * dynamic program (Algorithm 2) at the current rate and at the predicted
 * rate and call the workload stable when both yield the same configuration
 * (same instance count and batch size for every model).  cores (may be NULL =
 * the one-core instances of Algorithm 2): int32 [N][S].
 *
 * Outputs indexed from i0: stable = 1 only when both solves succeed and agree;
 * status/cost/ticks/cfg are those of the current rate.
 */
int themis_oracle_stability(int32_t n_stage, int32_t c_max, int32_t n_batch,
                            const int32_t *batch_sizes, int32_t r_max,
                            int32_t tick_us, int32_t slo_max_us, int32_t coef_shared,
                            const int32_t *coef, const int32_t *lambda_now,
                            const int32_t *lambda_pred, const int32_t *slo_us,
                            const int32_t *cores, int32_t i0, int32_t i1,
                            int32_t *stable, int32_t *status, int32_t *cost, int32_t *ticks,
                            int32_t *cfg)
{
    int S = n_stage, i, s, rc = 0;
    orc_scratch w = {0};
    int32_t *one = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
    int32_t *cfg_p = (int32_t *)malloc(sizeof(int32_t) * (size_t)S * 3);
    if (!one || !cfg_p) { free(one); free(cfg_p); return -1; }
    for (s = 0; s < S; ++s) one[s] = 1;
    for (i = i0; i < i1 && rc == 0; ++i) {
        const int32_t *cf = coef_shared ? coef : coef + (size_t)i * S * coef_stride();
        const int32_t *cx = cores ? cores + (size_t)i * S : one;
        int32_t *cg = cfg + (size_t)(i - i0) * S * 3;
        int32_t st_p, cost_p, ticks_p;
        stable[i - i0] = 0;
        rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                       lambda_now[i], slo_us[i], NULL, cx, &w, status + (i - i0),
                       cost + (i - i0), ticks + (i - i0), cg);
        if (rc) break;
        rc = solve_one(S, c_max, n_batch, batch_sizes, r_max, tick_us, slo_max_us, cf,
                       lambda_pred[i], slo_us[i], NULL, cx, &w, &st_p, &cost_p, &ticks_p, cfg_p);
        if (rc) break;
        if (status[i - i0] == 0 && st_p == 0 &&
            memcmp(cg, cfg_p, sizeof(int32_t) * S * 3) == 0)
            stable[i - i0] = 1;
    }
    free(one);
    free(cfg_p);
    scratch_free(&w);
    return rc;
}

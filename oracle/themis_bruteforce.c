/*
 * Exhaustive enumeration of the autoscaling integer program -- TEST
 * INFRASTRUCTURE ONLY.  Nothing in the product path may call this file.
 *
 * This is the problem of Section 4.3 (Eq. 6) written out as its definition:
 * walk over EVERY assignment ((c_s, b_s, n_s)) of cores, batch size and
 * instance count to the models of one pipeline, keep the assignments that
 * satisfy the two constraints, and return the smallest under the order
 *
 *     ( sum_s n_s*c_s ,  sum_s lt_s ,  (c_0,b_0,n_0), (c_1,b_1,n_1), ... )
 *
 * compared left to right.  There is no dynamic program, no derived instance
 * count and no candidate table here: n_s is enumerated over 1..r_max (or
 * pinned to the given count in the vertical case) and both constraints are
 * tested on the assignment as a whole,
 *
 *     lambda * proc_s <= n_s * b_s * 1e6      for every s      (throughput)
 *     sum_s lt_s <= floor(SLO / tick)                          (Eq. 5 on the grid)
 *
 * with proc_s = ceil((a + k b + q b^2)/min(c,p)) + o,
 * queue_s = ceil((b-1) * 1e6 * n / lambda), lt_s = ceil((proc_s+queue_s)/tick).
 * themis_bruteforce_set_model() switches to the paper's printed forms: the
 * queue of Eq. 4, ceil((b-1)*1e6/lambda), or of Eq. 3, the larger of that and
 * proc - floor((n b + 1)*1e6/lambda); and Eq. 1's term d*b added to proc.
 * Exponential in the number of models: only for tiny pipelines.
 *
 * It deliberately duplicates the few lines of latency arithmetic instead of
 * sharing them with themis_oracle.c, so that a slip in either shows up as a
 * disagreement.  The arithmetic itself is pinned by the hand-worked example
 * in tests/golden/.
 */
#include <stdint.h>
#include <string.h>

#define BF_MAX_STAGE 6

typedef struct {
    int S, c_max, n_batch, r_max;
    const int32_t *batch_sizes;
    const int32_t *coef;    /* [S][5], or [S][6] with the sixth coefficient d */
    int queue_model, profile_form;
    const int32_t *r_fixed; /* [S] or NULL */
    const int32_t *c_fixed; /* [S] or NULL */
    long long lambda, tick, T;
    int cur[BF_MAX_STAGE][3];
    int best[BF_MAX_STAGE][3];
    long long best_cost, best_ticks;
    int have;
    long long visited;
} bf_state;

static long long up_div(long long x, long long d) { return x / d + (x % d != 0); }

static int key_less(const bf_state *st, long long cost, long long ticks)
{
    int s, j;
    if (!st->have) return 1;
    if (cost != st->best_cost) return cost < st->best_cost;
    if (ticks != st->best_ticks) return ticks < st->best_ticks;
    for (s = 0; s < st->S; ++s)
        for (j = 0; j < 3; ++j)
            if (st->cur[s][j] != st->best[s][j]) return st->cur[s][j] < st->best[s][j];
    return 0;
}

static void walk(bf_state *st, int s, long long cost, long long ticks)
{
    int c, j, n, n_lo, n_hi, c_lo, c_hi;
    if (s == st->S) {
        st->visited++;
        if (ticks <= st->T && key_less(st, cost, ticks)) {
            memcpy(st->best, st->cur, sizeof st->cur);
            st->best_cost = cost;
            st->best_ticks = ticks;
            st->have = 1;
        }
        return;
    }
    n_lo = st->r_fixed ? st->r_fixed[s] : 1;
    n_hi = st->r_fixed ? st->r_fixed[s] : st->r_max;
    c_lo = st->c_fixed ? st->c_fixed[s] : 1;
    c_hi = st->c_fixed ? st->c_fixed[s] : st->c_max;
    for (c = c_lo; c <= c_hi; ++c)
        for (j = 0; j < st->n_batch; ++j)
            for (n = n_lo; n <= n_hi; ++n) {
                const int32_t *cf = st->coef + (st->profile_form ? 6 : 5) * s;
                long long b = st->batch_sizes[j];
                long long cores = c < cf[3] ? c : cf[3];
                long long proc = up_div((long long)cf[0] + (long long)cf[1] * b +
                                        (long long)cf[2] * b * b, cores) + cf[4];
                long long queue, lt;
                if (st->profile_form) proc += (long long)cf[5] * b;   /* Eq. 1's delta*b */
                if (st->lambda * proc > (long long)n * b * 1000000LL) continue;
                if (st->queue_model == 0) {
                    queue = up_div((b - 1) * 1000000LL * n, st->lambda);
                } else {
                    /* Eq. 4; for model 2 the larger of it and Eq. 3's busy term */
                    long long busy = proc - ((long long)n * b + 1) * 1000000LL / st->lambda;
                    queue = up_div((b - 1) * 1000000LL, st->lambda);
                    if (st->queue_model == 2 && busy > queue) queue = busy;
                }
                lt = up_div(proc + queue, st->tick);
                st->cur[s][0] = c;
                st->cur[s][1] = (int)b;
                st->cur[s][2] = n;
                walk(st, s + 1, cost + (long long)n * c, ticks + lt);
            }
}

/*
 * One instance.  Returns 0 solved, 1 nothing feasible, <0 bad call.
 * coef is [S][5] = (a,k,q,p,o); r_fixed NULL enumerates 1..r_max; c_fixed
 * NULL enumerates 1..c_max, else pins each model's cores.
 * Outputs: cost, ticks, cfg[S][3] = (c,b,n); *n_visited = leaves walked.
 */
static int bf_queue_model = 0, bf_profile_form = 0;

/* Model options as in themis_oracle.c's header; process-wide. */
int themis_bruteforce_set_model(int32_t queue_model, int32_t profile_form)
{
    if (queue_model < 0 || queue_model > 2 || profile_form < 0 || profile_form > 1) return -1;
    bf_queue_model = queue_model;
    bf_profile_form = profile_form;
    return 0;
}

int themis_bruteforce_ex(int32_t n_stage, int32_t c_max, int32_t n_batch,
                         const int32_t *batch_sizes, int32_t r_max, int32_t tick_us,
                         const int32_t *coef, int32_t lambda, int32_t slo_us,
                         const int32_t *r_fixed, const int32_t *c_fixed,
                         int32_t *cost, int32_t *ticks, int32_t *cfg, int64_t *n_visited)
{
    bf_state st;
    int s, j;
    if (n_stage < 1 || n_stage > BF_MAX_STAGE || lambda < 1 || slo_us < 0 || tick_us < 1)
        return -1;
    memset(&st, 0, sizeof st);
    st.S = n_stage;
    st.c_max = c_max;
    st.n_batch = n_batch;
    st.r_max = r_max;
    st.batch_sizes = batch_sizes;
    st.coef = coef;
    st.r_fixed = r_fixed;
    st.c_fixed = c_fixed;
    st.queue_model = bf_queue_model;
    st.profile_form = bf_profile_form;
    st.lambda = lambda;
    st.tick = tick_us;
    st.T = slo_us / tick_us;
    walk(&st, 0, 0, 0);
    if (n_visited) *n_visited = st.visited;
    *cost = -1;
    *ticks = -1;
    for (s = 0; s < n_stage; ++s)
        for (j = 0; j < 3; ++j) cfg[3 * s + j] = 0;
    if (!st.have) return 1;
    *cost = (int32_t)st.best_cost;
    *ticks = (int32_t)st.best_ticks;
    for (s = 0; s < n_stage; ++s)
        for (j = 0; j < 3; ++j) cfg[3 * s + j] = st.best[s][j];
    return 0;
}

int themis_bruteforce(int32_t n_stage, int32_t c_max, int32_t n_batch,
                      const int32_t *batch_sizes, int32_t r_max, int32_t tick_us,
                      const int32_t *coef, int32_t lambda, int32_t slo_us,
                      const int32_t *r_fixed,
                      int32_t *cost, int32_t *ticks, int32_t *cfg, int64_t *n_visited)
{
    return themis_bruteforce_ex(n_stage, c_max, n_batch, batch_sizes, r_max, tick_us, coef,
                                lambda, slo_us, r_fixed, (const int32_t *)0, cost, ticks, cfg,
                                n_visited);
}

/*
 * themis.h -- C ABI of the batched autoscaling solve for AMD MI355X (gfx950).
 *
 * One "instance" is one inference pipeline (a chain of n_stage models) at one
 * request arrival rate lambda under one end-to-end latency objective.  For
 * every instance the library solves the integer program of Section 4.3
 * (Eq. 6): choose, per model s, cores per replica c_s, batch size b_s and
 * replica count n_s so that the total cores sum_s n_s*c_s are least while
 *
 *     sum_s [ l_s(b_s,c_s) + q_s(b_s) ] <= SLO                 (Eq. 5)
 *     lambda <= h_s(b_s,c_s) * n_s      for every model s
 *
 * using the stage-by-stage dynamic program over a latency-budget grid that
 * Section 4.4 describes (Algorithm 1 with the replicas given = "vertical";
 * Algorithm 1's (c,b) search with Algorithm 2's derived replica count folded
 * into every candidate = "joint").  Thousands of independent instances are
 * solved per call, one after the other in HBM, all on one GPU.
 *
 * Integer model (all times in microseconds, every rounding upward).  For
 * model s with profile coefficients (a,k,q,p,o), cores c and batch b:
 *     proc  = ceil((a + k*b + q*b*b) / min(c,p)) + o        after Eq. 1
 *     n     = ceil(lambda*proc / (b*1e6))  (joint; infeasible if n > r_max)
 *             given r_fixed[s]             (vertical; infeasible unless
 *                                           lambda*proc <= n*b*1e6)
 *     queue = ceil((b-1)*1e6*n / lambda)                    after Eq. 4
 *     lt    = ceil((proc+queue) / tick_us)   grid ticks
 *     cost  = n*c
 * and the budget of an instance is T = floor(slo_us / tick_us) ticks.
 * The queue above is Eq. 4's batch-fill wait seen by one replica (each of the
 * n replicas receives lambda/n).  themis_problem_t.queue_model selects the
 * paper's printed forms instead:
 *     THEMIS_QUEUE_SHARED      queue = ceil((b-1)*1e6 / lambda)          Eq. 4
 *     THEMIS_QUEUE_WORST_CASE  queue = max of that and
 *                              proc - floor((n*b+1)*1e6 / lambda)        Eq. 3
 * and profile_form = THEMIS_PROFILE_EQ1 adds Eq. 1's term delta*b, which does
 * not shrink with the cores: six coefficients (a,k,q,p,o,d) per model and
 *     proc  = ceil((a + k*b + q*b*b) / min(c,p)) + d*b + o.
 * A candidate is the pair (c,b); its index is k = (c-1)*n_batch + j for
 * b = batch_sizes[j], so index order is (c ascending, b ascending).
 *
 * Result per instance: the feasible assignment with the smallest
 *     ( total cost, total ticks, (c,b,n) of model 0, (c,b,n) of model 1, ... )
 * compared left to right.  Exactly one assignment is smallest, so results
 * are reproducible bit for bit.
 *
 * Conventions common to all entry points
 *   - Pointers named d_* are DEVICE pointers owned by the caller; p is a HOST
 *     pointer.  The library allocates nothing, frees nothing and keeps no
 *     state between calls (themis_solve_joint_static remembers, per GPU, the
 *     address of its built-in workspace; nothing else is kept).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; the call returns without synchronising.
 *   - Return value: THEMIS_OK, or a negative THEMIS_ERR_* found on the host
 *     before anything is launched.  Nothing is printed; no exception crosses
 *     the boundary.
 *   - Per-instance trouble is reported in d_status, never as a return code.
 */
#ifndef THEMIS_H
#define THEMIS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define THEMIS_MAX_BATCH 16      /* entries in batch_sizes[]                    */
#define THEMIS_MAX_BATCH_SIZE 1024
#define THEMIS_MAX_CANDIDATES 8192 /* c_max*n_batch, rounded up to 8, must not exceed */
#define THEMIS_VALUE_MAX (1 << 20) /* upper bound on lambda and on a,k,q,o      */
#define THEMIS_COST_LIMIT 32767  /* n_stage*r_max*c_max must not exceed this    */
#define THEMIS_MAX_TICKS 32767   /* floor(slo_max_us/tick_us) must not exceed   */

/* return codes */
#define THEMIS_OK 0
#define THEMIS_ERR_NULL (-1)      /* a required pointer is NULL                 */
#define THEMIS_ERR_SHAPE (-2)     /* a count or size is out of range            */
#define THEMIS_ERR_BATCH (-3)     /* batch list not strictly increasing in 1..1024 */
#define THEMIS_ERR_RANGE (-4)     /* cost or tick range exceeds the limits above */
#define THEMIS_ERR_WORKSPACE (-5) /* workspace missing, misaligned or too small */
#define THEMIS_ERR_LAUNCH (-6)    /* the HIP runtime refused a launch           */
#define THEMIS_ERR_TOO_LARGE (-7) /* problem needs more than the built-in scratch */

/* bytes of the built-in workspace of themis_solve_joint_static, per GPU */
#define THEMIS_STATIC_SCRATCH_BYTES (64u << 20)

/* themis_problem_t.queue_model */
#define THEMIS_QUEUE_PER_REPLICA 0
#define THEMIS_QUEUE_SHARED 1
#define THEMIS_QUEUE_WORST_CASE 2
/* themis_problem_t.profile_form */
#define THEMIS_PROFILE_5 0   /* coefficients (a,k,q,p,o)                        */
#define THEMIS_PROFILE_EQ1 1 /* coefficients (a,k,q,p,o,d)                      */

/* themis_problem_t.prune: ways of doing less work for the same results; the
   two may be combined (THEMIS_PRUNE_DOMINATED | THEMIS_PRUNE_STEPS) */
#define THEMIS_PRUNE_NONE 0      /* every feasible candidate enters the recurrence,
                                    which combines it with every budget          */
#define THEMIS_PRUNE_DOMINATED 1 /* candidates that another candidate of the same
                                    model beats or ties on both latency and cost
                                    (ties: smaller index wins) are dropped first.
                                    Results are identical: such a candidate is
                                    in no instance's smallest assignment.       */
#define THEMIS_PRUNE_STEPS 2     /* the recurrence keeps every row as the list of
                                    budgets where it drops (rows never increase
                                    with the budget) and combines candidates
                                    with that list instead of with every budget.
                                    Results are identical, rows included.       */

/* per-instance status written to d_status */
#define THEMIS_SOLVED 0
#define THEMIS_INFEASIBLE 1 /* no assignment meets both constraints            */
#define THEMIS_INVALID 2    /* input out of range, see below                   */
#define THEMIS_INTERNAL 3   /* reconstruction failed; never expected           */

/*
 * The search space shared by every instance of a call.
 *
 * An instance is THEMIS_INVALID when lambda is outside 1..THEMIS_VALUE_MAX,
 * slo_us is outside 0..slo_max_us, any of a,k,q is outside
 * 0..THEMIS_VALUE_MAX (d too, where present), o is outside
 * 1..THEMIS_VALUE_MAX (so every stage takes at least one tick), p < 1, or
 * (vertical) a given replica count is outside 1..r_max.
 */
typedef struct themis_problem {
    int32_t n_inst;     /* N >= 1 instances                                    */
    int32_t n_stage;    /* S >= 1 models per pipeline                          */
    int32_t c_max;      /* cores per replica range over 1..c_max               */
    int32_t n_batch;    /* 1..THEMIS_MAX_BATCH                                 */
    int32_t batch_sizes[THEMIS_MAX_BATCH]; /* strictly increasing, 1..1024     */
    int32_t r_max;      /* replicas range over 1..r_max (vertical: bound on r_fixed) */
    int32_t tick_us;    /* grid resolution, >= 1                               */
    int32_t slo_max_us; /* caller's bound on every slo_us entry, >= 0          */
    int32_t coef_shared;/* 1: d_coef is [S][5]; 0: [N][S][5]; order a,k,q,p,o
                           ([S][6] / [N][S][6], order a,k,q,p,o,d, under
                           THEMIS_PROFILE_EQ1)                                  */
    int32_t queue_model;/* THEMIS_QUEUE_*                                      */
    int32_t profile_form;/* THEMIS_PROFILE_*                                   */
    int32_t prune;      /* THEMIS_PRUNE_*                                      */
    int32_t reserved[1];/* must be zero                                        */
} themis_problem_t;

/* Library version, major*100 + minor. */
int themis_version(void);

/*
 * Check a problem description on the host.  Returns THEMIS_OK or the
 * THEMIS_ERR_* the solve calls would return for it.
 */
int themis_check_problem(const themis_problem_t *p);

/*
 * Bytes of device workspace the solve and stage calls need for `p`
 * (0 if `p` is not acceptable).  The workspace holds the candidate tables
 * (Section 4.4, the per-candidate l, q, h evaluation hoisted out of the
 * budget loop), the DP rows of every model, and one word per instance.
 * It must be 256-byte aligned.  Contents need not be initialised.
 */
size_t themis_workspace_bytes(const themis_problem_t *p);

/*
 * Joint horizontal+vertical solve (Eq. 6 with n_s derived per candidate).
 *   d_coef    int32, [S][5] or [N][S][5] per coef_shared (six per model
 *             under THEMIS_PROFILE_EQ1)
 *   d_lambda  int32 [N]   requests per second
 *   d_slo_us  int32 [N]
 *   d_status  int32 [N]   THEMIS_SOLVED / INFEASIBLE / INVALID
 *   d_cost    int32 [N]   total cores, -1 unless solved
 *   d_ticks   int32 [N]   total latency in ticks, -1 unless solved
 *   d_cfg     int32 [N][S][3] = (c, b, n) per model, zeros unless solved
 * Runs the three stages below back to back on `stream`.
 */
int themis_solve_joint(const themis_problem_t *p, const int32_t *d_coef,
                       const int32_t *d_lambda, const int32_t *d_slo_us,
                       int32_t *d_status, int32_t *d_cost, int32_t *d_ticks,
                       int32_t *d_cfg, void *d_workspace, size_t workspace_bytes,
                       void *stream);

/*
 * themis_solve_joint for callers that cannot allocate device memory or hand
 * over a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same inputs, outputs and results as
 * themis_solve_joint; the workspace is an array of
 * THEMIS_STATIC_SCRATCH_BYTES built into the library's device code (every GPU
 * the library runs on holds one from the first launch until the process ends).
 * The call allocates and frees nothing.  A problem whose
 * themis_workspace_bytes(p) exceeds THEMIS_STATIC_SCRATCH_BYTES is refused
 * with THEMIS_ERR_TOO_LARGE and nothing is launched.  The first call on a
 * device looks the array's address up (not an allocation; make that call
 * outside a stream capture).  All calls on one GPU share the one array: the
 * next call overwrites what the last one left there, and two calls that
 * overlap in time on the same GPU (different streams, different threads) race;
 * callers serialise them, e.g. by using one stream.
 */
int themis_solve_joint_static(const themis_problem_t *p, const int32_t *d_coef,
                              const int32_t *d_lambda, const int32_t *d_slo_us,
                              int32_t *d_status, int32_t *d_cost, int32_t *d_ticks,
                              int32_t *d_cfg, void *stream);

/*
 * Vertical-only solve (Algorithm 1): replicas are given, d_r_fixed int32
 * [N][S], every entry in 1..r_max; cores and batch are chosen; cost is
 * r_fixed*c per model.  Other arguments as for themis_solve_joint.
 */
int themis_solve_vertical(const themis_problem_t *p, const int32_t *d_coef,
                          const int32_t *d_lambda, const int32_t *d_slo_us,
                          const int32_t *d_r_fixed,
                          int32_t *d_status, int32_t *d_cost, int32_t *d_ticks,
                          int32_t *d_cfg, void *d_workspace, size_t workspace_bytes,
                          void *stream);

/*
 * Horizontal-only solve (Algorithm 2): the cores of every model are given and
 * the instance count n and the batch size b are chosen, n derived from the
 * throughput constraint as in the joint solve; cost is n*c per model.
 *   d_cores   int32 [N][S], every entry in 1..c_max (anything else makes the
 *             instance THEMIS_INVALID), or NULL for the one-core instances of
 *             Algorithm 2.
 * Other arguments, outputs and workspace as for themis_solve_joint; the cfg
 * rows repeat the given cores.
 */
int themis_solve_horizontal(const themis_problem_t *p, const int32_t *d_coef,
                            const int32_t *d_lambda, const int32_t *d_slo_us,
                            const int32_t *d_cores,
                            int32_t *d_status, int32_t *d_cost, int32_t *d_ticks,
                            int32_t *d_cfg, void *d_workspace, size_t workspace_bytes,
                            void *stream);

/*
 * Bytes of device workspace themis_solve_vertical_fallback needs (0 if `p` is
 * not acceptable): themis_workspace_bytes(p) plus a few words per instance and
 * model for the rates and cores handed from pass to pass.  256-byte aligned, contents need not be initialised.
 */
size_t themis_fallback_workspace_bytes(const themis_problem_t *p);

/*
 * Vertical solve with the fallback of Algorithm 1 (Section 4.4, the step taken
 * when the main loop finds no configuration): where the given replicas cannot
 * serve lambda within the SLO, a binary search on the arrival rate finds a rate
 * lambda_v they can absorb (left = 1, right = lambda, a feasible midpoint
 * (left+right)/2 raises left, until right - left <= 1; lambda_v = left), the
 * vertical configuration is solved at lambda_v, and the remaining
 * lambda - lambda_v is given to NEW instances chosen by the horizontal solve
 * with each model's cores pinned to those of the vertical configuration.
 * Feasibility is not monotone in the rate (a higher rate fills batches
 * sooner), so like the paper's search this is a heuristic for "the largest
 * rate"; its steps are fixed and the result is deterministic.
 *
 * The search itself does not run the dynamic program: the replicas can absorb
 * a rate exactly when the fastest feasible candidate of every model (with the
 * replicas given, the one at the core cap) fits the budget together, which one
 * thread per instance tests with the candidate stage's arithmetic.  The three
 * stages run three times: at lambda for all instances, then at lambda_v and
 * for the remainder over the instances the first pass left open.
 *
 *   d_r_fixed   int32 [N][S]  running replicas, 1..r_max
 * Outputs, all int32 on the device:
 *   d_status/d_cost/d_ticks [N], d_cfg [N][S][3]   the vertical part at
 *               lambda_v; THEMIS_INFEASIBLE when not even rate 1 fits
 *   d_lambda_v [N]  rate the running replicas keep (lambda if the plain solve
 *               succeeds, 0 when there is no vertical part or the instance is
 *               invalid)
 *   d_status_h/d_cost_h/d_ticks_h [N], d_cfg_h [N][S][3]   the new instances:
 *               THEMIS_SOLVED with cost 0, ticks 0 and zero rows when nothing
 *               remains; THEMIS_INFEASIBLE when the remainder cannot be served
 *               within the SLO and r_max; THEMIS_INVALID when there is no
 *               vertical part to take the cores from.
 * d_workspace holds themis_fallback_workspace_bytes(p) bytes.  All passes run
 * on `stream`; nothing is allocated and the host does not wait.
 */
int themis_solve_vertical_fallback(const themis_problem_t *p, const int32_t *d_coef,
                                   const int32_t *d_lambda, const int32_t *d_slo_us,
                                   const int32_t *d_r_fixed,
                                   int32_t *d_status, int32_t *d_cost, int32_t *d_ticks,
                                   int32_t *d_cfg, int32_t *d_lambda_v,
                                   int32_t *d_status_h, int32_t *d_cost_h,
                                   int32_t *d_ticks_h, int32_t *d_cfg_h,
                                   void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Bytes of device workspace themis_check_stability needs (0 if `p` is not
 * acceptable): themis_workspace_bytes(p) plus one set of results.
 */
size_t themis_stability_workspace_bytes(const themis_problem_t *p);

/*
 * Workload-stability test (Section 5.1.3, "When"): the horizontal solve of
 * Algorithm 2 at the current rate and at the predicted rate; the workload is
 * stable when both succeed with the same (c, b, n) for every model, which is
 * the paper's cue to move from vertical to horizontal scaling.  The predicted
 * rate is an input (the paper's predictor is not part of this library).
 *   d_lambda_now, d_lambda_pred  int32 [N]
 *   d_cores    as for themis_solve_horizontal (NULL = one core)
 *   d_stable   int32 [N]  1 stable, 0 not (also when either solve fails or the
 *              instance is invalid)
 *   d_status/d_cost/d_ticks/d_cfg  the solve at the current rate, as for
 *              themis_solve_joint
 * d_workspace holds themis_stability_workspace_bytes(p) bytes.
 */
int themis_check_stability(const themis_problem_t *p, const int32_t *d_coef,
                           const int32_t *d_lambda_now, const int32_t *d_lambda_pred,
                           const int32_t *d_slo_us, const int32_t *d_cores,
                           int32_t *d_stable, int32_t *d_status, int32_t *d_cost,
                           int32_t *d_ticks, int32_t *d_cfg, void *d_workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Bytes of device workspace themis_solve_distinct needs (0 if `p` is not
 * acceptable): themis_workspace_bytes(p) plus two words per instance and a
 * hash table of at least two slots per instance.
 */
size_t themis_memo_workspace_bytes(const themis_problem_t *p);

/*
 * The joint (d_r_fixed NULL) or vertical solve of a batch in which the same
 * inputs recur, as in a sweep over an arrival-rate trace (Section 6 drives the
 * system with the per-second rates of one): instances are grouped by their
 * input words (lambda, slo_us, the replica counts if given, the coefficients
 * unless shared), one instance per group goes through the three stages, and
 * the others receive its results.  Outputs are those of themis_solve_joint /
 * themis_solve_vertical on the same arguments, word for word, invalid
 * instances included; only the work differs.  The measured hot path does not
 * use it: there every instance is solved.
 * d_workspace holds themis_memo_workspace_bytes(p) bytes.
 */
int themis_solve_distinct(const themis_problem_t *p, const int32_t *d_coef,
                          const int32_t *d_lambda, const int32_t *d_slo_us,
                          const int32_t *d_r_fixed, int32_t *d_status, int32_t *d_cost,
                          int32_t *d_ticks, int32_t *d_cfg, void *d_workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Stage 1 alone: evaluate every candidate of every model of every instance
 * (the "calculate l, q, h" step of Algorithms 1 and 2, done once instead of
 * once per budget cell) into the workspace.  d_r_fixed NULL = joint.
 */
int themis_stage_candidates(const themis_problem_t *p, const int32_t *d_coef,
                            const int32_t *d_lambda, const int32_t *d_slo_us,
                            const int32_t *d_r_fixed, void *d_workspace,
                            size_t workspace_bytes, void *stream);

/*
 * Stage 2 alone: the min-plus recurrence over the budget grid,
 *   f[S][t] = 0,  f[s][t] = min over candidates k with lt <= t of
 *                           cost[s][k] + f[s+1][t - lt[s][k]],
 * for the tables stage 1 left in the workspace (Section 4.4: add the models
 * one at a time and split each budget between the current model and the
 * rest).  Leaves the rows f[s][0..T] in the workspace for stage 3, except
 * that of the model handled last (s = 0) where the stage computes the answer
 * (least cost, least budget attaining it) directly from row 1: that pair is
 * left in the workspace instead and stage 3 starts from it.
 * Call it exactly once after each themis_stage_candidates on the same
 * workspace: the stage consumes the per-class work queues that stage 1 sets
 * up, so a second call without a new stage 1 would serve only the first
 * instances of every queue (and must not be used to time the stage).
 */
int themis_stage_minplus(const themis_problem_t *p, void *d_workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Stage 3 alone: answer selection (least cost, then least ticks) and forward
 * reconstruction of the per-model choices from the rows of stage 2
 * (the scan and the recursive read-out that follow Algorithm 1's main loop).
 */
int themis_stage_backtrack(const themis_problem_t *p, int32_t *d_status,
                           int32_t *d_cost, int32_t *d_ticks, int32_t *d_cfg,
                           void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Copy stage 1's tables out of the workspace for inspection:
 * d_lt, d_cost int32 [N][S][K], K = c_max*n_batch; infeasible entries are -1
 * in both (under THEMIS_PRUNE_DOMINATED the dropped candidates too: what is
 * left is the cost/latency staircase of each row).  The replica count of a
 * feasible entry is cost / c.
 */
int themis_export_candidates(const themis_problem_t *p, const void *d_workspace,
                             size_t workspace_bytes, int32_t *d_lt, int32_t *d_cost,
                             void *stream);

/*
 * Number of min-plus relaxations stage 2 executes for the tables currently
 * in the workspace, summed over all instances, written to d_count[0]
 * (d_count: uint64 [3], device): for every valid instance, model and feasible candidate,
 * T + 1 - lt, except for two models that take no relaxations when they
 * have candidates enough to make it pay: the one the recurrence starts with
 * (the last of the pipeline), whose row is then a running minimum over its
 * candidates, and the one it ends with (the first of a pipeline of two or
 * more), of whose row then only the answer is computed.  (Rows of more than
 * 16384 cells and pruned problems excepted: there every model is swept.  With
 * THEMIS_PRUNE_STEPS nothing is swept; the count is then that of sweeping
 * every model, the work the step form replaces.)  d_count[1] takes the number
 * of entries those tables hold: the feasible candidates of the valid instances
 * (less the pruned ones), 8 bytes each.  d_count[2] takes the number of cells
 * (model, budget) whose value stage 2 forms: T + 1 per model of a valid
 * instance, less the rows of which only the answer is computed.  For
 * throughput accounting only.
 */
int themis_count_relaxations(const themis_problem_t *p, const void *d_workspace,
                             size_t workspace_bytes, unsigned long long *d_count,
                             void *stream);

#ifdef __cplusplus
}
#endif
#endif /* THEMIS_H */

// Host side of the C ABI declared in include/themis.h: argument checks and
// launches.  No allocation, no synchronisation; the only state is the per-device
// address of the built-in scratch array of themis_solve_joint_static.
#include "themis_internal.h"

#include <mutex>

using namespace themis;

// Workspace of themis_solve_joint_static: one array per GPU, held from the
// moment the library's code is loaded on that GPU until the process ends.  In
// host code this name is only a handle for hipGetSymbolAddress; kernels get the
// address that call returns.
static __device__ __align__(256) unsigned char scratch[THEMIS_STATIC_SCRATCH_BYTES];

namespace {

int check(const themis_problem_t* p)
{
    if (!p) return THEMIS_ERR_NULL;
    if (p->n_inst < 1 || p->n_stage < 1 || p->c_max < 1 || p->r_max < 1 || p->tick_us < 1 ||
        p->slo_max_us < 0 || (p->coef_shared != 0 && p->coef_shared != 1))
        return THEMIS_ERR_SHAPE;
    if (p->queue_model < THEMIS_QUEUE_PER_REPLICA || p->queue_model > THEMIS_QUEUE_WORST_CASE ||
        p->profile_form < THEMIS_PROFILE_5 || p->profile_form > THEMIS_PROFILE_EQ1 ||
        p->prune < 0 || p->prune > (THEMIS_PRUNE_DOMINATED | THEMIS_PRUNE_STEPS) || p->reserved[0] != 0)
        return THEMIS_ERR_SHAPE;
    if (p->n_batch < 1 || p->n_batch > THEMIS_MAX_BATCH) return THEMIS_ERR_BATCH;
    for (int j = 0; j < p->n_batch; ++j) {
        if (p->batch_sizes[j] < 1 || p->batch_sizes[j] > THEMIS_MAX_BATCH_SIZE)
            return THEMIS_ERR_BATCH;
        if (j > 0 && p->batch_sizes[j] <= p->batch_sizes[j - 1]) return THEMIS_ERR_BATCH;
    }
    // 16-bit DP values: the largest total must stay below the "none" marker
    long long cost_bound = (long long)p->n_stage * p->r_max * p->c_max;
    if (p->c_max > THEMIS_COST_LIMIT || p->r_max > THEMIS_COST_LIMIT ||
        cost_bound > THEMIS_COST_LIMIT)
        return THEMIS_ERR_RANGE;
    if (p->slo_max_us / p->tick_us > THEMIS_MAX_TICKS) return THEMIS_ERR_RANGE;
    // flat candidate index is 32-bit
    long long kp = ((long long)p->c_max * p->n_batch + 7) / 8 * 8;
    if (kp > MAX_CAND) return THEMIS_ERR_SHAPE;
    long long nsk = (long long)p->n_inst * p->n_stage * kp;
    if (nsk >= (1ll << 31)) return THEMIS_ERR_SHAPE;
    return THEMIS_OK;
}

int check_ws(const themis_problem_t* p, const void* ws, size_t bytes, Layout* L)
{
    int rc = check(p);
    if (rc != THEMIS_OK) return rc;
    *L = make_layout(*p);
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || bytes < L->total)
        return THEMIS_ERR_WORKSPACE;
    return THEMIS_OK;
}

// one pass of the three stages
int pass(const themis_problem_t& p, const Layout& L, const int32_t* d_coef,
         const int32_t* d_lambda, const int32_t* d_slo_us, const int32_t* d_r_fixed,
         int32_t* d_status, int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg, char* w,
         hipStream_t st, const PassOpts& opts)
{
    if (launch_candidates(p, L, d_coef, d_lambda, d_slo_us, d_r_fixed, w, st, opts) != hipSuccess)
        return THEMIS_ERR_LAUNCH;
    if (launch_minplus(p, L, w, st) != hipSuccess) return THEMIS_ERR_LAUNCH;
    if (launch_backtrack(p, L, d_status, d_cost, d_ticks, d_cfg, w, st, opts) != hipSuccess)
        return THEMIS_ERR_LAUNCH;
    return THEMIS_OK;
}

int solve(const themis_problem_t* p, const int32_t* d_coef, const int32_t* d_lambda,
          const int32_t* d_slo_us, const int32_t* d_r_fixed, int32_t* d_status,
          int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg, void* ws, size_t bytes,
          void* stream, const PassOpts& opts = PassOpts())
{
    if (!d_coef || !d_lambda || !d_slo_us || !d_status || !d_cost || !d_ticks || !d_cfg)
        return THEMIS_ERR_NULL;
    Layout L;
    int rc = check_ws(p, ws, bytes, &L);
    if (rc != THEMIS_OK) return rc;
    return pass(*p, L, d_coef, d_lambda, d_slo_us, d_r_fixed, d_status, d_cost, d_ticks, d_cfg,
                static_cast<char*>(ws), static_cast<hipStream_t>(stream), opts);
}

// Address of `scratch` on the current device, looked up once per device.
constexpr int MAX_DEVICES = 64;
std::mutex scratch_lock;
void* scratch_of_device[MAX_DEVICES];

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return THEMIS_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_of_device[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return THEMIS_ERR_LAUNCH;
        scratch_of_device[dev] = ptr;
    }
    *out = scratch_of_device[dev];
    return THEMIS_OK;
}

}  // namespace

extern "C" {

int themis_version(void) { return 102; }

int themis_check_problem(const themis_problem_t* p) { return check(p); }

size_t themis_workspace_bytes(const themis_problem_t* p)
{
    if (check(p) != THEMIS_OK) return 0;
    return make_layout(*p).total;
}

int themis_solve_joint(const themis_problem_t* p, const int32_t* d_coef,
                       const int32_t* d_lambda, const int32_t* d_slo_us, int32_t* d_status,
                       int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg, void* d_workspace,
                       size_t workspace_bytes, void* stream)
{
    return solve(p, d_coef, d_lambda, d_slo_us, nullptr, d_status, d_cost, d_ticks, d_cfg,
                 d_workspace, workspace_bytes, stream);
}

int themis_solve_joint_static(const themis_problem_t* p, const int32_t* d_coef,
                              const int32_t* d_lambda, const int32_t* d_slo_us,
                              int32_t* d_status, int32_t* d_cost, int32_t* d_ticks,
                              int32_t* d_cfg, void* stream)
{
    if (!d_coef || !d_lambda || !d_slo_us || !d_status || !d_cost || !d_ticks || !d_cfg)
        return THEMIS_ERR_NULL;
    int rc = check(p);
    if (rc != THEMIS_OK) return rc;
    const Layout L = make_layout(*p);
    if (L.total > (size_t)THEMIS_STATIC_SCRATCH_BYTES) return THEMIS_ERR_TOO_LARGE;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != THEMIS_OK) return rc;
    return pass(*p, L, d_coef, d_lambda, d_slo_us, nullptr, d_status, d_cost, d_ticks, d_cfg,
                static_cast<char*>(ws), static_cast<hipStream_t>(stream), PassOpts());
}

int themis_solve_vertical(const themis_problem_t* p, const int32_t* d_coef,
                          const int32_t* d_lambda, const int32_t* d_slo_us,
                          const int32_t* d_r_fixed, int32_t* d_status, int32_t* d_cost,
                          int32_t* d_ticks, int32_t* d_cfg, void* d_workspace,
                          size_t workspace_bytes, void* stream)
{
    if (!d_r_fixed) return THEMIS_ERR_NULL;
    return solve(p, d_coef, d_lambda, d_slo_us, d_r_fixed, d_status, d_cost, d_ticks, d_cfg,
                 d_workspace, workspace_bytes, stream);
}

int themis_solve_horizontal(const themis_problem_t* p, const int32_t* d_coef,
                            const int32_t* d_lambda, const int32_t* d_slo_us,
                            const int32_t* d_cores, int32_t* d_status, int32_t* d_cost,
                            int32_t* d_ticks, int32_t* d_cfg, void* d_workspace,
                            size_t workspace_bytes, void* stream)
{
    PassOpts opts;
    opts.c_fixed = d_cores;
    opts.c_all = d_cores ? 0 : 1;
    return solve(p, d_coef, d_lambda, d_slo_us, nullptr, d_status, d_cost, d_ticks, d_cfg,
                 d_workspace, workspace_bytes, stream, opts);
}

size_t themis_fallback_workspace_bytes(const themis_problem_t* p)
{
    if (check(p) != THEMIS_OK) return 0;
    return make_fallback_layout(make_layout(*p)).total;
}

int themis_solve_vertical_fallback(const themis_problem_t* p, const int32_t* d_coef,
                                   const int32_t* d_lambda, const int32_t* d_slo_us,
                                   const int32_t* d_r_fixed, int32_t* d_status, int32_t* d_cost,
                                   int32_t* d_ticks, int32_t* d_cfg, int32_t* d_lambda_v,
                                   int32_t* d_status_h, int32_t* d_cost_h, int32_t* d_ticks_h,
                                   int32_t* d_cfg_h, void* d_workspace, size_t workspace_bytes,
                                   void* stream)
{
    if (!d_coef || !d_lambda || !d_slo_us || !d_r_fixed || !d_status || !d_cost || !d_ticks ||
        !d_cfg || !d_lambda_v || !d_status_h || !d_cost_h || !d_ticks_h || !d_cfg_h)
        return THEMIS_ERR_NULL;
    int rc = check(p);
    if (rc != THEMIS_OK) return rc;
    const Layout L = make_layout(*p);
    const FallbackLayout F = make_fallback_layout(L);
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0 ||
        workspace_bytes < F.total)
        return THEMIS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* w = static_cast<char*>(d_workspace);
    const FallbackOut out{d_status, d_cost,     d_ticks, d_cfg,    d_lambda_v,
                          d_status_h, d_cost_h, d_ticks_h, d_cfg_h};

    // the plain vertical solve, reported for every instance
    rc = pass(*p, L, d_coef, d_lambda, d_slo_us, d_r_fixed, d_status, d_cost, d_ticks, d_cfg, w,
              st, PassOpts());
    if (rc != THEMIS_OK) return rc;
    // the search, for the instances it found no configuration for
    if (launch_fallback_search(*p, L, F, d_coef, d_lambda, d_slo_us, d_r_fixed, out, w, st) !=
        hipSuccess)
        return THEMIS_ERR_LAUNCH;
    // their vertical configuration at the rate the search settled on
    PassOpts only_active;
    only_active.sparse = 1;
    rc = pass(*p, L, d_coef, (const int32_t*)(w + F.lam_cur_off), d_slo_us, d_r_fixed, d_status,
              d_cost, d_ticks, d_cfg, w, st, only_active);
    if (rc != THEMIS_OK) return rc;
    if (launch_fallback_finish(L, F, d_lambda, out, w, st) != hipSuccess) return THEMIS_ERR_LAUNCH;
    // new instances for what the running replicas could not absorb
    PassOpts rest;
    rest.sparse = 1;
    rest.c_fixed = (const int32_t*)(w + F.cores_off);
    return pass(*p, L, d_coef, (const int32_t*)(w + F.lam_rem_off), d_slo_us, nullptr,
                d_status_h, d_cost_h, d_ticks_h, d_cfg_h, w, st, rest);
}

size_t themis_memo_workspace_bytes(const themis_problem_t* p)
{
    if (check(p) != THEMIS_OK) return 0;
    return make_memo_layout(make_layout(*p)).total;
}

int themis_solve_distinct(const themis_problem_t* p, const int32_t* d_coef,
                          const int32_t* d_lambda, const int32_t* d_slo_us,
                          const int32_t* d_r_fixed, int32_t* d_status, int32_t* d_cost,
                          int32_t* d_ticks, int32_t* d_cfg, void* d_workspace,
                          size_t workspace_bytes, void* stream)
{
    if (!d_coef || !d_lambda || !d_slo_us || !d_status || !d_cost || !d_ticks || !d_cfg)
        return THEMIS_ERR_NULL;
    int rc = check(p);
    if (rc != THEMIS_OK) return rc;
    const Layout L = make_layout(*p);
    const MemoLayout M = make_memo_layout(L);
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0 ||
        workspace_bytes < M.total)
        return THEMIS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* w = static_cast<char*>(d_workspace);
    if (launch_memo_dedupe(*p, L, M, d_coef, d_lambda, d_slo_us, d_r_fixed, d_status, d_cost,
                           d_ticks, d_cfg, w, st) != hipSuccess)
        return THEMIS_ERR_LAUNCH;
    // one pass over the instances that stand for themselves; the others carry a
    // rate of zero, which switches them off
    PassOpts only_distinct;
    only_distinct.sparse = 1;
    rc = pass(*p, L, d_coef, (const int32_t*)(w + M.lam_off), d_slo_us, d_r_fixed, d_status, d_cost,
              d_ticks, d_cfg, w, st, only_distinct);
    if (rc != THEMIS_OK) return rc;
    return launch_memo_scatter(L, M, d_status, d_cost, d_ticks, d_cfg, w, st) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

size_t themis_stability_workspace_bytes(const themis_problem_t* p)
{
    if (check(p) != THEMIS_OK) return 0;
    return make_stability_layout(make_layout(*p)).total;
}

int themis_check_stability(const themis_problem_t* p, const int32_t* d_coef,
                           const int32_t* d_lambda_now, const int32_t* d_lambda_pred,
                           const int32_t* d_slo_us, const int32_t* d_cores, int32_t* d_stable,
                           int32_t* d_status, int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg,
                           void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!d_coef || !d_lambda_now || !d_lambda_pred || !d_slo_us || !d_stable || !d_status ||
        !d_cost || !d_ticks || !d_cfg)
        return THEMIS_ERR_NULL;
    int rc = check(p);
    if (rc != THEMIS_OK) return rc;
    const Layout L = make_layout(*p);
    const StabilityLayout B = make_stability_layout(L);
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0 ||
        workspace_bytes < B.total)
        return THEMIS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* w = static_cast<char*>(d_workspace);
    PassOpts opts;
    opts.c_fixed = d_cores;
    opts.c_all = d_cores ? 0 : 1;
    int32_t* status_p = (int32_t*)(w + B.status_off);
    int32_t* cfg_p = (int32_t*)(w + B.cfg_off);
    rc = pass(*p, L, d_coef, d_lambda_pred, d_slo_us, nullptr, status_p,
              (int32_t*)(w + B.cost_off), (int32_t*)(w + B.ticks_off), cfg_p, w, st, opts);
    if (rc != THEMIS_OK) return rc;
    rc = pass(*p, L, d_coef, d_lambda_now, d_slo_us, nullptr, d_status, d_cost, d_ticks, d_cfg, w,
              st, opts);
    if (rc != THEMIS_OK) return rc;
    return launch_same_config(L, d_status, d_cfg, status_p, cfg_p, d_stable, st) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

int themis_stage_candidates(const themis_problem_t* p, const int32_t* d_coef,
                            const int32_t* d_lambda, const int32_t* d_slo_us,
                            const int32_t* d_r_fixed, void* d_workspace,
                            size_t workspace_bytes, void* stream)
{
    if (!d_coef || !d_lambda || !d_slo_us) return THEMIS_ERR_NULL;
    Layout L;
    int rc = check_ws(p, d_workspace, workspace_bytes, &L);
    if (rc != THEMIS_OK) return rc;
    return launch_candidates(*p, L, d_coef, d_lambda, d_slo_us, d_r_fixed,
                             static_cast<char*>(d_workspace),
                             static_cast<hipStream_t>(stream)) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

int themis_stage_minplus(const themis_problem_t* p, void* d_workspace, size_t workspace_bytes,
                         void* stream)
{
    Layout L;
    int rc = check_ws(p, d_workspace, workspace_bytes, &L);
    if (rc != THEMIS_OK) return rc;
    return launch_minplus(*p, L, static_cast<char*>(d_workspace),
                          static_cast<hipStream_t>(stream)) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

int themis_stage_backtrack(const themis_problem_t* p, int32_t* d_status, int32_t* d_cost,
                           int32_t* d_ticks, int32_t* d_cfg, void* d_workspace,
                           size_t workspace_bytes, void* stream)
{
    if (!d_status || !d_cost || !d_ticks || !d_cfg) return THEMIS_ERR_NULL;
    Layout L;
    int rc = check_ws(p, d_workspace, workspace_bytes, &L);
    if (rc != THEMIS_OK) return rc;
    return launch_backtrack(*p, L, d_status, d_cost, d_ticks, d_cfg,
                            static_cast<char*>(d_workspace),
                            static_cast<hipStream_t>(stream)) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

int themis_export_candidates(const themis_problem_t* p, const void* d_workspace,
                             size_t workspace_bytes, int32_t* d_lt, int32_t* d_cost,
                             void* stream)
{
    if (!d_lt || !d_cost) return THEMIS_ERR_NULL;
    Layout L;
    int rc = check_ws(p, d_workspace, workspace_bytes, &L);
    if (rc != THEMIS_OK) return rc;
    return launch_export_candidates(L, static_cast<const char*>(d_workspace), d_lt, d_cost,
                                    static_cast<hipStream_t>(stream)) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

int themis_count_relaxations(const themis_problem_t* p, const void* d_workspace,
                             size_t workspace_bytes, unsigned long long* d_count, void* stream)
{
    if (!d_count) return THEMIS_ERR_NULL;
    Layout L;
    int rc = check_ws(p, d_workspace, workspace_bytes, &L);
    if (rc != THEMIS_OK) return rc;
    return launch_count_relaxations(*p, L, static_cast<const char*>(d_workspace), d_count,
                                    static_cast<hipStream_t>(stream)) == hipSuccess
               ? THEMIS_OK
               : THEMIS_ERR_LAUNCH;
}

}  // extern "C"

// The fallback of Algorithm 1 (Section 4.4): when the replicas that are already
// running cannot meet the SLO at the arrival rate lambda, a binary search finds
// a rate they can absorb, the vertical configuration is taken at that rate, and
// new instances with the same cores serve what is left.
//
// Reading of the printed search, which does not converge as listed: the
// midpoint is (left + right) / 2 and a midpoint the replicas can absorb raises
// the lower end; the answer is the configuration at the lower end.
//
// Whether the replicas can absorb a rate does not take the dynamic program: a
// configuration within the budget exists exactly when the fastest feasible
// candidate of every model, taken together, fits it (the program then only
// chooses the cheapest such configuration).  With the replicas given, a
// candidate's latency never grows with the cores, so the fastest candidate of a
// (model, batch size) is the one at the core cap: the test costs one model
// evaluation per (model, batch size), with the very arithmetic of the candidate
// stage.  One thread runs the whole search of one instance; the configurations
// at the rate it settles on, and for the remainder, come from ordinary passes of
// the three stages over those instances only.
#include "candidate_eval.h"
#include "themis_internal.h"

namespace themis {
namespace {

enum : int32_t {
    FB_DONE = 0,   // nothing further to solve for the vertical part
    FB_FINAL = 1,  // the next vertical pass solves the instance at its lower end
};

struct FallbackPtrs {
    int32_t *status, *cost, *ticks, *cfg;          // vertical part
    int32_t* lambda_v;
    int32_t *status_h, *cost_h, *ticks_h, *cfg_h;  // new instances
    int32_t *lam_cur, *state, *lam_rem, *cores;    // workspace
};

// what the new-instance half reports when there is nothing for it to solve
__device__ __forceinline__ void close_new_instances(const FallbackPtrs& f, int i, int S,
                                                    int32_t status_h, int32_t cost_h)
{
    f.status_h[i] = status_h;
    f.cost_h[i] = cost_h;
    f.ticks_h[i] = cost_h;
    for (int x = 0; x < 3 * S; ++x) f.cfg_h[(size_t)i * S * 3 + x] = 0;
    f.lam_rem[i] = 0;
    f.state[i] = FB_DONE;
    f.lam_cur[i] = 0;
}

// After the plain vertical solve at lambda: settle the instances it solved or
// rejected, search for the others.
template <int QUEUE>
__global__ __launch_bounds__(64) void k4_search(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed, FallbackPtrs f,
    BatchList bl, int N, int S, uint32_t c_max, uint32_t r_max, uint32_t tick, double rtick,
    int coef_shared, uint32_t cs)
{
    __shared__ BatchHdr batch[THEMIS_MAX_BATCH];
    if ((int)threadIdx.x < bl.n) batch[threadIdx.x] = make_batch_hdr(bl.b[threadIdx.x]);
    __syncthreads();
    const int i = blockIdx.x * 64 + threadIdx.x;
    if (i >= N) return;
    const int32_t lam = lambda[i];
    const int32_t st = f.status[i];
    if (st != THEMIS_INFEASIBLE) {
        const bool solved = st == THEMIS_SOLVED;
        f.lambda_v[i] = solved ? lam : 0;
        close_new_instances(f, i, S, solved ? THEMIS_SOLVED : THEMIS_INVALID, solved ? 0 : -1);
        return;
    }
    // the instance passed the input check, so its budget is well defined
    const int32_t slo = slo_us[i];
    const int32_t T = (int32_t)((uint32_t)slo / tick);
    const int32_t* const cf0 = coef + (coef_shared ? 0 : (size_t)i * S * cs);
    const int32_t* const rf = r_fixed + (size_t)i * S;

    auto absorbs = [&](int32_t rate) {
        int32_t total = 0;
        for (int s = 0; s < S; ++s) {
            const int32_t* cf = cf0 + (size_t)s * cs;
            const RowHdr h = make_row_hdr(cf, cs, rate, slo, T, tick, rf[s]);
            const uint32_t pcap = (uint32_t)cf[3];
            const double d = (double)(pcap < c_max ? pcap : c_max);
            int32_t best = 0x7FFFFFFF;
            for (int j = 0; j < bl.n; ++j) {
                const Eval ev = eval_candidate<QUEUE>(h, batch[j], d, (double)r_max, (double)tick, rtick);
                if (ev.lt >= 0 && ev.lt < best) best = ev.lt;
            }
            if (best == 0x7FFFFFFF) return false;  // no candidate of this model fits at all
            total += best;
            if (total > T) return false;
        }
        return true;
    };

    int32_t lo = 1, hi = lam;
    while (hi - lo > 1) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (absorbs(mid)) lo = mid; else hi = mid;
    }
    f.lam_cur[i] = lo;
    f.state[i] = FB_FINAL;
}

// After the vertical solve at the lower end: record what the running replicas
// keep and what is left for new instances.
__global__ __launch_bounds__(256) void k4_finish(const int32_t* __restrict__ lambda,
                                                 FallbackPtrs f, int N, int S)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N || f.state[i] != FB_FINAL) return;
    const int32_t lam = lambda[i], lo = f.lam_cur[i];
    if (f.status[i] != THEMIS_SOLVED) {
        // not even the lowest rate fits: no cores to carry over
        f.lambda_v[i] = 0;
        close_new_instances(f, i, S, THEMIS_INVALID, -1);
    } else if (lo < lam) {
        // new instances for the rest, cores as in the vertical configuration
        f.lambda_v[i] = lo;
        f.lam_rem[i] = lam - lo;
        for (int s = 0; s < S; ++s) f.cores[(size_t)i * S + s] = f.cfg[((size_t)i * S + s) * 3];
        f.state[i] = FB_DONE;
        f.lam_cur[i] = 0;
    } else {
        f.lambda_v[i] = lo;
        close_new_instances(f, i, S, THEMIS_SOLVED, 0);
    }
}

FallbackPtrs pointers(const FallbackLayout& F, const FallbackOut& o, char* ws)
{
    return FallbackPtrs{o.status,   o.cost,   o.ticks,   o.cfg,   o.lambda_v,
                        o.status_h, o.cost_h, o.ticks_h, o.cfg_h,
                        (int32_t*)(ws + F.lam_cur_off), (int32_t*)(ws + F.state_off),
                        (int32_t*)(ws + F.lam_rem_off), (int32_t*)(ws + F.cores_off)};
}

}  // namespace

hipError_t launch_fallback_search(const themis_problem_t& p, const Layout& L,
                                  const FallbackLayout& F, const int32_t* d_coef,
                                  const int32_t* d_lambda, const int32_t* d_slo_us,
                                  const int32_t* d_r_fixed, const FallbackOut& out, char* ws,
                                  hipStream_t st)
{
    BatchList bl{};
    bl.n = p.n_batch;
    for (int j = 0; j < p.n_batch; ++j) bl.b[j] = p.batch_sizes[j];
    const uint32_t cs = p.profile_form == THEMIS_PROFILE_EQ1 ? 6u : 5u;
    const FallbackPtrs f = pointers(F, out, ws);
    const dim3 grid((L.N + 63) / 64), block(64);
    const double rtick = (1.0 / (double)p.tick_us) * (1.0 - 0x1p-45);
#define SEARCH(Q)                                                                              \
    hipLaunchKernelGGL(k4_search<Q>, grid, block, 0, st, d_coef, d_lambda, d_slo_us, d_r_fixed, \
                       f, bl, L.N, L.S, (uint32_t)p.c_max, (uint32_t)p.r_max,                   \
                       (uint32_t)p.tick_us, rtick, p.coef_shared, cs)
    switch (p.queue_model) {
    case THEMIS_QUEUE_SHARED: SEARCH(THEMIS_QUEUE_SHARED); break;
    case THEMIS_QUEUE_WORST_CASE: SEARCH(THEMIS_QUEUE_WORST_CASE); break;
    default: SEARCH(THEMIS_QUEUE_PER_REPLICA); break;
    }
#undef SEARCH
    return hipGetLastError();
}

hipError_t launch_fallback_finish(const Layout& L, const FallbackLayout& F,
                                  const int32_t* d_lambda, const FallbackOut& out, char* ws,
                                  hipStream_t st)
{
    hipLaunchKernelGGL(k4_finish, dim3((L.N + 255) / 256), dim3(256), 0, st, d_lambda,
                       pointers(F, out, ws), L.N, L.S);
    return hipGetLastError();
}

}  // namespace themis

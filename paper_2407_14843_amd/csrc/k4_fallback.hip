// The fallback of Algorithm 1 (Section 4.4): when the replicas that are already
// running cannot meet the SLO at the arrival rate lambda, a binary search finds
// the largest rate they can absorb, the vertical configuration is taken at that
// rate, and new instances with the same cores serve what is left.
//
// The search of every instance advances in lockstep, one pass of the three
// solve stages per halving; this kernel is the step between two passes.  It
// reads the status the last pass left for an instance, moves the ends of its
// interval and sets the rate of its next pass.  An instance whose search is
// over gets rate 0, which the next pass's input check rejects, so later passes
// skip it and its outputs stay as its last pass wrote them.
//
// Reading of the printed search, which does not converge as listed: the
// midpoint is (left + right) / 2 and a midpoint the replicas can absorb raises
// the lower end; the answer is the configuration at the lower end.
#include "themis_internal.h"

namespace themis {
namespace {

enum : int32_t {
    FB_DONE = 0,    // nothing further to solve for the vertical part
    FB_SEARCH = 1,  // the pass just run was at a midpoint
    FB_FINAL = 2,   // the pass just run was at the lower end: it is the answer
};

__global__ __launch_bounds__(256) void k4_fallback_step(
    int first, const int32_t* __restrict__ lambda, int32_t lambda_max,
    int32_t* __restrict__ status, int32_t* __restrict__ cost, int32_t* __restrict__ ticks,
    int32_t* __restrict__ cfg, int32_t* __restrict__ lam_cur, int32_t* __restrict__ left,
    int32_t* __restrict__ right, int32_t* __restrict__ state, int32_t* __restrict__ lam_rem,
    int32_t* __restrict__ cores, int32_t* __restrict__ lambda_v, int32_t* __restrict__ status_h,
    int32_t* __restrict__ cost_h, int32_t* __restrict__ ticks_h, int32_t* __restrict__ cfg_h,
    int N, int S)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    const int32_t lam = lambda[i];
    int32_t st = status[i];
    int32_t lo, hi;

    // what the new-instance half reports when there is nothing for it to solve
    auto close_h = [&](int32_t sh, int32_t ch) {
        status_h[i] = sh;
        cost_h[i] = ch;
        ticks_h[i] = ch;
        for (int x = 0; x < 3 * S; ++x) cfg_h[(size_t)i * S * 3 + x] = 0;
        lam_rem[i] = 0;
        state[i] = FB_DONE;
        lam_cur[i] = 0;
    };

    if (first) {
        // the pass just run was the plain vertical solve at lambda
        if (st != THEMIS_INVALID && lam > lambda_max) {
            // beyond the rate the caller sized the search for
            st = THEMIS_INVALID;
            status[i] = st;
            cost[i] = -1;
            ticks[i] = -1;
            for (int x = 0; x < 3 * S; ++x) cfg[(size_t)i * S * 3 + x] = 0;
        }
        if (st != THEMIS_INFEASIBLE) {
            const bool solved = st == THEMIS_SOLVED;
            lambda_v[i] = solved ? lam : 0;
            close_h(solved ? THEMIS_SOLVED : THEMIS_INVALID, solved ? 0 : -1);
            return;
        }
        lo = 1;
        hi = lam;
    } else {
        const int32_t sti = state[i];
        if (sti == FB_DONE) return;
        lo = left[i];
        hi = right[i];
        if (sti == FB_FINAL) {
            if (st == THEMIS_SOLVED && lo < lam) {
                // new instances for the rest, cores as in the vertical configuration
                lambda_v[i] = lo;
                lam_rem[i] = lam - lo;
                for (int s = 0; s < S; ++s)
                    cores[(size_t)i * S + s] = cfg[((size_t)i * S + s) * 3];
                state[i] = FB_DONE;
                lam_cur[i] = 0;
            } else if (st == THEMIS_SOLVED) {
                lambda_v[i] = lo;
                close_h(THEMIS_SOLVED, 0);
            } else {
                // not even the lowest rate fits: no cores to carry over
                lambda_v[i] = 0;
                close_h(THEMIS_INVALID, -1);
            }
            return;
        }
        const int32_t mid = lam_cur[i];
        if (st == THEMIS_SOLVED) lo = mid; else hi = mid;
    }
    left[i] = lo;
    right[i] = hi;
    const bool more = hi - lo > 1;
    state[i] = more ? FB_SEARCH : FB_FINAL;
    lam_cur[i] = more ? lo + ((hi - lo) >> 1) : lo;
}

}  // namespace

hipError_t launch_fallback_step(const Layout& L, const FallbackLayout& F, int first,
                                const int32_t* d_lambda, int32_t lambda_max,
                                const FallbackOut& o, char* ws, hipStream_t st)
{
    hipLaunchKernelGGL(k4_fallback_step, dim3((L.N + 255) / 256), dim3(256), 0, st, first,
                       d_lambda, lambda_max, o.status, o.cost, o.ticks, o.cfg,
                       (int32_t*)(ws + F.lam_cur_off), (int32_t*)(ws + F.left_off),
                       (int32_t*)(ws + F.right_off), (int32_t*)(ws + F.state_off),
                       (int32_t*)(ws + F.lam_rem_off), (int32_t*)(ws + F.cores_off), o.lambda_v,
                       o.status_h, o.cost_h, o.ticks_h, o.cfg_h, L.N, L.S);
    return hipGetLastError();
}

}  // namespace themis

// Evaluation of one candidate (cores c, batch size b) of one model: the integer
// latency model, the replica count and the latency on the tick grid.  Shared by
// the candidate stage and by the feasibility test of the fallback search, which
// must agree bit for bit.
//
// Integer model (microseconds, all roundings upward), after Eq. 1, Eq. 4 and
// the throughput constraint of Eq. 6:
//   proc  = ceil((a + k b + q b^2) / min(c,p)) + d b + o
//   n     = ceil(lambda proc / (b 1e6))   joint,  or the given replicas
//   queue = ceil((b-1) 1e6 n / lambda)    (or the forms of Eq. 4 / Eq. 3)
//   lt    = ceil((proc + queue) / tick)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "themis.h"

namespace themis {

// All quantities of the model are integers below 2^53 (see the input rules in
// themis.h), so they are carried in double precision, where sums, products and
// fused multiply-adds of such integers are exact; gfx950 issues fp64 FMAs at the
// full vector rate, while 64-bit integer multiplies and divides are several
// times slower.

// A reciprocal that is never above 1/d and at most 2^-44 (relative) below it:
// hardware estimate, two Newton steps (enough to reach full precision from an
// estimate good to only 2^-13), then a nudge downward.
__device__ __forceinline__ double recip_below(double d)
{
    double r = __builtin_amdgcn_rcp(d);
    r = __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);
    r = __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);
    return r * (1.0 - 0x1p-45);
}

// ceil(n / d) for integers 0 <= n, 1 <= d, n + d < 2^53, quotient < 2^43, with
// rd = recip_below(d).  ceil(n/d) = floor(m/d) for m = n + d - 1.  m * rd is
// below m/d by less than one, so its floor is the true floor or one less; the
// exact remainder m - q*d (one FMA) tells which.
__device__ __forceinline__ double ceil_div_d(double n, double d, double rd)
{
    const double m = n + (d - 1.0);
    const double q = __builtin_floor(m * rd);
    const double r = __builtin_fma(-q, d, m);
    return r >= d ? q + 1.0 : q;
}

// What every candidate of a row shares.
struct RowHdr {
    double a, k, q, o;   // profile coefficients
    double d;            // Eq. 1's delta (0 when the profile has five coefficients)
    double p;            // core cap
    double lam, rlam;    // arrival rate and recip_below() of it
    double lt_den, rlt_den;  // lambda * tick and recip_below() of it
    double slo, T;       // SLO in microseconds, budget in ticks
    double n_given;      // replicas (vertical) or 0 (joint: derive)
};

// What every candidate with the same batch size shares.
struct BatchHdr {
    double b, b2;        // batch size and its square
    double M, rM;        // b * 1e6 and recip_below() of it
    double w;            // (b - 1) * 1e6
};

// Latency in ticks and replica count of candidate (d = min(c,p), b), or lt < 0
// when it is infeasible.  Both are the same for every c >= p.
struct Eval {
    int32_t lt, n;
};

template <int QUEUE>
__device__ __forceinline__ Eval eval_candidate(const RowHdr& h, const BatchHdr& bh, double d,
                                               double r_max, double tick, double rtick)
{
    // Straight-line: every test only clears `ok`, so the lanes of a wavefront
    // stay together.  A candidate that fails an early test may push later
    // intermediates past 2^53; they are then inexact but never used.
    const double num = __builtin_fma(h.q, bh.b2, __builtin_fma(h.k, bh.b, h.a));  // < 2^41
    const double proc = ceil_div_d(num, d, recip_below(d)) + __builtin_fma(h.d, bh.b, h.o);
    // anything slower than the SLO also exceeds T ticks; cutting it here keeps
    // every later product of a surviving candidate below 2^53
    bool ok = proc <= h.slo;
    const double lp = h.lam * proc;  // < 2^51
    const bool derive = h.n_given <= 0.0;
    // least n with lambda <= n * b / proc; at least 1 since lambda * proc >= 1
    double n = ceil_div_d(lp, bh.M, bh.rM);
    n = derive ? n : h.n_given;
    // joint: no more than r_max replicas; vertical: the given ones must carry lambda
    ok = ok && (derive ? lp <= r_max * bh.M : lp <= n * bh.M);
    // batch-fill wait: per replica (each sees lambda / n) or Eq. 4's shared queue
    const double qn = QUEUE == THEMIS_QUEUE_PER_REPLICA ? bh.w * n : bh.w;  // < 2^45
    ok = ok && qn <= (h.slo - proc) * h.lam;  // proc + queue <= SLO
    double lt;
    if (QUEUE == THEMIS_QUEUE_WORST_CASE) {
        double queue = ceil_div_d(qn, h.lam, h.rlam);
        // Eq. 3: all n instances busy.  floor(x / lambda) = ceil((x + 1) / lambda) - 1;
        // x = (n b + 1) 1e6 < 2^46
        const double x = __builtin_fma(n, bh.M, 1.0e6);
        const double busy = proc - (ceil_div_d(x + 1.0, h.lam, h.rlam) - 1.0);
        queue = busy > queue ? busy : queue;
        ok = ok && proc + queue <= h.slo;
        lt = ceil_div_d(proc + queue, tick, rtick);
    } else {
        // ceil((proc + ceil(qn / lambda)) / tick) = ceil((proc lambda + qn) / (lambda tick)):
        // one division; numerator <= SLO * lambda < 2^51 for a surviving candidate
        lt = ceil_div_d(__builtin_fma(proc, h.lam, qn), h.lt_den, h.rlt_den);
    }
    ok = ok && lt <= h.T;
    return Eval{ok ? (int32_t)lt : -1, ok ? (int32_t)n : 0};
}

// The row-level and batch-level parts of the above from the raw inputs.
__device__ __forceinline__ RowHdr make_row_hdr(const int32_t* cf, uint32_t cs, int32_t lambda,
                                               int32_t slo_us, int32_t T, uint32_t tick,
                                               int32_t n_given)
{
    RowHdr h;
    h.a = (double)cf[0];
    h.k = (double)cf[1];
    h.q = (double)cf[2];
    h.p = (double)cf[3];
    h.o = (double)cf[4];
    h.d = cs == 6 ? (double)cf[5] : 0.0;
    h.lam = (double)lambda;
    h.rlam = recip_below(h.lam);
    h.lt_den = h.lam * (double)tick;
    h.rlt_den = recip_below(h.lt_den);
    h.slo = (double)slo_us;
    h.T = (double)T;
    h.n_given = (double)n_given;
    return h;
}

__device__ __forceinline__ BatchHdr make_batch_hdr(int32_t b)
{
    BatchHdr bh;
    bh.b = (double)b;
    bh.b2 = bh.b * bh.b;
    bh.M = bh.b * 1.0e6;
    bh.rM = recip_below(bh.M);
    bh.w = (bh.b - 1.0) * 1.0e6;
    return bh;
}

}  // namespace themis

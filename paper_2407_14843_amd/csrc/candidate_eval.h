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

// ceil(n / d) for integers 0 <= n <= 2^42, d >= 1, with rd = recip_below(d): one
// multiply and a ceiling.  Write n = k d + r, 0 <= r < d.  If r = 0, n * rd lies
// in (k - 1, k] (it is below k by at most k 2^-44 < 1) and rounds to a value in
// that range, k itself being representable: the ceiling is k.  If r >= 1,
// n * rd >= (k + 1/d)(1 - 2^-44) = k + (1 - n 2^-44) / d >= k + 0.75 / d, which
// is above k by far more than half a unit in the last place of k (k 2^-53 <=
// 2^-11 / d), and at most n / d < k + 1: the product rounds into (k, k + 1] and
// the ceiling is k + 1.
__device__ __forceinline__ double ceil_div_small(double n, double rd)
{
    return __builtin_ceil(n * rd);
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

// SMALL: the row's lambda * SLO is at most 2^42, so every numerator of a
// candidate that survives the tests is, and the divisions take the short form
// (a candidate whose last numerator exceeds 2^42 has a quotient above the
// budget T, since T * lambda * tick <= lambda * SLO, and still gets one: the
// product is above T by at least 0.75 / (lambda * tick), far more than a
// rounding).  rd = recip_below(d).
// NMODE: where the replica count comes from: N_DERIVED (joint), N_GIVEN
// (vertical, h.n_given), or N_EITHER (h.n_given decides at run time).
constexpr int N_EITHER = 0, N_DERIVED = 1, N_GIVEN = 2;

template <int QUEUE, bool SMALL, int NMODE>
__device__ __forceinline__ Eval eval_candidate_rd(const RowHdr& h, const BatchHdr& bh, double d,
                                                  double rd, double r_max, double tick,
                                                  double rtick)
{
    // Straight-line: every test only clears a bit of `ok`, so the lanes of a
    // wavefront stay together.  A candidate that fails an early test may push
    // later intermediates past 2^53; they are then inexact but never used.
    const double num = __builtin_fma(h.q, bh.b2, __builtin_fma(h.k, bh.b, h.a));  // < 2^41
    const double proc = ceil_div_small(num, rd) + __builtin_fma(h.d, bh.b, h.o);
    // anything slower than the SLO also exceeds T ticks; cutting it here keeps
    // every later product of a surviving candidate below 2^53
    int ok = (int)(proc <= h.slo);
    const double lp = h.lam * proc;  // < 2^51
    const bool derive = NMODE == N_DERIVED || (NMODE == N_EITHER && h.n_given <= 0.0);
    // least n with lambda <= n * b / proc; at least 1 since lambda * proc >= 1
    double n = h.n_given;
    if (NMODE != N_GIVEN) {
        const double need = SMALL ? ceil_div_small(lp, bh.rM) : ceil_div_d(lp, bh.M, bh.rM);
        n = derive ? need : n;
    }
    // joint: no more than r_max replicas; vertical: the given ones must carry lambda
    // (either way n <= r_max < 2^15 from here on)
    ok &= (int)(lp <= (derive ? r_max : n) * bh.M);
    // batch-fill wait: per replica (each sees lambda / n) or Eq. 4's shared queue
    const double qn = QUEUE == THEMIS_QUEUE_PER_REPLICA ? bh.w * n : bh.w;  // < 2^45
    double lt;
    if (QUEUE == THEMIS_QUEUE_WORST_CASE) {
        double queue = ceil_div_d(qn, h.lam, h.rlam);
        // Eq. 3: all n instances busy.  floor(x / lambda) = ceil((x + 1) / lambda) - 1;
        // x = (n b + 1) 1e6 < 2^46
        const double x = __builtin_fma(n, bh.M, 1.0e6);
        const double busy = proc - (ceil_div_d(x + 1.0, h.lam, h.rlam) - 1.0);
        queue = busy > queue ? busy : queue;
        ok &= (int)(proc + queue <= h.slo);
        lt = ceil_div_d(proc + queue, tick, rtick);
    } else {
        // ceil((proc + ceil(qn / lambda)) / tick) = ceil((proc lambda + qn) / (lambda tick)):
        // one division; numerator < 2^52 for a candidate that passed the tests above.
        // (lt <= T below also says proc + queue <= SLO, T being floor(SLO / tick).)
        const double top = __builtin_fma(proc, h.lam, qn);
        lt = SMALL ? ceil_div_small(top, h.rlt_den) : ceil_div_d(top, h.lt_den, h.rlt_den);
    }
    ok &= (int)(lt <= h.T);
    return Eval{ok ? (int32_t)lt : -1, ok ? (int32_t)n : 0};
}

template <int QUEUE>
__device__ __forceinline__ Eval eval_candidate(const RowHdr& h, const BatchHdr& bh, double d,
                                               double r_max, double tick, double rtick)
{
    return eval_candidate_rd<QUEUE, false, N_EITHER>(h, bh, d, recip_below(d), r_max, tick, rtick);
}

// Whether a row's candidates may take the short divisions (see eval_candidate_rd).
__device__ __forceinline__ bool row_is_small(const RowHdr& h) { return h.lam * h.slo <= 0x1p42; }

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

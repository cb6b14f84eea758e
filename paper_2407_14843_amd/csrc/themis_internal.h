// Internal layout shared by the kernels and the host entry points.
// Not part of the public interface (that is include/themis.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "themis.h"

namespace themis {

// DP values are unsigned 16-bit.  Feasible totals are <= THEMIS_COST_LIMIT,
// "no configuration" is F_INF, and F_INF + (largest single cost) still fits,
// so the hot loop needs no saturation.
constexpr uint32_t F_INF = 0x8000u;
constexpr uint32_t F_INF2 = 0x80008000u;

// Workspace carve-up.  Every region starts on a 256-byte boundary.
//   lt    int32 [N][S][K]   latency of a candidate in ticks, -1 = infeasible
//   cost  int32 [N][S][K]   replicas*cores of a candidate,   -1 = infeasible
//   frow  u16   [N][S][row_stride]  f[s][t] of the min-plus recurrence
//   tmeta int32 [N]         budget T of the instance, -1 = invalid instance
struct Layout {
    size_t lt_off, cost_off, frow_off, tmeta_off, total;
    int32_t N, S, K, t_max, row_stride;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline Layout make_layout(const themis_problem_t& p)
{
    Layout L{};
    L.N = p.n_inst;
    L.S = p.n_stage;
    L.K = p.c_max * p.n_batch;
    L.t_max = p.slo_max_us / p.tick_us;
    // two cells of slack so a paired 32-bit store of cells (T, T+1) stays in
    // the row; rows start 256-byte aligned
    L.row_stride = (int32_t)((L.t_max + 2 + 127) / 128 * 128);
    size_t nsk = (size_t)L.N * L.S * L.K;
    size_t at = 0;
    L.lt_off = at;    at = align256(at + nsk * sizeof(int32_t));
    L.cost_off = at;  at = align256(at + nsk * sizeof(int32_t));
    L.frow_off = at;  at = align256(at + (size_t)L.N * L.S * L.row_stride * sizeof(uint16_t));
    L.tmeta_off = at; at = align256(at + (size_t)L.N * sizeof(int32_t));
    L.total = at;
    return L;
}

struct BatchList {
    int32_t n;
    int32_t b[THEMIS_MAX_BATCH];
};

// kernel launchers (one per stage), defined next to their kernels
hipError_t launch_candidates(const themis_problem_t& p, const Layout& L,
                             const int32_t* d_coef, const int32_t* d_lambda,
                             const int32_t* d_slo_us, const int32_t* d_r_fixed,
                             char* ws, hipStream_t st);
hipError_t launch_minplus(const themis_problem_t& p, const Layout& L, char* ws,
                          hipStream_t st);
hipError_t launch_backtrack(const themis_problem_t& p, const Layout& L,
                            int32_t* d_status, int32_t* d_cost, int32_t* d_ticks,
                            int32_t* d_cfg, char* ws, hipStream_t st);
hipError_t launch_count_relaxations(const Layout& L, const char* ws,
                                    unsigned long long* d_count, hipStream_t st);

}  // namespace themis

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

// One candidate as stage 1 leaves it for stages 2 and 3.
struct __attribute__((aligned(8))) CandEntry {
    int32_t lt;    // latency in ticks, -1 = infeasible
    int32_t cost;  // replicas * cores,  -1 = infeasible
};

// ---- work classes of the min-plus stage ---------------------------------
// An instance with budget T owns T+1 cells.  The "wide" kernel gives every
// wavefront a chunk of WIDE_CHUNK cells (64 lanes x 4 quads of 4 cells), so an
// instance needs ceil((T+1)/WIDE_CHUNK) wavefronts; instances are grouped by
// that count (rounded up to the next entry of CLS_WAVES) and each group is
// launched with a workgroup of exactly that many wavefronts and the LDS that
// goes with it.  Budgets beyond 16 chunks go to the "narrow" kernel, which
// keeps two instead of four row copies and so fits rows twice as long.
constexpr int WIDE_V = 4;                        // quads (4 cells) per lane
constexpr int WIDE_CHUNK = 64 * 4 * WIDE_V;      // 1024 cells per wavefront
constexpr int N_WIDE_CLS = 10;
constexpr int CLS_WAVES[N_WIDE_CLS] = {1, 2, 3, 4, 6, 8, 10, 12, 14, 16};
constexpr int NARROW_CLS = N_WIDE_CLS;           // class index of the narrow kernel
constexpr int N_CLS = N_WIDE_CLS + 1;
constexpr int WIDE_MAX_CELLS = 16 * WIDE_CHUNK;  // 16384

__host__ __device__ inline int class_of_budget(int T)
{
    int cells = T + 1;
    if (cells > WIDE_MAX_CELLS) return NARROW_CLS;
    int nw = (cells + WIDE_CHUNK - 1) / WIDE_CHUNK;
    int c = 0;
    while (CLS_WAVES[c] < nw) ++c;
    return c;
}

// Workspace carve-up.  Every region starts on a 256-byte boundary.
//   cand   CandEntry [N][S][Kp]   Kp = K rounded up to 8; pad entries infeasible
//   frow   u16 [N][S][row_stride] f[s][t] of the min-plus recurrence
//   tmeta  int32 [N]              budget T of the instance, -1 = invalid instance
//   order  int32 [N_CLS][N]       instance ids grouped by work class
//   ctrl   int32 [2][N_CLS]       per class: number of instances, queue cursor
struct Layout {
    size_t cand_off, frow_off, tmeta_off, order_off, ctrl_off, total;
    int32_t N, S, K, Kp, t_max, row_stride;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline Layout make_layout(const themis_problem_t& p)
{
    Layout L{};
    L.N = p.n_inst;
    L.S = p.n_stage;
    L.K = p.c_max * p.n_batch;
    L.Kp = (L.K + 7) / 8 * 8;
    L.t_max = p.slo_max_us / p.tick_us;
    // a lane stores the four cells of a quad at once, so up to three cells
    // past T are written; rows start 256-byte aligned
    L.row_stride = (int32_t)((L.t_max + 4 + 127) / 128 * 128);
    size_t at = 0;
    L.cand_off = at;  at = align256(at + (size_t)L.N * L.S * L.Kp * sizeof(CandEntry));
    L.frow_off = at;  at = align256(at + (size_t)L.N * L.S * L.row_stride * sizeof(uint16_t));
    L.tmeta_off = at; at = align256(at + (size_t)L.N * sizeof(int32_t));
    L.order_off = at; at = align256(at + (size_t)N_CLS * L.N * sizeof(int32_t));
    L.ctrl_off = at;  at = align256(at + (size_t)2 * N_CLS * sizeof(int32_t));
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
hipError_t launch_export_candidates(const Layout& L, const char* ws, int32_t* d_lt,
                                    int32_t* d_cost, hipStream_t st);
hipError_t launch_count_relaxations(const Layout& L, const char* ws,
                                    unsigned long long* d_count, hipStream_t st);

hipError_t launch_lds_probe(int width, int misalign, int iters, int blocks, uint32_t* sink,
                            hipStream_t st);

}  // namespace themis

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

// Stage 1 leaves one table of 8-byte entries, ordered within a row by latency
// bucket lt >> BUCKET_SHIFT (feasible candidates only), so that the
// candidates that can reach a given stretch of the budget grid form a prefix
// of the row.  An entry holds
//   shift  the byte offset that turns "my place in row copy 0" into "the
//          aligned place lt cells below, in the copy whose shift fits"; it
//          depends on the LDS layout of the instance's work class and is
//          invertible (lt_of_shift), so lt itself is not stored;
//   ck     cost | k << 16: replicas * cores (<= 32767) and the candidate index.
// A row's entries are its first bcum[nb] slots; infeasible candidates are not
// written, and the slots beyond hold whatever they held before.
struct __attribute__((aligned(8))) StepEntry {
    uint32_t shift;
    uint32_t ck;
};
constexpr int BUCKET_SHIFT = 9;                 // 512 cells per bucket
constexpr int BUCKET_CELLS = 1 << BUCKET_SHIFT;
constexpr int MAX_BUCKETS = (THEMIS_MAX_TICKS >> BUCKET_SHIFT) + 1;   // 64
constexpr int MAX_CAND = THEMIS_MAX_CANDIDATES; // candidates per model (LDS staging, 13-bit k)

// ---- work classes of the min-plus stage ---------------------------------
// An instance with budget T owns T+1 cells.  The "wide" kernel gives every
// wavefront WIDE_CHUNK cells (two positions of 512), so an instance needs
// ceil((T+1)/WIDE_CHUNK) wavefronts; instances are grouped by that count
// (rounded up to the next entry of CLS_WAVES) and each group is launched with a
// workgroup of exactly that many wavefronts and the LDS that goes with it.
// Budgets beyond 16 chunks go to the "narrow" kernel, whose sixteen wavefronts
// take static chunks of a row twice as long.
constexpr int WIDE_CHUNK = 1024;                 // cells per wavefront
constexpr int N_WIDE_CLS = 10;
constexpr int CLS_WAVES[N_WIDE_CLS] = {1, 2, 3, 4, 6, 8, 10, 12, 14, 16};
// The same table in closed form, for device code: indexing the array with a
// value not known at compile time is a load from memory, which the walk of
// stage 3 would wait for once per group of entries.
__host__ __device__ constexpr int cls_waves(int c) { return c < 4 ? c + 1 : 2 * (c - 1); }
constexpr bool cls_waves_agree()
{
    for (int c = 0; c < N_WIDE_CLS; ++c)
        if (cls_waves(c) != CLS_WAVES[c]) return false;
    return true;
}
static_assert(cls_waves_agree(), "cls_waves() is CLS_WAVES in closed form");
constexpr int NARROW_CLS = N_WIDE_CLS;           // class index of the narrow kernel
constexpr int N_CLS = N_WIDE_CLS + 1;
constexpr int WIDE_MAX_CELLS = 16 * WIDE_CHUNK;  // 16384

__host__ __device__ inline int class_of_budget(int T)
{
    int cells = T + 1;
    if (cells > WIDE_MAX_CELLS) return NARROW_CLS;
    int nw = (cells + WIDE_CHUNK - 1) / WIDE_CHUNK;
    // the first class with at least nw wavefronts: 1 2 3 4 6 8 10 12 14 16
    return nw <= 4 ? nw - 1 : (nw + 1) / 2 + 1;
}

// ---- LDS geometry of the min-plus stage (stage 1 bakes it into StepEntry) --
// Wide kernel: two copies of the row, copy m holds cell t at half-word
// (WIDE_PAD_BYTES/2 + t - m); each copy is WIDE_PAD_BYTES of F_INF followed by
// two positions (2 * 512 cells) per wavefront of the class.
constexpr int WIDE_PAD_BYTES = BUCKET_CELLS * 2;
constexpr int WIDE_COPIES = 2;

__host__ __device__ inline int wide_copy_bytes(int waves)
{
    return WIDE_PAD_BYTES + waves * WIDE_CHUNK * 2;
}

// lt = 2h - m: read copy m, h pairs (4 bytes) below the lane's pair.
__host__ __device__ inline uint32_t wide_shift(uint32_t lt, int copy_bytes)
{
    return (lt & 1u) * (uint32_t)copy_bytes - 4u * ((lt + 1u) >> 1);
}

// Narrow kernel: 16 wavefronts x 1024 dwords; copy A holds cells (2j, 2j+1) in
// dword j, copy B cells (2j+1, 2j+2); each copy is preceded by one wavefront's
// worth of F_INF.
constexpr int NAR_WAVES = 16;
constexpr int NAR_CHUNK_DW = 1024;                       // dwords per wavefront
constexpr int NAR_COPY_DW = (NAR_WAVES + 1) * NAR_CHUNK_DW;

// even lt = 2h: A[j - h]; odd lt = 2h + 1: B[j - h - 1]; in bytes from LDS start
__host__ __device__ inline uint32_t narrow_shift(uint32_t lt)
{
    const uint32_t h = lt >> 1;
    return 4u * ((lt & 1u) ? (uint32_t)(NAR_COPY_DW + NAR_CHUNK_DW - 1) - h
                           : (uint32_t)NAR_CHUNK_DW - h);
}

// Inverses.  Wide: the term 4h is less than one copy, so the sign of the offset
// tells the copy.  Narrow: even shifts lie at or below the pad, odd ones above it.
__host__ __device__ inline uint32_t wide_lt_of_shift(uint32_t shift, int copy_bytes)
{
    const int32_t sh = (int32_t)shift;
    // sh = m * copy_bytes - 4 h with 0 <= 4 h < copy_bytes
    const int32_t m = sh > 0;
    const uint32_t back = (uint32_t)(m * copy_bytes - sh);
    return 2u * (back >> 2) - (uint32_t)m;
}

__host__ __device__ inline uint32_t narrow_lt_of_shift(uint32_t shift)
{
    const int32_t x = (int32_t)shift / 4;
    return x <= NAR_CHUNK_DW ? 2u * (uint32_t)(NAR_CHUNK_DW - x)
                             : 2u * (uint32_t)(NAR_COPY_DW + NAR_CHUNK_DW - 1 - x) + 1u;
}

// One launch per class pays a start and a thinning end per class, so classes
// are served in groups: the launch of a group's highest class (the "head", whose
// geometry fits every shorter row) also serves the classes below it down to the
// next head.  class_map holds, four bits per wide class, the head that serves it.
__host__ __device__ inline int head_of_class(int c, uint64_t class_map)
{
    return c == NARROW_CLS ? c : (int)((class_map >> (4 * c)) & 15u);
}

__host__ __device__ inline int effective_class(int T, uint64_t class_map)
{
    return head_of_class(class_of_budget(T), class_map);
}

// The first and the last model of the recurrence have shortcuts in the wide
// kernel (a scan instead of sweeps; the answer without the row).  They pay when
// they replace enough sweeping: n entries over npos positions, shared by the
// workgroup's wavefronts.  Used by the kernel and by the relaxation count.
__host__ __device__ inline bool worth_shortcut(int n_entries, int npos, int waves)
{
    return n_entries * npos >= 24 * waves;
}

struct Layout;
struct MinplusPlan {
    int cus;          // compute units of the current device
    int top;          // highest class any instance can be in
    int top_wide;     // highest wide class in use
    uint64_t class_map;  // see head_of_class()
};
MinplusPlan make_plan(const Layout& L);

// Workspace carve-up.  Every region starts on a 256-byte boundary.
//   step   StepEntry [N*S][Kp] bucket-ordered; Kp = K rounded up to 8
//   bcum   u16 [N*S][nbs]      bcum[j] = entries of the row with bucket < j, j = 0..nb
//   frow   u16 [N][S][row_stride] f[s][t] of the min-plus recurrence
//   tmeta  int32 [N]           budget T of the instance, -1 = invalid instance
//   ans    int32 [N][2]        least cost and least latency attaining it, where stage 2
//                              finds them itself; latency -1 = stage 3 reads them off row 0
//   order  int32 [N_CLS][N]    instance ids grouped by work class
//   ctrl   int32 [2][N_CLS]    per class: number of instances, queue cursor
struct Layout {
    size_t step_off, bcum_off, frow_off, tmeta_off, ans_off, order_off, ctrl_off, total;
    int32_t N, S, K, Kp, t_max, row_stride, nb, nbs;
    int32_t fixed_form;  // stage 2 runs its kernel for pruned rows (the launch plan depends on it)
    int32_t step_rows;   // stage 2 keeps rows as step functions (likewise)
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
    L.fixed_form = (p.prune & THEMIS_PRUNE_DOMINATED) != 0 && (p.prune & THEMIS_PRUNE_STEPS) == 0;
    L.step_rows = (p.prune & THEMIS_PRUNE_STEPS) != 0;
    L.nb = (L.t_max >> BUCKET_SHIFT) + 1;
    L.nbs = (L.nb + 1 + 1) / 2 * 2;
    // a lane stores the four cells of a quad at once, so up to three cells
    // past T are written; rows start 256-byte aligned
    L.row_stride = (int32_t)((L.t_max + 4 + 127) / 128 * 128);
    size_t rows = (size_t)L.N * L.S;
    size_t at = 0;
    L.step_off = at;  at = align256(at + rows * L.Kp * sizeof(StepEntry));
    L.bcum_off = at;  at = align256(at + rows * L.nbs * sizeof(uint16_t));
    L.frow_off = at;  at = align256(at + rows * L.row_stride * sizeof(uint16_t));
    L.tmeta_off = at; at = align256(at + (size_t)L.N * sizeof(int32_t));
    L.ans_off = at;   at = align256(at + (size_t)2 * L.N * sizeof(int32_t));
    L.order_off = at; at = align256(at + (size_t)N_CLS * L.N * sizeof(int32_t));
    L.ctrl_off = at;  at = align256(at + (size_t)2 * N_CLS * sizeof(int32_t));
    L.total = at;
    return L;
}

struct BatchList {
    int32_t n;
    int32_t b[THEMIS_MAX_BATCH];
};

// Options of one pass over the three stages.
//   c_fixed  int32 [N][S] or null: only candidates with exactly these cores
//            compete (an entry outside 1..c_max makes the instance invalid)
//   c_all    the same cores for every model of every instance (host value)
//   sparse   nonzero: instances that fail the input check are skipped outright
//            (no table rows, no outputs written) instead of being reported;
//            used by multi-pass solves that switch instances off by handing
//            them an arrival rate of zero
struct PassOpts {
    const int32_t* c_fixed = nullptr;
    int c_all = 0;  // nonzero and c_fixed null: these cores for every model
    int sparse = 0;
};

// kernel launchers (one per stage), defined next to their kernels
hipError_t launch_candidates(const themis_problem_t& p, const Layout& L,
                             const int32_t* d_coef, const int32_t* d_lambda,
                             const int32_t* d_slo_us, const int32_t* d_r_fixed,
                             char* ws, hipStream_t st, const PassOpts& opts = PassOpts());
hipError_t launch_minplus(const themis_problem_t& p, const Layout& L, char* ws,
                          hipStream_t st);
// the min-plus stage with rows as step functions, for one group of classes
hipError_t launch_steps_group(const Layout& L, char* ws, hipStream_t st, int cls, int low,
                              int cus);
// lt of an entry of an instance with budget T (see StepEntry)
__host__ __device__ inline uint32_t lt_of_entry(uint32_t shift, int T, uint64_t class_map)
{
    const int cls = effective_class(T, class_map);
    if (cls == NARROW_CLS) return narrow_lt_of_shift(shift);
    return wide_lt_of_shift(shift, wide_copy_bytes(cls_waves(cls)));
}

hipError_t launch_backtrack(const themis_problem_t& p, const Layout& L,
                            int32_t* d_status, int32_t* d_cost, int32_t* d_ticks,
                            int32_t* d_cfg, char* ws, hipStream_t st,
                            const PassOpts& opts = PassOpts());

// State of the vertical solve with fallback, appended to the workspace after
// Layout::total (every region 256-byte aligned):
//   lam_cur int32 [N]  rate of the second vertical pass, 0 = instance switched off
//   state   int32 [N]  see k4_fallback.hip
//   lam_rem int32 [N]  rate left for new instances, 0 = none
//   cores   int32 [N][S] cores of the vertical configuration
struct FallbackLayout {
    size_t lam_cur_off, state_off, lam_rem_off, cores_off, total;
};

inline FallbackLayout make_fallback_layout(const Layout& L)
{
    FallbackLayout F{};
    size_t at = L.total;
    const size_t n4 = (size_t)L.N * sizeof(int32_t);
    F.lam_cur_off = at; at = align256(at + n4);
    F.state_off = at;   at = align256(at + n4);
    F.lam_rem_off = at; at = align256(at + n4);
    F.cores_off = at;   at = align256(at + n4 * L.S);
    F.total = at;
    return F;
}

struct FallbackOut {
    int32_t *status, *cost, *ticks, *cfg;          // vertical part
    int32_t* lambda_v;
    int32_t *status_h, *cost_h, *ticks_h, *cfg_h;  // new instances
};
hipError_t launch_fallback_search(const themis_problem_t& p, const Layout& L,
                                  const FallbackLayout& F, const int32_t* d_coef,
                                  const int32_t* d_lambda, const int32_t* d_slo_us,
                                  const int32_t* d_r_fixed, const FallbackOut& out, char* ws,
                                  hipStream_t st);
hipError_t launch_fallback_finish(const Layout& L, const FallbackLayout& F,
                                  const int32_t* d_lambda, const FallbackOut& out, char* ws,
                                  hipStream_t st);
// Results of the solve at the predicted rate, appended to the workspace after
// Layout::total for the stability test: status, cost, ticks int32 [N] each and
// cfg int32 [N][S][3].
struct StabilityLayout {
    size_t status_off, cost_off, ticks_off, cfg_off, total;
};

inline StabilityLayout make_stability_layout(const Layout& L)
{
    StabilityLayout B{};
    size_t at = L.total;
    const size_t n4 = (size_t)L.N * sizeof(int32_t);
    B.status_off = at; at = align256(at + n4);
    B.cost_off = at;   at = align256(at + n4);
    B.ticks_off = at;  at = align256(at + n4);
    B.cfg_off = at;    at = align256(at + n4 * L.S * 3);
    B.total = at;
    return B;
}

// State of the solve that handles every distinct instance once, appended to
// the workspace after Layout::total:
//   rep    int32 [N]      index of the instance that stands for this one's inputs
//   lam    int32 [N]      arrival rates of the pass: 0 unless the instance stands for itself
//   table  int32 [slots]  hash table of instance indices, slots = power of two >= 2 N
struct MemoLayout {
    size_t rep_off, lam_off, table_off, total;
    uint32_t slots;
};

inline MemoLayout make_memo_layout(const Layout& L)
{
    MemoLayout M{};
    size_t at = L.total;
    const size_t n4 = (size_t)L.N * sizeof(int32_t);
    M.slots = 256u;
    while (M.slots < 2u * (uint32_t)L.N) M.slots <<= 1;
    M.rep_off = at;   at = align256(at + n4);
    M.lam_off = at;   at = align256(at + n4);
    M.table_off = at; at = align256(at + (size_t)M.slots * sizeof(int32_t));
    M.total = at;
    return M;
}

hipError_t launch_memo_dedupe(const themis_problem_t& p, const Layout& L, const MemoLayout& M,
                              const int32_t* d_coef, const int32_t* d_lambda,
                              const int32_t* d_slo_us, const int32_t* d_r_fixed,
                              int32_t* d_status, int32_t* d_cost, int32_t* d_ticks,
                              int32_t* d_cfg, char* ws, hipStream_t st);
hipError_t launch_memo_scatter(const Layout& L, const MemoLayout& M, int32_t* d_status,
                               int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg, const char* ws,
                               hipStream_t st);

hipError_t launch_same_config(const Layout& L, const int32_t* status_now, const int32_t* cfg_now,
                              const int32_t* status_pred, const int32_t* cfg_pred,
                              int32_t* stable, hipStream_t st);

hipError_t launch_export_candidates(const Layout& L, const char* ws, int32_t* d_lt,
                                    int32_t* d_cost, hipStream_t st);
hipError_t launch_count_relaxations(const themis_problem_t& p, const Layout& L, const char* ws,
                                    unsigned long long* d_count, hipStream_t st);

}  // namespace themis

// Stage 1: candidate tables.
//
// Algorithms 1 and 2 (Section 4.4) recompute a candidate's latency l, queueing
// delay q and throughput h inside the budget loop although none of them depends
// on the budget.  This kernel evaluates each (model, cores, batch) candidate of
// each instance exactly once and writes its latency in grid ticks and its cost
// (replicas * cores) to HBM, packed into one word, each row ordered by latency
// bucket so that the min-plus stage can work on prefixes of a row.
//
// Integer model (microseconds, all roundings upward), after Eq. 1, Eq. 4 and
// the throughput constraint of Eq. 6:
//   proc  = ceil((a + k b + q b^2) / min(c,p)) + o
//   n     = ceil(lambda proc / (b 1e6))   joint,  or the given replicas
//   queue = ceil((b-1) 1e6 n / lambda)
//   lt    = ceil((proc + queue) / tick),  cost = n c
// A candidate is dropped (lt = cost = -1) when n exceeds r_max, when the given
// replicas cannot carry lambda, or when lt exceeds the instance's budget T.
#include "themis_internal.h"

namespace themis {
namespace {

// floor(n / d) for n < 2^53, 1 <= d < 2^32, quotient < 2^32.
// A double-precision estimate (exact conversion, reciprocal refined by one
// Newton step) is corrected by exact 64-bit integer arithmetic, so the result
// does not depend on how the estimate rounds.  *rem receives n - q*d.
__device__ __forceinline__ uint32_t floor_div_u64(uint64_t n, uint32_t d, uint64_t* rem)
{
    double dd = (double)d;
    double r = __builtin_amdgcn_rcp(dd);
    r = __builtin_fma(__builtin_fma(-dd, r, 1.0), r, r);
    uint64_t q = (uint64_t)((double)n * r);
    uint64_t prod = q * (uint64_t)d;
    while (prod > n) { --q; prod -= d; }
    while (n - prod >= d) { ++q; prod += d; }
    *rem = n - prod;
    return (uint32_t)q;
}

__device__ __forceinline__ uint32_t ceil_div_u64(uint64_t n, uint32_t d)
{
    uint64_t rem;
    uint32_t q = floor_div_u64(n, d, &rem);
    return q + (rem != 0);
}

struct Cand {
    int32_t lt, cost;
};

// r_given <= 0: derive the replica count (joint); otherwise use it (vertical).
__device__ __forceinline__ Cand eval_candidate(uint32_t a, uint32_t k, uint32_t q,
                                               uint32_t p, uint32_t o, uint32_t lambda,
                                               uint32_t slo_us, uint32_t T, uint32_t tick,
                                               uint32_t c, uint32_t b, uint32_t r_max,
                                               int32_t r_given)
{
    const Cand none{-1, -1};
    // Anything whose latency exceeds slo_us also exceeds T ticks, so the tests
    // against slo_us below only cut candidates that lt > T would cut anyway;
    // they keep every later quotient inside 32 bits.
    if (o > slo_us) return none;
    uint64_t num = (uint64_t)a + (uint64_t)k * b + (uint64_t)q * b * b;
    uint32_t d = c < p ? c : p;
    if (num > (uint64_t)(slo_us - o) * d) return none;      // proc > slo_us
    uint32_t proc = ceil_div_u64(num, d) + o;                // <= slo_us
    uint64_t lp = (uint64_t)lambda * proc;                   // < 2^51
    uint32_t M = b * 1000000u;                               // < 2^30
    uint32_t n;
    if (r_given <= 0) {
        if (lp > (uint64_t)r_max * M) return none;           // needs > r_max replicas
        n = ceil_div_u64(lp, M);
        if (n < 1) n = 1;
    } else {
        n = (uint32_t)r_given;
        if (lp > (uint64_t)n * M) return none;               // throughput too low
    }
    uint64_t qn = (uint64_t)(b - 1) * 1000000u * n;          // < 2^45
    if (qn > (uint64_t)(slo_us - proc) * lambda) return none; // proc + queue > slo_us
    uint32_t lat = proc + ceil_div_u64(qn, lambda);          // <= slo_us < 2^31
    uint32_t lt = (lat + tick - 1) / tick;
    if (lt > T) return none;
    return Cand{(int32_t)lt, (int32_t)(n * c)};
}

__device__ __forceinline__ bool in_range(int32_t v, int32_t lo, int32_t hi)
{
    return v >= lo && v <= hi;
}

// Input check and work classification, one thread per instance:
// tmeta[i] = budget T in ticks, or -1 when any input of the instance is out of
// range; valid instances are appended to the list of their work class.  Lanes
// of a wavefront that fall into the same class share one atomic.
__global__ __launch_bounds__(256) void k1_validate(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    int32_t* __restrict__ tmeta, int32_t* __restrict__ order, int32_t* __restrict__ ctrl,
    uint32_t N, uint32_t S, int32_t r_max, uint32_t tick, int32_t slo_max, int coef_shared,
    int merge_to)
{
    uint32_t i = blockIdx.x * 256u + threadIdx.x;
    int cls = -1;
    if (i < N) {
        int32_t lam = lambda[i], slo = slo_us[i];
        const int32_t* cf = coef + (coef_shared ? 0 : (size_t)i * S * 5);
        bool ok = in_range(lam, 1, THEMIS_VALUE_MAX) && in_range(slo, 0, slo_max);
        for (uint32_t z = 0; z < S; ++z) {
            const int32_t* cz = cf + z * 5;
            ok = ok && in_range(cz[0], 0, THEMIS_VALUE_MAX) &&
                 in_range(cz[1], 0, THEMIS_VALUE_MAX) && in_range(cz[2], 0, THEMIS_VALUE_MAX) &&
                 cz[3] >= 1 && in_range(cz[4], 1, THEMIS_VALUE_MAX);
            if (r_fixed) ok = ok && in_range(r_fixed[(size_t)i * S + z], 1, r_max);
        }
        int32_t T = ok ? (int32_t)((uint32_t)slo / tick) : -1;
        tmeta[i] = T;
        if (ok) cls = effective_class(T, merge_to);
    }
    const unsigned lane = threadIdx.x & 63u;
    for (int c = 0; c < N_CLS; ++c) {
        const unsigned long long m = __ballot(cls == c);
        if (m == 0ull) continue;
        int base = 0;
        const int leader = __builtin_ctzll(m);
        if ((int)lane == leader) base = atomicAdd(&ctrl[c], __builtin_popcountll(m));
        base = __shfl(base, leader, 64);
        if (cls == c)
            order[(size_t)c * N + base + __builtin_popcountll(m & ((1ull << lane) - 1ull))] = (int32_t)i;
    }
}

// ctrl[0..N_CLS) = instances per class, ctrl[N_CLS..2 N_CLS) = queue cursors
__global__ void k1_reset_ctrl(int32_t* ctrl)
{
    if (threadIdx.x < 2 * N_CLS) ctrl[threadIdx.x] = 0;
}

// Candidate evaluation plus a counting sort of each row by bucket.
//
// A workgroup of 256 threads handles R = 256/G rows ((instance, model) pairs),
// G threads per row, G = Kp rounded up to a power of two (at most 256; longer
// rows are walked in steps of G).  Pass 1 evaluates every candidate, parks its
// (lt, cost) in LDS and counts its bucket; after a prefix sum over the
// buckets, pass 2 hands every entry a slot inside its bucket's range and
// writes it to HBM in the two forms the later stages read.  The order inside a bucket is whatever
// the LDS atomics yield; nothing downstream depends on it.
__global__ __launch_bounds__(256) void k1_candidates(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    const int32_t* __restrict__ tmeta, StepEntry* __restrict__ step_tab,
    uint32_t* __restrict__ tag_tab, uint16_t* __restrict__ bcum, BatchList bl, uint32_t rows,
    uint32_t S, uint32_t K, uint32_t Kp, uint32_t r_max, uint32_t tick, int coef_shared,
    uint32_t G, uint32_t nb, uint32_t nbs, int copies_mask, int merge_to)
{
    extern __shared__ uint32_t smem[];
    const uint32_t R = 256u / G;
    // per local row: hist[MAX_BUCKETS + 1], cursor[MAX_BUCKETS + 1], then staging[Kp]
    constexpr uint32_t HB = MAX_BUCKETS + 1;
    uint32_t* const hist_all = smem;
    uint32_t* const cur_all = smem + R * HB;
    uint32_t* const stage_all = smem + 2 * R * HB;

    const uint32_t rl = threadIdx.x / G, g = threadIdx.x - rl * G;
    const uint32_t row = blockIdx.x * R + rl;
    const bool live = row < rows;
    uint32_t* const hist = hist_all + rl * HB;
    uint32_t* const cur = cur_all + rl * HB;
    uint32_t* const stage = stage_all + rl * Kp;

    for (uint32_t x = threadIdx.x; x < 2 * R * HB; x += 256u) smem[x] = 0u;
    __syncthreads();

    int32_t T = -1;
    if (live) {
        const uint32_t i = row / S, s = row - i * S;
        T = tmeta[i];
        const int32_t* cf = coef + (coef_shared ? 0 : (size_t)i * S * 5) + s * 5;
        const uint32_t a = cf[0], kc = cf[1], q = cf[2], pcap = cf[3], o = cf[4];
        const uint32_t lam = lambda[i], slo = slo_us[i];
        const int32_t rgiven = r_fixed ? r_fixed[(size_t)i * S + s] : 0;
        for (uint32_t kk = g; kk < Kp; kk += G) {
            uint32_t w0 = TAG_NONE;  // lt | cost << 16
            if (T >= 0 && kk < K) {
                const uint32_t c = kk / (uint32_t)bl.n + 1, j = kk % (uint32_t)bl.n;
                const Cand cd = eval_candidate(a, kc, q, pcap, o, lam, slo, (uint32_t)T, tick, c,
                                               bl.b[j], r_max, rgiven);
                if (cd.lt >= 0) w0 = (uint32_t)cd.lt | ((uint32_t)cd.cost << 16);
            }
            stage[kk] = w0;
            const uint32_t b = w0 == TAG_NONE ? nb : (w0 & 0xFFFFu) >> BUCKET_SHIFT;
            atomicAdd(&hist[b], 1u);
        }
    }
    __syncthreads();
    if (live) {
        // exclusive prefix over the buckets; bucket nb (infeasible) comes last
        for (uint32_t j = g; j <= nb; j += G) {
            uint32_t c = 0;
            for (uint32_t b = 0; b < j; ++b) c += hist[b];
            cur[j] = c;
            bcum[(size_t)row * nbs + j] = (uint16_t)c;
        }
    }
    __syncthreads();
    if (live) {
        // the LDS geometry the min-plus stage will use for this instance
        const int cls = T >= 0 ? effective_class(T, merge_to) : 0;
        const int copy_bytes = wide_copy_bytes(CLS_WAVES[cls == NARROW_CLS ? 0 : cls]);
        const int copies = class_copies(cls, copies_mask);
        for (uint32_t kk = g; kk < Kp; kk += G) {
            const uint32_t w0 = stage[kk];
            const bool none = w0 == TAG_NONE;
            const uint32_t lt = w0 & 0xFFFFu;
            const uint32_t b = none ? nb : lt >> BUCKET_SHIFT;
            const uint32_t slot = atomicAdd(&cur[b], 1u);
            StepEntry se;
            se.shift = none ? 0u : (cls == NARROW_CLS ? narrow_shift(lt) : wide_shift(lt, copies, copy_bytes));
            se.cost2 = none ? 0u : (w0 >> 16) * 0x10001u;
            step_tab[(size_t)row * Kp + slot] = se;
            tag_tab[(size_t)row * Kp + slot] = lt | (kk << 16);
        }
    }
}

__global__ void k_zero64(unsigned long long* p) { *p = 0ull; }

// Undo the bucket order: separate lt / cost arrays [N][S][K], index k.
__global__ __launch_bounds__(256) void k_export(const StepEntry* __restrict__ step_tab,
                                                const uint32_t* __restrict__ tag_tab,
                                                int32_t* __restrict__ lt,
                                                int32_t* __restrict__ cost, uint32_t rows,
                                                uint32_t K, uint32_t Kp)
{
    uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g >= rows * Kp) return;
    uint32_t row = g / Kp;
    uint32_t tag = tag_tab[g], k = tag >> 16;
    if (k >= K) return;  // padding entry
    const bool none = (tag & 0xFFFFu) == TAG_NONE;
    lt[(size_t)row * K + k] = none ? -1 : (int32_t)(tag & 0xFFFFu);
    cost[(size_t)row * K + k] = none ? -1 : (int32_t)(step_tab[g].cost2 & 0xFFFFu);
}

// Sum over valid instances, models and feasible candidates of (T + 1 - lt).
__global__ __launch_bounds__(256) void k_count_relax(const uint32_t* __restrict__ tag_tab,
                                                     const int32_t* __restrict__ tmeta,
                                                     unsigned long long* __restrict__ out,
                                                     uint32_t N, uint32_t SK)
{
    __shared__ unsigned long long part[256];
    unsigned long long acc = 0;
    for (uint32_t i = blockIdx.x; i < N; i += gridDim.x) {
        int32_t T = tmeta[i];
        if (T < 0) continue;
        for (uint32_t e = threadIdx.x; e < SK; e += 256) {
            uint32_t lt = tag_tab[(size_t)i * SK + e] & 0xFFFFu;
            if (lt != TAG_NONE) acc += (unsigned long long)(T + 1 - (int32_t)lt);
        }
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicAdd(out, part[0]);
}

}  // namespace

hipError_t launch_candidates(const themis_problem_t& p, const Layout& L,
                             const int32_t* d_coef, const int32_t* d_lambda,
                             const int32_t* d_slo_us, const int32_t* d_r_fixed,
                             char* ws, hipStream_t st)
{
    BatchList bl{};
    bl.n = p.n_batch;
    for (int j = 0; j < p.n_batch; ++j) bl.b[j] = p.batch_sizes[j];
    int32_t* tmeta = (int32_t*)(ws + L.tmeta_off);
    int32_t* ctrl = (int32_t*)(ws + L.ctrl_off);
    const MinplusPlan plan = make_plan(L);
    hipLaunchKernelGGL(k1_reset_ctrl, dim3(1), dim3(64), 0, st, ctrl);
    hipLaunchKernelGGL(k1_validate, dim3((L.N + 255) / 256), dim3(256), 0, st, d_coef,
                       d_lambda, d_slo_us, d_r_fixed, tmeta, (int32_t*)(ws + L.order_off), ctrl,
                       (uint32_t)L.N, (uint32_t)L.S, p.r_max, (uint32_t)p.tick_us,
                       p.slo_max_us, p.coef_shared, plan.merge_to);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    uint32_t G = 64;
    while (G < 256u && G < (uint32_t)L.Kp) G <<= 1;
    const uint32_t R = 256u / G;
    const uint32_t rows = (uint32_t)L.N * L.S;
    const size_t lds = (size_t)(2 * R * (MAX_BUCKETS + 1) + R * L.Kp) * sizeof(uint32_t);
    hipLaunchKernelGGL(k1_candidates, dim3((rows + R - 1) / R), dim3(256), lds, st, d_coef,
                       d_lambda, d_slo_us, d_r_fixed, (const int32_t*)tmeta,
                       (StepEntry*)(ws + L.step_off), (uint32_t*)(ws + L.tag_off),
                       (uint16_t*)(ws + L.bcum_off), bl, rows, (uint32_t)L.S, (uint32_t)L.K,
                       (uint32_t)L.Kp, (uint32_t)p.r_max, (uint32_t)p.tick_us, p.coef_shared, G,
                       (uint32_t)L.nb, (uint32_t)L.nbs, plan.copies_mask, plan.merge_to);
    return hipGetLastError();
}

hipError_t launch_export_candidates(const Layout& L, const char* ws, int32_t* d_lt,
                                    int32_t* d_cost, hipStream_t st)
{
    uint32_t rows = (uint32_t)L.N * L.S;
    uint32_t blocks = (rows * (uint32_t)L.Kp + 255u) / 256u;
    hipLaunchKernelGGL(k_export, dim3(blocks), dim3(256), 0, st,
                       (const StepEntry*)(ws + L.step_off), (const uint32_t*)(ws + L.tag_off), d_lt,
                       d_cost, rows, (uint32_t)L.K, (uint32_t)L.Kp);
    return hipGetLastError();
}

hipError_t launch_count_relaxations(const Layout& L, const char* ws,
                                    unsigned long long* d_count, hipStream_t st)
{
    hipLaunchKernelGGL(k_zero64, dim3(1), dim3(1), 0, st, d_count);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    uint32_t blocks = (uint32_t)(L.N < 4096 ? L.N : 4096);
    hipLaunchKernelGGL(k_count_relax, dim3(blocks), dim3(256), 0, st,
                       (const uint32_t*)(ws + L.tag_off), (const int32_t*)(ws + L.tmeta_off),
                       d_count, (uint32_t)L.N, (uint32_t)(L.S * L.Kp));
    return hipGetLastError();
}

}  // namespace themis

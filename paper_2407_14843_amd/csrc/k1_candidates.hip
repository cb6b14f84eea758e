// Stage 1: candidate tables.
//
// Algorithms 1 and 2 (Section 4.4) recompute a candidate's latency l, queueing
// delay q and throughput h inside the budget loop although none of them depends
// on the budget.  This kernel evaluates each (model, cores, batch) candidate of
// each instance exactly once and writes it to HBM as an 8-byte entry (its cost,
// its index, and its latency in grid ticks in the form of the LDS offset the
// min-plus stage will read at), each row ordered by latency bucket so that the
// min-plus stage can work on prefixes of a row.
//
// Integer model (microseconds, all roundings upward), after Eq. 1, Eq. 4 and
// the throughput constraint of Eq. 6:
//   proc  = ceil((a + k b + q b^2) / min(c,p)) + o
//   n     = ceil(lambda proc / (b 1e6))   joint,  or the given replicas
//   queue = ceil((b-1) 1e6 n / lambda)
//   lt    = ceil((proc + queue) / tick),  cost = n c
// Options: the queue of Eq. 4 as printed, ceil((b-1) 1e6 / lambda), or of
// Eq. 3, the larger of that and proc - floor((n b + 1) 1e6 / lambda); and a
// sixth coefficient d for Eq. 1's term delta*b: proc += d b.
// A candidate is dropped when n exceeds r_max, when the given replicas cannot
// carry lambda, or when lt exceeds the instance's budget T.
#include "candidate_eval.h"
#include "themis_internal.h"

namespace themis {
namespace {


// Orders the LDS traffic of one wavefront: what its lanes wrote before is
// visible to all its lanes after (a wavefront's LDS operations complete in
// order; this only keeps the compiler from moving them across).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ int in_range(int32_t v, int32_t lo, int32_t hi)
{
    return (int)(v >= lo) & (int)(v <= hi);
}

// Input check and work classification, one thread per instance:
// tmeta[i] = budget T in ticks, or -1 when any input of the instance is out of
// range; valid instances are appended to the list of their work class.  The
// lanes of a wavefront that fall into the same class share one LDS atomic, and
// a workgroup reserves its stretch of every class list with one global atomic
// per class: returning atomics on one address cost tens of nanoseconds each.
constexpr uint32_t VALIDATE_THREADS = 1024;

__global__ __launch_bounds__(VALIDATE_THREADS) void k1_validate(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    const int32_t* __restrict__ c_fixed, int32_t* __restrict__ tmeta, int32_t* __restrict__ ans,
    int32_t* __restrict__ order, int32_t* __restrict__ ctrl, uint32_t N, uint32_t S,
    int32_t r_max, int32_t c_max, uint32_t tick, int32_t slo_max, int coef_shared, uint32_t cs)
{
    __shared__ int32_t in_block[N_CLS];   // instances of the class in this workgroup
    __shared__ int32_t list_base[N_CLS];  // where the workgroup's stretch of the list starts
    if (threadIdx.x < N_CLS) in_block[threadIdx.x] = 0;
    __syncthreads();

    uint32_t i = blockIdx.x * VALIDATE_THREADS + threadIdx.x;
    int cls = -1;
    if (i < N) {
        int32_t lam = lambda[i], slo = slo_us[i];
        const int32_t* cf = coef + (coef_shared ? 0 : (size_t)i * S * cs);  // cs words per model
        // no short-circuiting: the loads of all models are independent
        int ok = in_range(lam, 1, THEMIS_VALUE_MAX) & in_range(slo, 0, slo_max);
        for (uint32_t z = 0; z < S; ++z) {
            const int32_t* cz = cf + z * cs;
            const int32_t a = cz[0], k = cz[1], q = cz[2], pc = cz[3], o = cz[4];
            if (cs == 6) ok &= in_range(cz[5], 0, THEMIS_VALUE_MAX);
            ok &= in_range(a, 0, THEMIS_VALUE_MAX) & in_range(k, 0, THEMIS_VALUE_MAX) &
                  in_range(q, 0, THEMIS_VALUE_MAX) & (int)(pc >= 1) & in_range(o, 1, THEMIS_VALUE_MAX);
            if (r_fixed) ok &= in_range(r_fixed[(size_t)i * S + z], 1, r_max);
            if (c_fixed) ok &= in_range(c_fixed[(size_t)i * S + z], 1, c_max);
        }
        int32_t T = ok ? (int32_t)((uint32_t)slo / tick) : -1;
        tmeta[i] = T;
        ans[2 * i] = 0;
        ans[2 * i + 1] = -1;  // until stage 2 says otherwise, stage 3 reads row 0
        // listed under its own class even when a launch of a higher class will
        // serve it: that launch walks the lists from the longest rows down
        if (ok) cls = class_of_budget(T);
    }
    // place inside the workgroup's stretch: wavefront offset + rank among the lanes
    const unsigned lane = threadIdx.x & 63u;
    int within = 0;
    for (int c = 0; c < N_CLS; ++c) {
        const unsigned long long m = __ballot(cls == c);
        if (m == 0ull) continue;
        int base = 0;
        const int leader = __builtin_ctzll(m);
        if ((int)lane == leader) base = atomicAdd(&in_block[c], __builtin_popcountll(m));
        base = __shfl(base, leader, 64);
        if (cls == c) within = base + __builtin_popcountll(m & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    if (threadIdx.x < N_CLS) {
        const int32_t n = in_block[threadIdx.x];
        list_base[threadIdx.x] = n ? atomicAdd(&ctrl[threadIdx.x], n) : 0;
    }
    __syncthreads();
    if (cls >= 0) order[(size_t)cls * N + list_base[cls] + within] = (int32_t)i;
}

// ctrl[0..N_CLS) = instances per class, ctrl[N_CLS..2 N_CLS) = queue cursors
__global__ void k1_reset_ctrl(int32_t* ctrl)
{
    if (threadIdx.x < 2 * N_CLS) ctrl[threadIdx.x] = 0;
}

// Candidate evaluation plus a counting sort of each row by bucket.
//
// One thread per (row, batch size), or `split` threads taking alternate cores; a
// workgroup of 256 threads covers RPW = 256 / (n_batch * split) rows ((instance,
// model) pairs).  The thread walks its cores c <= c_max: the latency model only
// depends on min(c, p), so it is evaluated for c <= p and reused (with cost n*c)
// beyond.  Pass 1 parks every
// candidate's (lt, cost) in LDS and counts the bucket of the feasible ones; a
// wavefront scan turns the counts into bucket offsets; pass 2 hands every
// feasible entry a slot inside its bucket's range and writes it to HBM in the
// form the min-plus stage reads.  Infeasible candidates are not written at all:
// a row's entries are its first bcum[row][nb] slots and the rest of the row's
// stretch of the table is never read.
// The order inside a bucket is whatever the LDS atomics yield; nothing
// downstream depends on it.
//
// PRUNE: between the passes, candidates that cannot be part of the answer are
// turned into infeasible ones, so that the min-plus stage never sees them.  A
// candidate is dropped when another one of the same row is at least as fast and
// cheaper, or as cheap and faster, or equal in both with a smaller index: swapping
// it for that other one in any assignment gives a smaller (cost, ticks, indices)
// key, so it is in no instance's answer, and since the rows of the recurrence
// never increase with the budget it attains no minimum that its replacement does
// not attain as well.  Per row one wavefront fills a table min over candidates of
// (lt, index) by cost (costs binned by 2^prune_sh when r_max * c_max exceeds the
// table; then only strictly cheaper bins are compared, which drops fewer
// candidates but never a needed one), takes its running minimum, and looks every
// candidate up in it.
//
// c_fixed (may be null; then c_all, 0 = free): cores given per row; the model is
// evaluated for those cores only and every other candidate of the row is marked infeasible.
// sparse: rows of instances that failed the input check are left untouched.
constexpr uint32_t STAGE_NONE = 0xFFFFu;  // lt field of an infeasible candidate in LDS

constexpr uint32_t PRUNE_TAB_WORDS = 2560;  // per wavefront, at most: sentinel + cost bins
constexpr uint32_t PRUNE_KEY_SHIFT = 13;    // key = lt << 13 | index (index < 8192)

template <int QUEUE, bool PRUNE>
__global__ __launch_bounds__(256) void k1_candidates(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    const int32_t* __restrict__ c_fixed, const int32_t* __restrict__ tmeta,
    StepEntry* __restrict__ step_tab, uint16_t* __restrict__ bcum, BatchList bl, uint32_t rows,
    uint32_t S, uint32_t K, uint32_t Kp, uint32_t c_max, uint32_t r_max, uint32_t tick,
    double rtick, int coef_shared, uint32_t RPW, uint32_t nb, uint32_t nbs,
    uint64_t class_map, int sparse, uint32_t c_all, uint32_t cs, uint32_t prune_sh,
    uint32_t prune_bins, uint32_t split)
{
    extern __shared__ uint32_t smem[];
    // per local row: hist[nb + 1], cursor[nb + 1], staging[Kp]
    const uint32_t HB = nb + 1;
    const uint32_t row_words = 2 * HB + Kp;
    const uint32_t nbat = (uint32_t)bl.n;

    // `split` threads share the cores of one (row, batch size): thread `part` takes
    // c = part + 1, part + 1 + split, ...
    const uint32_t tpr = nbat * split;
    const uint32_t rl = threadIdx.x / tpr, rem = threadIdx.x - rl * tpr;
    const uint32_t part = rem / nbat, j = rem - part * nbat;
    const uint32_t row = blockIdx.x * RPW + rl;
    bool live = rl < RPW && row < rows;
    uint32_t* const hist = smem + rl * row_words;
    uint32_t* const cur = hist + HB;
    uint32_t* const stage = cur + HB;

    const int32_t T = live ? tmeta[row / S] : -1;
    if (sparse) {
        if (!__syncthreads_or(T >= 0)) return;  // nothing to do for any row of this workgroup
        live = live && T >= 0;
    }

    for (uint32_t x = threadIdx.x; x < RPW * row_words; x += 256u)
        if (x % row_words < 2 * HB) smem[x] = 0u;
    __syncthreads();

    if (live) {
        const uint32_t i = row / S, s = row - i * S;
        if (T >= 0) {
            const int32_t* cf = coef + (coef_shared ? 0 : (size_t)i * S * cs) + s * cs;
            const RowHdr h = make_row_hdr(cf, cs, lambda[i], slo_us[i], T, tick,
                                          r_fixed ? r_fixed[(size_t)i * S + s] : 0);
            const BatchHdr bh = make_batch_hdr(bl.b[j]);
            const uint32_t pcap = (uint32_t)cf[3];
            const uint32_t only = c_fixed ? (uint32_t)c_fixed[row] : c_all;
            Eval ev{-1, 0};
            if (only) {
                const uint32_t d = only < pcap ? only : pcap;
                ev = eval_candidate<QUEUE>(h, bh, (double)d, (double)r_max, (double)tick, rtick);
            }
            bool capped = false;  // ev already is the evaluation at the core cap
            for (uint32_t c = part + 1; c <= c_max; c += split) {
                if (!only && !capped) {
                    const uint32_t d = c < pcap ? c : pcap;
                    ev = eval_candidate<QUEUE>(h, bh, (double)d, (double)r_max, (double)tick, rtick);
                    capped = c >= pcap;
                }
                const bool none = ev.lt < 0 || (only && c != only);
                const uint32_t w0 = none ? STAGE_NONE
                                         : (uint32_t)ev.lt | (((uint32_t)ev.n * c) << 16);
                stage[(c - 1) * nbat + j] = w0;
                if (!PRUNE && !none) atomicAdd(&hist[(uint32_t)ev.lt >> BUCKET_SHIFT], 1u);
            }
        } else {
            for (uint32_t c = part + 1; c <= c_max; c += split) stage[(c - 1) * nbat + j] = STAGE_NONE;
        }
    }
    __syncthreads();
    {
        // exclusive prefix over the buckets, one row at a time per wavefront;
        // the offset of bucket nb is the number of feasible entries
        const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
        for (uint32_t r = wv; r < RPW; r += 4) {
            const uint32_t grow = blockIdx.x * RPW + r;
            if (grow >= rows) break;
            if (sparse && tmeta[grow / S] < 0) continue;
            uint32_t* const hh = smem + r * row_words;
            if (PRUNE && tmeta[grow / S] >= 0) {
                // tab[0] = "nothing cheaper"; tab[1 + bin] = least (lt, index) of the bin,
                // then of all bins up to it
                uint32_t* const tab = smem + RPW * row_words + wv * ((prune_bins + 4u) & ~3u);
                const uint32_t* const stg = hh + 2 * HB;
                // The fastest candidate (least lt, then least cost) beats everything
                // that costs more than it does, so only the bins up to its own take
                // part in the table: usually a small part of the cost range.
                uint32_t fastest = 0xFFFFFFFFu;  // lt << 16 | cost
                for (uint32_t kk = lane; kk < K; kk += 64u) {
                    const uint32_t w0 = stg[kk];
                    const uint32_t key = (w0 << 16) | (w0 >> 16);
                    fastest = key < fastest ? key : fastest;
                }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const uint32_t o = __shfl_xor(fastest, d, 64);
                    fastest = o < fastest ? o : fastest;
                }
                // no feasible candidate: lt field 0xFFFF, the bins below stay empty
                const uint32_t top_bin = (fastest & 0xFFFFu) >> prune_sh;
                const uint32_t bins = (fastest >> 16) == STAGE_NONE ? 1u
                                      : (top_bin + 1u < prune_bins ? top_bin + 1u : prune_bins);
                for (uint32_t x = lane; x <= bins; x += 64u) tab[x] = 0xFFFFFFFFu;
                wave_lds_fence();
                for (uint32_t kk = lane; kk < K; kk += 64u) {
                    const uint32_t w0 = stg[kk], lt = w0 & 0xFFFFu;
                    const uint32_t bin = (w0 >> 16) >> prune_sh;
                    if (lt != STAGE_NONE && bin < bins)
                        atomicMin(&tab[1u + bin], (lt << PRUNE_KEY_SHIFT) | kk);
                }
                wave_lds_fence();
                {
                    // running minimum over the bins: each lane owns a stretch
                    const uint32_t per = (bins + 63u) / 64u;
                    const uint32_t lo = 1u + lane * per;
                    const uint32_t hi = lo + per < bins + 1u ? lo + per : bins + 1u;
                    uint32_t m = 0xFFFFFFFFu;
                    for (uint32_t x = lo; x < hi; ++x) m = tab[x] < m ? tab[x] : m;
                    uint32_t before = m;  // becomes the minimum of all earlier stretches
#pragma unroll
                    for (int d = 1; d < 64; d <<= 1) {
                        const uint32_t t = __shfl_up(before, d, 64);
                        if ((int)lane >= d) before = t < before ? t : before;
                    }
                    before = __shfl_up(before, 1, 64);
                    if (lane == 0) before = 0xFFFFFFFFu;
                    for (uint32_t x = lo; x < hi; ++x) {
                        const uint32_t v0 = tab[x];
                        before = v0 < before ? v0 : before;
                        tab[x] = before;
                    }
                }
                wave_lds_fence();
                for (uint32_t kk = lane; kk < K; kk += 64u) {
                    const uint32_t w0 = stg[kk], lt = w0 & 0xFFFFu;
                    const uint32_t bin = (w0 >> 16) >> prune_sh;
                    bool keep = lt != STAGE_NONE && bin < bins;
                    if (keep) {
                        // nothing strictly cheaper is as fast ...
                        keep = (tab[bin] >> PRUNE_KEY_SHIFT) > lt;
                        // ... and, where a bin is one cost, nothing as cheap is faster or
                        // equally fast with a smaller index
                        if (prune_sh == 0) keep = keep && tab[1u + bin] == ((lt << PRUNE_KEY_SHIFT) | kk);
                    }
                    if (!keep) hh[2 * HB + kk] = STAGE_NONE;
                    if (keep) atomicAdd(&hh[lt >> BUCKET_SHIFT], 1u);
                }
                wave_lds_fence();
            }
            const uint32_t v = lane < nb ? hh[lane] : 0u;
            uint32_t incl = v;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t t = __shfl_up(incl, d, 64);
                if ((int)lane >= d) incl += t;
            }
            const uint32_t excl = incl - v;
            if (lane <= nb) {
                hh[HB + lane] = excl;
                bcum[(size_t)grow * nbs + lane] = (uint16_t)excl;
            }
            if (lane == 63 && nb == 64) {
                hh[HB + 64] = incl;
                bcum[(size_t)grow * nbs + 64] = (uint16_t)incl;
            }
        }
    }
    __syncthreads();
    if (live) {
        // the LDS geometry the min-plus stage will use for this instance
        const int cls = T >= 0 ? effective_class(T, class_map) : 0;
        // wide_shift() / narrow_shift() in one branch-free form:
        //   shift = base + ((-lt) & cm) * step - (((lt + add) >> sh) << (sh + 1))
        uint32_t cm, sh, add, step, base;
        if (cls == NARROW_CLS) {
            cm = 1, sh = 1, add = 0, step = 4u * (NAR_COPY_DW - 1), base = 4u * NAR_CHUNK_DW;
        } else {
            cm = 1, sh = 1, add = 1, step = (uint32_t)wide_copy_bytes(cls_waves(cls)), base = 0;
        }
        StepEntry* const out = step_tab + (size_t)row * Kp;
        // Only the feasible candidates are written: they fill the first
        // bcum[row][nb] slots of the row, and nothing reads the table beyond them.
        for (uint32_t c = part + 1; c <= c_max; c += split) {
            const uint32_t kk = (c - 1) * nbat + j;
            const uint32_t w0 = stage[kk];
            const uint32_t lt = w0 & 0xFFFFu;
            if (lt == STAGE_NONE) continue;
            const uint32_t slot = atomicAdd(&cur[lt >> BUCKET_SHIFT], 1u);
            StepEntry se;
            se.shift = base + __umul24((0u - lt) & cm, step) - (((lt + add) >> sh) << (sh + 1));
            se.ck = (w0 >> 16) | (kk << 16);
            out[slot] = se;
        }
    }
}

__global__ void k_zero64x3(unsigned long long* p) { p[0] = p[1] = p[2] = 0ull; }

// Undo the bucket order: separate lt / cost arrays [N][S][K], index k.
__global__ __launch_bounds__(256) void k_export(const StepEntry* __restrict__ step_tab,
                                                const uint16_t* __restrict__ bcum,
                                                const int32_t* __restrict__ tmeta,
                                                int32_t* __restrict__ lt,
                                                int32_t* __restrict__ cost, uint32_t rows,
                                                uint32_t S, uint32_t K, uint32_t Kp, uint32_t nb,
                                                uint32_t nbs, uint64_t class_map)
{
    uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g >= rows * Kp) return;
    const uint32_t row = g / Kp, e = g - row * Kp;
    const int32_t T = tmeta[row / S];
    // the table holds the feasible candidates only; the arrays were filled with -1
    if (T < 0 || e >= bcum[(size_t)row * nbs + nb]) return;
    const StepEntry se = step_tab[g];
    const uint32_t k = se.ck >> 16;
    lt[(size_t)row * K + k] = (int32_t)lt_of_entry(se.shift, T, class_map);
    cost[(size_t)row * K + k] = (int32_t)(se.ck & 0xFFFFu);
}

__global__ __launch_bounds__(256) void k_fill_minus_one(int32_t* __restrict__ a,
                                                        int32_t* __restrict__ b, size_t n)
{
    const size_t g = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (g < n) {
        a[g] = -1;
        b[g] = -1;
    }
}

// Sum over valid instances, models and feasible candidates of (T + 1 - lt): the
// relaxations stage 2 executes.  Where the wide kernel serves the instance and
// nothing is pruned, the model it handles first (s = S-1) and, in a pipeline of two or more, the one it
// handles last (s = 0) are left out when they have entries enough for their
// shortcuts (see worth_shortcut): the first row is then built by a scatter and
// a scan, and of the last only the answer is computed.  out[1] takes the number
// of entries the table holds for those instances (the feasible candidates),
// out[2] the cells (model, budget) whose value stage 2 forms: T + 1 per model,
// less the model handled last where only the answer is computed.
__global__ __launch_bounds__(256) void k_count_relax(const StepEntry* __restrict__ step_tab,
                                                     const uint16_t* __restrict__ bcum,
                                                     const int32_t* __restrict__ tmeta,
                                                     unsigned long long* __restrict__ out,
                                                     uint32_t N, uint32_t S, uint32_t Kp,
                                                     uint32_t nb, uint32_t nbs,
                                                     uint64_t class_map, int pruned, int steps)
{
    __shared__ unsigned long long part[256];
    unsigned long long acc = 0, entries = 0, formed = 0;
    for (uint32_t i = blockIdx.x; i < N; i += gridDim.x) {
        const int32_t T = tmeta[i];
        if (T < 0) continue;
        const int cls = effective_class(T, class_map);
        const bool wide = cls != NARROW_CLS && !pruned;  // the kernels that have the shortcuts
        const int npos = (T + BUCKET_CELLS) / BUCKET_CELLS;
        for (uint32_t s = 0; s < S; ++s) {
            const size_t row = (size_t)i * S + s;
            const uint32_t n = bcum[row * nbs + nb];
            entries += n;
            // the wide kernel's shortcuts for the model it handles first and for the
            // one it handles last take no relaxations, and of the last one's row only
            // the answer is formed (the step-row form never forms that row)
            const bool shortcut = wide && (s == S - 1 || (s == 0 && S > 1)) &&
                                  worth_shortcut((int)n, npos, cls_waves(cls));
            const bool answer_only = s == 0 && ((shortcut && S > 1) || (steps && cls != NARROW_CLS));
            if (!answer_only) formed += (unsigned long long)(T + 1);
            if (shortcut) continue;
            for (uint32_t e = threadIdx.x; e < n; e += 256)
                acc += (unsigned long long)(T + 1) -
                       lt_of_entry(step_tab[row * Kp + e].shift, T, class_map);
        }
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        atomicAdd(out, part[0]);
        atomicAdd(out + 1, entries);  // every thread of the workgroup counted the same rows
        atomicAdd(out + 2, formed);
    }
}

}  // namespace

hipError_t launch_candidates(const themis_problem_t& p, const Layout& L,
                             const int32_t* d_coef, const int32_t* d_lambda,
                             const int32_t* d_slo_us, const int32_t* d_r_fixed,
                             char* ws, hipStream_t st, const PassOpts& opts)
{
    BatchList bl{};
    bl.n = p.n_batch;
    for (int j = 0; j < p.n_batch; ++j) bl.b[j] = p.batch_sizes[j];
    const uint32_t cs = p.profile_form == THEMIS_PROFILE_EQ1 ? 6u : 5u;
    int32_t* tmeta = (int32_t*)(ws + L.tmeta_off);
    int32_t* ctrl = (int32_t*)(ws + L.ctrl_off);
    const MinplusPlan plan = make_plan(L);
    hipLaunchKernelGGL(k1_reset_ctrl, dim3(1), dim3(64), 0, st, ctrl);
    hipLaunchKernelGGL(k1_validate, dim3((L.N + VALIDATE_THREADS - 1) / VALIDATE_THREADS),
                       dim3(VALIDATE_THREADS), 0, st, d_coef,
                       d_lambda, d_slo_us, d_r_fixed, opts.c_fixed, tmeta,
                       (int32_t*)(ws + L.ans_off),
                       (int32_t*)(ws + L.order_off), ctrl, (uint32_t)L.N, (uint32_t)L.S, p.r_max,
                       p.c_max, (uint32_t)p.tick_us, p.slo_max_us, p.coef_shared, cs);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    const bool prune = (p.prune & THEMIS_PRUNE_DOMINATED) != 0;
    // cost bins of the pruning table: one per cost when r_max * c_max fits, else
    // 2^prune_sh costs each; one table (sentinel + bins) per wavefront
    uint32_t prune_sh = 0;
    const uint32_t cost_top = (uint32_t)p.r_max * (uint32_t)p.c_max;
    while ((cost_top >> prune_sh) + 2u > PRUNE_TAB_WORDS) ++prune_sh;
    const uint32_t prune_bins = (cost_top >> prune_sh) + 1u;
    const uint32_t tab_bytes = prune ? 4u * ((prune_bins + 4u) & ~3u) * (uint32_t)sizeof(uint32_t) : 0u;

    // This kernel is bound by latency (dependent double-precision chains, LDS
    // atomics, the loads at its start), so it needs wavefronts more than it needs
    // every lane busy.  Where one thread per (row, batch size) would make a
    // workgroup hold more than 32 KB of LDS, two threads share the cores of a
    // (row, batch size): half the rows and LDS per workgroup, twice the workgroups
    // per compute unit, for one extra model evaluation per thread.
    const uint32_t row_bytes = (uint32_t)(2 * (L.nb + 1) + L.Kp) * sizeof(uint32_t);
    // The same split serves small batches, whose workgroups would not fill the chip.
    const uint32_t rpw1 = 256u / (uint32_t)p.n_batch;
    const bool few = ((uint32_t)L.N * L.S + rpw1 - 1) / rpw1 < 4u * (uint32_t)plan.cus;
    const uint32_t split =
        p.c_max >= 8 && (rpw1 * row_bytes + tab_bytes > 32u * 1024u || few) ? 2u : 1u;
    // rows per workgroup: as many as 256 threads cover, within 76 KB of LDS
    uint32_t RPW = 256u / ((uint32_t)p.n_batch * split);
    if (RPW == 0) RPW = 1;
    while (RPW > 1 && RPW * row_bytes + tab_bytes > 76u * 1024u) --RPW;
    const uint32_t rows = (uint32_t)L.N * L.S;
    const size_t lds = (size_t)RPW * row_bytes + tab_bytes;
    auto launch = [&](auto kernel) -> hipError_t {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(kernel, dim3((rows + RPW - 1) / RPW), dim3(256), lds, st, d_coef,
                           d_lambda, d_slo_us, d_r_fixed, opts.c_fixed, (const int32_t*)tmeta,
                           (StepEntry*)(ws + L.step_off), (uint16_t*)(ws + L.bcum_off), bl, rows,
                           (uint32_t)L.S, (uint32_t)L.K, (uint32_t)L.Kp, (uint32_t)p.c_max,
                           (uint32_t)p.r_max, (uint32_t)p.tick_us,
                           (1.0 / (double)p.tick_us) * (1.0 - 0x1p-45), p.coef_shared, RPW,
                           (uint32_t)L.nb, (uint32_t)L.nbs, plan.class_map,
                           opts.sparse, (uint32_t)opts.c_all, cs, prune_sh, prune_bins, split);
        return hipGetLastError();
    };
    switch (p.queue_model * 2 + (prune ? 1 : 0)) {
    case THEMIS_QUEUE_SHARED * 2: return launch(&k1_candidates<THEMIS_QUEUE_SHARED, false>);
    case THEMIS_QUEUE_SHARED * 2 + 1: return launch(&k1_candidates<THEMIS_QUEUE_SHARED, true>);
    case THEMIS_QUEUE_WORST_CASE * 2:
        return launch(&k1_candidates<THEMIS_QUEUE_WORST_CASE, false>);
    case THEMIS_QUEUE_WORST_CASE * 2 + 1:
        return launch(&k1_candidates<THEMIS_QUEUE_WORST_CASE, true>);
    case THEMIS_QUEUE_PER_REPLICA * 2 + 1:
        return launch(&k1_candidates<THEMIS_QUEUE_PER_REPLICA, true>);
    default: return launch(&k1_candidates<THEMIS_QUEUE_PER_REPLICA, false>);
    }
}

hipError_t launch_export_candidates(const Layout& L, const char* ws, int32_t* d_lt,
                                    int32_t* d_cost, hipStream_t st)
{
    const MinplusPlan plan = make_plan(L);
    uint32_t rows = (uint32_t)L.N * L.S;
    uint32_t blocks = (rows * (uint32_t)L.Kp + 255u) / 256u;
    const size_t cells = (size_t)rows * (size_t)L.K;
    hipLaunchKernelGGL(k_fill_minus_one, dim3((unsigned)((cells + 255u) / 256u)), dim3(256), 0, st,
                       d_lt, d_cost, cells);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_export, dim3(blocks), dim3(256), 0, st,
                       (const StepEntry*)(ws + L.step_off), (const uint16_t*)(ws + L.bcum_off),
                       (const int32_t*)(ws + L.tmeta_off), d_lt, d_cost, rows, (uint32_t)L.S,
                       (uint32_t)L.K, (uint32_t)L.Kp, (uint32_t)L.nb, (uint32_t)L.nbs,
                       plan.class_map);
    return hipGetLastError();
}

hipError_t launch_count_relaxations(const themis_problem_t& p, const Layout& L, const char* ws,
                                    unsigned long long* d_count, hipStream_t st)
{
    const MinplusPlan plan = make_plan(L);
    hipLaunchKernelGGL(k_zero64x3, dim3(1), dim3(1), 0, st, d_count);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    uint32_t blocks = (uint32_t)(L.N < 4096 ? L.N : 4096);
    hipLaunchKernelGGL(k_count_relax, dim3(blocks), dim3(256), 0, st,
                       (const StepEntry*)(ws + L.step_off), (const uint16_t*)(ws + L.bcum_off),
                       (const int32_t*)(ws + L.tmeta_off), d_count, (uint32_t)L.N, (uint32_t)L.S,
                       (uint32_t)L.Kp, (uint32_t)L.nb, (uint32_t)L.nbs, plan.class_map,
                       p.prune != THEMIS_PRUNE_NONE, (p.prune & THEMIS_PRUNE_STEPS) != 0);
    return hipGetLastError();
}

}  // namespace themis

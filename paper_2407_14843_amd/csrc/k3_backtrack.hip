// Stage 3: answer selection and forward reconstruction.
//
// After Algorithm 1's main loop the paper scans the budgets upward and keeps a
// strictly smaller total (least cost, then least latency), then reads the
// per-model choices back out of its tables.  Here the rows f[s][0..T] of the
// suffix recurrence are in HBM.  f[0][.] never increases with t, so the least
// cost is f[0][T] and the least latency is the first t that attains it.  From
// there the choices are rebuilt forward: at model s with t ticks left, take the
// candidate with the smallest index k (cores ascending, then batch ascending)
// among those with
//     cost[s][k] + f[s+1][t - lt[s][k]] == f[s][t],
// which yields the lexicographically smallest optimal assignment, model 0 most
// significant.  LANES lanes per instance (a wavefront, or a half or a quarter of
// one where the rows have few entries: the walk is a chain of dependent memory
// latencies, so what matters then is how many instances are in flight): they
// test LANES table entries at a time (the table is ordered by latency bucket,
// not by k) and a butterfly reduction picks the smallest k.
#include "themis_internal.h"

namespace themis {
namespace {

template <int LANES>
__global__ __launch_bounds__(256) void k3_backtrack(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum, const int32_t* __restrict__ tmeta,
    const uint16_t* __restrict__ frow, const int32_t* __restrict__ ans,
    int32_t* __restrict__ status,
    int32_t* __restrict__ cost_out, int32_t* __restrict__ ticks_out, int32_t* __restrict__ cfg,
    BatchList bl, int N, int S, int Kp, int nbs, int row_stride, uint64_t class_map,
    int sparse)
{
    static_assert(LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "a power-of-two part of a wavefront");
    const int lane = threadIdx.x & (LANES - 1);
    const int seg_shift = (int)(threadIdx.x & 63) & ~(LANES - 1);  // first lane of this instance's lanes
    const int i = (int)((blockIdx.x * 256u + threadIdx.x) / LANES);
    if (i >= N) return;

    int32_t* my_cfg = cfg + (size_t)i * S * 3;

    const int T = tmeta[i];
    const int ans_cost = ans[2 * i], ans_t = ans[2 * i + 1];  // set for every instance by stage 1
    if (sparse && T < 0) return;  // switched off in this pass: outputs stay as they are
    const uint16_t* row0 = frow + (size_t)i * S * row_stride;
    // the least cost and the least latency attaining it: from stage 2 where it
    // found them itself (it then left row 0 unwritten), else read off row 0
    const int given_t = T >= 0 ? ans_t : -1;
    uint32_t best = F_INF;
    if (T >= 0) best = given_t >= 0 ? (uint32_t)ans_cost : (uint32_t)row0[T];
    if (T < 0 || best >= F_INF) {
        for (int x = lane; x < S * 3; x += LANES) my_cfg[x] = 0;
        if (lane == 0) {
            status[i] = T < 0 ? THEMIS_INVALID : THEMIS_INFEASIBLE;
            cost_out[i] = -1;
            ticks_out[i] = -1;
        }
        return;
    }

    int t_star = given_t;
    if (given_t < 0) {
        // first t with f[0][t] == best: LANES-ary search on a non-increasing row.
        // invariant: f[0][hi] == best, and f[0][t] > best for every t < lo.
        int lo = 0, hi = T;
        while (lo < hi) {
            const int span = hi - lo;  // probes lo + span*lane/LANES all lie below hi
            const int probe = lo + (int)(((long long)span * lane) / LANES);
            const bool hit = row0[probe] == best;
            // the votes of this instance's lanes (other instances of the wavefront may
            // have left the loop; their bits are zero and are cut off anyway)
            unsigned long long m = __ballot(hit) >> seg_shift;
            if (LANES < 64) m &= (1ull << (LANES & 63)) - 1ull;
            if (m == 0ull) {
                // even the last probe is above best: the answer lies beyond it
                lo = lo + (int)(((long long)span * (LANES - 1)) / LANES) + 1;
            } else {
                const int first = __builtin_ctzll(m);
                const int new_hi = lo + (int)(((long long)span * first) / LANES);
                const int new_lo =
                    first == 0 ? lo : lo + (int)(((long long)span * (first - 1)) / LANES) + 1;
                hi = new_hi;
                lo = new_lo;
            }
        }
        t_star = lo;
    }

    int t = t_star;
    bool fail = false;
    for (int s = 0; s < S; ++s) {
        const uint32_t target = s == 0 ? best : (uint32_t)row0[(size_t)s * row_stride + t];
        const uint16_t* next = row0 + (size_t)(s + 1) * row_stride;  // only read if s+1 < S
        const size_t row = (size_t)i * S + s;
        const StepEntry* sp = step_tab + row * Kp;
        // only entries whose bucket does not exceed t's can fit
        const int n = bcum[row * nbs + (t >> BUCKET_SHIFT) + 1];
        // smallest index k among the entries that attain the target; lt and cost
        // ride along in the low bits of the key
        unsigned long long key = ~0ull;
        // Four groups of LANES entries at a time, in two rounds of independent loads
        // (the entries, then the cells of the next row they point at): the walk is
        // a chain of dependent memory latencies, so loads issued together cost one.
        constexpr int GROUPS = 4;
        for (int e0 = 0; e0 < n; e0 += LANES * GROUPS) {
            // Every load is issued whatever the lane's entry is (beyond the row's
            // entries slot 0 is read, beyond the budget left cell 0, and dropped): a
            // load under a test of its own is waited for before the next is issued.
            StepEntry se[GROUPS];
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const int e = e0 + LANES * g + lane;
                se[g] = sp[e < n ? e : 0];  // every entry below n is feasible
            }
            int lt[GROUPS];
            uint32_t rest[GROUPS];
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const int e = e0 + LANES * g + lane;
                lt[g] = e < n ? (int)lt_of_entry(se[g].shift, T, class_map) : t + 1;
                rest[g] = 0u;
                if (s + 1 < S) rest[g] = next[lt[g] <= t ? t - lt[g] : 0];
            }
#pragma unroll
            for (int g = 0; g < GROUPS; ++g)
                if (lt[g] > t) rest[g] = F_INF;
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const uint32_t co = se[g].ck & 0xFFFFu;
                if (rest[g] < F_INF && co + rest[g] == target) {
                    const unsigned long long cand =
                        ((unsigned long long)(se[g].ck >> 16) << 32) | (co << 16) | (uint32_t)lt[g];
                    key = cand < key ? cand : key;
                }
            }
        }
#pragma unroll
        for (int d = LANES / 2; d >= 1; d >>= 1) {
            const unsigned long long other = __shfl_xor(key, d, 64);
            key = other < key ? other : key;
        }
        if (key == ~0ull) {
            fail = true;
            break;
        }
        const int found_k = (int)(key >> 32);
        const int found_lt = (int)(key & 0xFFFFu);
        const int found_cost = (int)((key >> 16) & 0xFFFFu);
        if (lane == 0) {
            const int c = found_k / bl.n + 1;
            my_cfg[3 * s + 0] = c;
            my_cfg[3 * s + 1] = bl.b[found_k % bl.n];
            my_cfg[3 * s + 2] = found_cost / c;
        }
        t -= found_lt;
    }
    if (t != 0) fail = true;  // the optimum at t_star uses exactly t_star ticks

    if (lane == 0) {
        // lane 0 wrote the choices above, so it also takes them back
        if (fail)
            for (int x = 0; x < S * 3; ++x) my_cfg[x] = 0;
        status[i] = fail ? THEMIS_INTERNAL : THEMIS_SOLVED;
        cost_out[i] = fail ? -1 : (int32_t)best;
        ticks_out[i] = fail ? -1 : t_star;
    }
}

}  // namespace

hipError_t launch_backtrack(const themis_problem_t& p, const Layout& L, int32_t* d_status,
                            int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg, char* ws,
                            hipStream_t st, const PassOpts& opts)
{
    BatchList bl{};
    bl.n = p.n_batch;
    for (int j = 0; j < p.n_batch; ++j) bl.b[j] = p.batch_sizes[j];
    const MinplusPlan plan = make_plan(L);
    // Lanes per instance: a wavefront where a row can have more than 256 entries; a
    // half (two rounds of four groups at 256 entries, measured faster than one
    // round of a whole wavefront) or a quarter where it cannot; an eighth where
    // dominated candidates were dropped (a few dozen entries are left at most)
    const bool pruned = (p.prune & THEMIS_PRUNE_DOMINATED) != 0;
    const int lanes = pruned ? 8 : L.Kp <= 64 ? 16 : L.Kp <= 256 ? 32 : 64;
    auto launch = [&](auto kernel, int per_block) {
        hipLaunchKernelGGL(kernel, dim3((L.N + per_block - 1) / per_block), dim3(256), 0, st,
                           (const StepEntry*)(ws + L.step_off), (const uint16_t*)(ws + L.bcum_off),
                           (const int32_t*)(ws + L.tmeta_off), (const uint16_t*)(ws + L.frow_off),
                           (const int32_t*)(ws + L.ans_off), d_status, d_cost, d_ticks, d_cfg, bl,
                           L.N, L.S, L.Kp, L.nbs, L.row_stride, plan.class_map, opts.sparse);
        return hipGetLastError();
    };
    if (lanes == 8) return launch(&k3_backtrack<8>, 32);
    if (lanes == 16) return launch(&k3_backtrack<16>, 16);
    if (lanes == 32) return launch(&k3_backtrack<32>, 8);
    return launch(&k3_backtrack<64>, 4);
}

}  // namespace themis

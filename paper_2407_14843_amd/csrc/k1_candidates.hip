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

#include <type_traits>

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

// Inclusive prefix sums (MIN = false) or running minima (MIN = true) over segments
// of `width` consecutive lanes (a power of two; q = lane within its segment), with
// the data-parallel primitives instead of LDS permutes: shifts by 1, 2, 4, 8 inside
// each row of 16 lanes (a lane whose source lies outside its row, or its segment,
// takes the identity), then the last lane of a row of 16 broadcast to the next row
// (32-lane segments: rows 1 and 3) and lane 31 to rows 2 and 3 (64).
template <bool MIN, int CTRL, int ROWS>
__device__ __forceinline__ uint32_t scan_step(uint32_t x, bool keep)
{
    uint32_t t = (uint32_t)__builtin_amdgcn_update_dpp(MIN ? -1 : 0, (int)x, CTRL, ROWS, 0xF, false);
    if (!keep) t = MIN ? 0xFFFFFFFFu : 0u;
    return MIN ? (t < x ? t : x) : x + t;
}

template <bool MIN>
__device__ __forceinline__ uint32_t segmented_scan(uint32_t x, uint32_t q, uint32_t width)
{
    // segments shorter than a row of 16: a shift must not reach into the segment before
    const bool narrow = width < 16u;
    if (width > 1u) x = scan_step<MIN, 0x111, 0xF>(x, !narrow || q >= 1u);
    if (width > 2u) x = scan_step<MIN, 0x112, 0xF>(x, !narrow || q >= 2u);
    if (width > 4u) x = scan_step<MIN, 0x114, 0xF>(x, !narrow || q >= 4u);
    if (width > 8u) x = scan_step<MIN, 0x118, 0xF>(x, true);
    if (width > 16u) x = scan_step<MIN, 0x142 /* row_bcast:15 */, 0xA>(x, true);
    if (width > 32u) x = scan_step<MIN, 0x143 /* row_bcast:31 */, 0xC>(x, true);
    return x;
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
constexpr uint32_t VALIDATE_THREADS = 256;

// The check of instance i; returns its work class, or -1 when it is refused.
__device__ __forceinline__ int validate_instance(
    uint32_t i, const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    const int32_t* __restrict__ c_fixed, int32_t* __restrict__ tmeta, int32_t* __restrict__ ans,
    uint32_t S, int32_t r_max, int32_t c_max, uint32_t tick, int32_t slo_max, int coef_shared,
    uint32_t cs)
{
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
    return ok ? class_of_budget(T) : -1;
}

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
    if (i < N)
        cls = validate_instance(i, coef, lambda, slo_us, r_fixed, c_fixed, tmeta, ans, S, r_max,
                                c_max, tick, slo_max, coef_shared, cs);
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

// The same check for a small batch, by one workgroup that owns the class lists:
// slots come from LDS counters, and the workgroup writes the class sizes and
// zeroes the queue cursors itself, so that no launch has to clear them first.
constexpr uint32_t VALIDATE_SINGLE_THREADS = 1024;
constexpr uint32_t VALIDATE_SINGLE_MAX = VALIDATE_SINGLE_THREADS;  // beyond one pass, one compute unit is the slower way

__global__ __launch_bounds__(VALIDATE_SINGLE_THREADS) void k1_validate_single(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    const int32_t* __restrict__ c_fixed, int32_t* __restrict__ tmeta, int32_t* __restrict__ ans,
    int32_t* __restrict__ order, int32_t* __restrict__ ctrl, uint32_t N, uint32_t S,
    int32_t r_max, int32_t c_max, uint32_t tick, int32_t slo_max, int coef_shared, uint32_t cs)
{
    __shared__ int32_t listed[N_CLS];
    if (threadIdx.x < N_CLS) listed[threadIdx.x] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < N; i += VALIDATE_SINGLE_THREADS) {
        const int cls = validate_instance(i, coef, lambda, slo_us, r_fixed, c_fixed, tmeta, ans, S,
                                          r_max, c_max, tick, slo_max, coef_shared, cs);
        if (cls >= 0) order[(size_t)cls * N + atomicAdd(&listed[cls], 1)] = (int32_t)i;
    }
    __syncthreads();
    if (threadIdx.x < N_CLS) {
        ctrl[threadIdx.x] = listed[threadIdx.x];
        ctrl[N_CLS + threadIdx.x] = 0;
    }
}

// Candidate evaluation plus a counting sort of each row by bucket.
//
// A wavefront serves RW = 64 / LPR rows ((instance, model) pairs) at a time with
// LPR lanes each (LPR a power of two), and walks the table in steps of all
// resident wavefronts: the raw inputs of its next rows are loaded while it works
// on the current ones.  Within a row, lane q = part * n_batch + j works on batch
// size j; the `split` (a power of two) parts share that batch size's cores.  A
// row's lanes never leave the wavefront, so the phases below are separated by
// wavefront-level LDS fences only: after the shared table of reciprocals is set up
// there is no workgroup barrier in the kernel.
//
// The latency model depends on the cores through min(c, p) only, so a row has
// at most min(p, c_max) distinct evaluations per batch size ("singles", one per
// core count up to the cap) and a "tail" of candidates beyond the cap that share
// the cap's latency and replica count and differ in cost = n * c and index only.
//
//   A  every lane evaluates its share of the singles (strided over the parts, two
//      at a time so that their dependent chains overlap), parks (lt, cost) in LDS
//      and counts its latency bucket; the lane that evaluates the cap adds the
//      whole tail to that bucket.
//   P  (PRUNE) dominated singles are dropped, see below; the tail always is (the
//      cap's candidate has the same latency and a smaller cost), so a pruned row
//      is built from the singles alone.
//   B  one segmented scan per wavefront (data-parallel primitives, no LDS) turns
//      every row's bucket counts into bucket offsets, which serve as the slot
//      cursors of phase C.
//   C  every lane reserves slots: one returning LDS atomic per single and one per
//      batch size for the whole tail (its entries differ by a constant and are
//      dealt to the parts in turn, so a tail entry costs an add and a store), and
//      writes the 8-byte entries into the row's image in LDS, in bucket order.
//   D  the row's lanes copy the image to HBM, 16 bytes per lane, front to back:
//      every store instruction writes one contiguous stretch per row.  The
//      cursors, which now stand at the bucket ends, are the row's bcum.
// Infeasible candidates are not written at all: a row's entries are its first
// bcum[row][nb] slots and the rest of the row's stretch of the table is never
// read.  The order inside a bucket is whatever the LDS atomics yield; nothing
// downstream depends on it.
//
// PRUNE: between phases A and B, candidates that cannot be part of the answer are
// turned into infeasible ones, so that the min-plus stage never sees them.  A
// candidate is dropped when another one of the same row is at least as fast and
// cheaper, or as cheap and faster, or equal in both with a smaller index: swapping
// it for that other one in any assignment gives a smaller (cost, ticks, indices)
// key, so it is in no instance's answer, and since the rows of the recurrence
// never increase with the budget it attains no minimum that its replacement does
// not attain as well.  The lanes of a row fill a table min over candidates of
// (lt, index) by cost in the row's image (free until phase C), take its running
// minimum, and look every candidate up in it.  Where the costs up to the fastest
// candidate's exceed the table, 2^sh costs share a bin and only strictly cheaper
// bins are compared, which drops fewer candidates but never a needed one.
//
// c_fixed (may be null; then c_all, 0 = free): cores given per row; the model is
// evaluated for those cores only and no other candidate of the row competes.
// sparse: rows of instances that failed the input check are left untouched.
constexpr uint32_t STAGE_NONE = 0xFFFFu;  // lt field of an infeasible candidate in LDS

constexpr uint32_t PRUNE_KEY_SHIFT = 13;    // key = lt << 13 | index (index < 8192)

// LDS words of one row: the image of its table entries (two words each), the
// parked singles, the bucket counts / cursors, the replica count of the tail.
struct K1Row {
    uint32_t image, parked, counts, tail, words;  // offsets in words; total, a multiple of four
};
__host__ __device__ inline K1Row k1_row(uint32_t Kp, uint32_t c_max, uint32_t nbat, uint32_t nb,
                                        bool in_registers)
{
    K1Row r;
    r.image = 0;
    r.parked = 2 * Kp;  // no room where the lanes keep their singles in registers
    r.counts = r.parked + (in_registers ? 0u : (c_max * nbat + 3u) & ~3u);
    r.tail = r.counts + ((nb + 1u + 3u) & ~3u);
    // per batch size: replica count and latency at the cap, first slot of the tail
    r.words = r.tail + ((3u * nbat + 3u) & ~3u);
    // an odd number of 16-byte units, so that the rows of a wavefront start on
    // different LDS banks (a multiple of 64 words would put them all on the same ones)
    if ((r.words & 4u) == 0u) r.words += 4u;
    return r;
}

typedef uint32_t k1_u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t K1_WAVES = 4;  // wavefronts per workgroup; they share nothing but a table

// The raw inputs of one row, as loaded.  A wavefront loads those of its next rows
// before it works on the current ones, so that it never waits for them.
struct K1RowIn {
    int32_t T, lam, slo, n_given, only;
    int32_t cf[6];
};

// ME > 0: a lane has at most ME singles and keeps them in registers from phase A to
// phase C (the loops over them are unrolled), so the rows need no room for parked
// singles and more wavefronts fit a compute unit; ME = 0: they are parked in LDS
// (any number; the pruning pass needs them there).
template <int QUEUE, bool PRUNE, bool DERIVE, int ME>
__global__ __launch_bounds__(64 * K1_WAVES) __attribute__((amdgpu_waves_per_eu(4, 8))) void k1_candidates(
    const int32_t* __restrict__ coef, const int32_t* __restrict__ lambda,
    const int32_t* __restrict__ slo_us, const int32_t* __restrict__ r_fixed,
    const int32_t* __restrict__ c_fixed, const int32_t* __restrict__ tmeta,
    StepEntry* __restrict__ step_tab, uint16_t* __restrict__ bcum, BatchList bl, uint32_t rows,
    uint32_t S, uint32_t Kp, uint32_t c_max, uint32_t r_max, uint32_t tick, double rtick,
    int coef_shared, uint32_t lpr_log2, uint32_t split_log2, uint32_t nb, uint32_t nbs,
    uint64_t class_map, int sparse, uint32_t c_all, uint32_t cs, uint32_t s_magic,
    uint32_t n_groups)
{
    extern __shared__ uint32_t smem[];
    const uint32_t nbat = (uint32_t)bl.n;
    static_assert(!(PRUNE && ME > 0) && ME % 2 == 0, "pruning works on parked singles");
    const K1Row R = k1_row(Kp, c_max, nbat, nb, ME > 0);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t RW = 64u >> lpr_log2;  // rows per wavefront
    // LDS: recip_below() of the core counts 1..c_max, shared; then per wavefront its rows
    double* const rcores = reinterpret_cast<double*>(smem);
    uint32_t* const mine = smem + 2u * ((c_max + 1u) & ~1u) + wv * (RW * R.words);
    for (uint32_t c = threadIdx.x + 1u; c <= c_max; c += blockDim.x)
        rcores[c - 1u] = recip_below((double)c);
    __syncthreads();  // the only workgroup barrier: from here on the wavefronts are on their own

    const uint32_t lpr = 1u << lpr_log2, split = 1u << split_log2;
    const uint32_t rl = lane >> lpr_log2, q = lane & (lpr - 1u);
    // q = part * nbat + j; lanes beyond split * nbat only help with phases B and D
    uint32_t part = 0, j = q;
    while (j >= nbat) j -= nbat, ++part;  // at most lpr / nbat steps
    const bool worker = part < split;
    uint32_t* const image = mine + rl * R.words;
    uint32_t* const parked = image + R.parked;
    uint32_t* const counts = image + R.counts;
    uint32_t* const tail_n = image + R.tail;
    const BatchHdr bh = make_batch_hdr(bl.b[j]);

    // every load is issued whatever the row (beyond the table the last row is read
    // and dropped): a load under a test of its own would be waited for on the spot
    auto load_rows = [&](uint32_t g) {
        uint32_t row = g * RW + rl;
        row = row < rows ? row : rows - 1u;
        const uint32_t i = s_magic ? __umulhi(row, s_magic) : row / S;
        const uint32_t s = row - i * S;
        K1RowIn in;
        in.T = tmeta[i];
        in.lam = lambda[i];
        in.slo = slo_us[i];
        in.n_given = DERIVE ? 0 : r_fixed[row];
        in.only = c_fixed ? c_fixed[row] : (int32_t)c_all;
        const int32_t* cf = coef + (coef_shared ? 0 : (size_t)i * S * cs) + s * cs;
#pragma unroll
        for (int x = 0; x < 5; ++x) in.cf[x] = cf[x];
        in.cf[5] = cs == 6 ? cf[5] : 0;
        return in;
    };

    const uint32_t n_wv = blockDim.x >> 6;  // K1_WAVES, or fewer where their rows would not fit
    const uint32_t g_step = gridDim.x * n_wv;
    uint32_t g = blockIdx.x * n_wv + wv;
    if (g >= n_groups) return;
    K1RowIn next = load_rows(g);
    for (; g < n_groups; g += g_step) {
        const K1RowIn in = next;
        if (g + g_step < n_groups) next = load_rows(g + g_step);

        const uint32_t row = g * RW + rl;
        bool live = row < rows;
        const int32_t T = live ? in.T : -1;
        if (sparse) live = live && T >= 0;
        if (__ballot(live) == 0ull) continue;  // nothing to do for any row of this wavefront
        const bool valid = live && T >= 0;

        for (uint32_t x = q; x < R.words - R.counts; x += lpr) counts[x] = 0u;
        wave_lds_fence();

        // which cores compete: all of 1..c_max, or the given ones only
        const uint32_t pcap = (uint32_t)in.cf[3];
        const uint32_t only = (uint32_t)in.only;
        const uint32_t c_lo = only ? only : 1u;
        const uint32_t c_hi = only ? only : c_max;
        // singles: c_lo .. last, each evaluated at min(c, p); tail: the cores beyond
        const uint32_t reach = pcap > c_lo ? pcap : c_lo;
        const uint32_t last = c_hi < reach ? c_hi : reach;
        const uint32_t n_eval = valid ? last - c_lo + 1u : 0u;
        const uint32_t tail_len = valid ? c_hi - last : 0u;
        const uint32_t my_evals = worker ? n_eval : 0u;
        uint32_t single[ME > 0 ? ME : 2];  // this lane's singles (ME > 0), as parked
        {
            // A: this lane's singles
            const RowHdr h = make_row_hdr(in.cf, cs, in.lam, in.slo, T, tick, in.n_given);
            const bool small = !valid || row_is_small(h);
            int32_t last_lt = -1;
            uint32_t last_n = 0;
            // Two singles per turn: their chains of dependent double-precision
            // operations are independent of each other, so one fills the other's waits
            // (the second of a turn may not exist; it is then computed and dropped).
            auto evaluate = [&](auto small_tag) {
                auto one = [&](uint32_t c) {
                    const uint32_t d = c < pcap ? c : pcap;
                    return eval_candidate_rd<QUEUE, decltype(small_tag)::value,
                                             DERIVE ? N_DERIVED : N_GIVEN>(
                        h, bh, (double)d, rcores[d - 1u], (double)r_max, (double)tick, rtick);
                };
                auto word = [](const Eval& ev, uint32_t c) {
                    return ev.lt < 0 ? STAGE_NONE
                                     : (uint32_t)ev.lt | (__umul24((uint32_t)ev.n, c) << 16);
                };
                auto turn = [&](uint32_t e, uint32_t& w0, uint32_t& w1) {
                    const bool both = e + split < my_evals;
                    const uint32_t e1 = both ? e + split : e;
                    const Eval ev0 = one(c_lo + e), ev1 = one(c_lo + e1);
                    w0 = word(ev0, c_lo + e);
                    w1 = both ? word(ev1, c_lo + e1) : STAGE_NONE;
                    if (!PRUNE && ev0.lt >= 0)
                        atomicAdd(&counts[(uint32_t)ev0.lt >> BUCKET_SHIFT], 1u);
                    if (!PRUNE && both && ev1.lt >= 0)
                        atomicAdd(&counts[(uint32_t)ev1.lt >> BUCKET_SHIFT], 1u);
                    last_lt = ev1.lt;
                    last_n = (uint32_t)ev1.n;
                };
                if constexpr (ME > 0) {
#pragma unroll
                    for (int u = 0; u < ME; u += 2) {
                        const uint32_t e = part + (uint32_t)u * split;
                        single[u] = single[u + 1] = STAGE_NONE;
                        if (e < my_evals) turn(e, single[u], single[u + 1]);
                    }
                } else {
                    for (uint32_t e = part; e < my_evals; e += 2u * split) {
                        uint32_t w0, w1;
                        turn(e, w0, w1);
                        parked[e * nbat + j] = w0;
                        if (e + split < my_evals) parked[(e + split) * nbat + j] = w1;
                    }
                }
            };
            // the short divisions where every row of the wavefront allows them
            if (__ballot(!small) == 0ull)
                evaluate(std::true_type{});
            else
                evaluate(std::false_type{});
            // the lane that evaluated the cap answers for the cores beyond it
            if (my_evals > 0u && ((n_eval - 1u) & (split - 1u)) == part) {
                tail_n[j] = last_n;
                tail_n[2u * nbat + j] = last_lt < 0 ? STAGE_NONE : (uint32_t)last_lt;
                if (!PRUNE && tail_len > 0u && last_lt >= 0)
                    atomicAdd(&counts[(uint32_t)last_lt >> BUCKET_SHIFT], tail_len);
            }
        }
        wave_lds_fence();

        if (PRUNE) {
            // P: every row's lanes prune their own row; the row's image, not yet in
            // use, is the table: tab[0] = "nothing cheaper", tab[1 + bin] = least
            // (lt, index) of the cost bin, then of all bins up to it.
            uint32_t* const tab = image;
            const uint32_t K = n_eval * nbat;  // the row's parked singles, in index order
            // The fastest candidate (least lt, then least cost) beats everything that
            // costs more than it does, so only the costs up to its own take part:
            // usually a small part of the cost range.
            uint32_t fastest = 0xFFFFFFFFu;  // lt << 16 | cost
            for (uint32_t kk = q; kk < K; kk += lpr) {
                const uint32_t w0 = parked[kk];
                const uint32_t key = (w0 << 16) | (w0 >> 16);
                fastest = key < fastest ? key : fastest;
            }
            fastest = __shfl(segmented_scan<true>(fastest, q, lpr), (int)(lane | (lpr - 1u)), 64);
            // One cost per bin where the table (the image's 2 Kp words) holds them all,
            // else 2^sh costs per bin; then only strictly cheaper bins are compared,
            // which drops fewer candidates but never a needed one.
            const uint32_t cost_top = fastest & 0xFFFFu;
            uint32_t sh = 0;
            while ((cost_top >> sh) + 2u > 2u * Kp) ++sh;
            // no feasible candidate: lt field 0xFFFF, the table stays empty
            const uint32_t bins = (fastest >> 16) == STAGE_NONE ? 1u : (cost_top >> sh) + 1u;
            for (uint32_t x = q; x <= bins; x += lpr) tab[x] = 0xFFFFFFFFu;
            wave_lds_fence();
            for (uint32_t kk = q; kk < K; kk += lpr) {
                const uint32_t w0 = parked[kk], lt = w0 & 0xFFFFu;
                const uint32_t bin = (w0 >> 16) >> sh;
                if (lt != STAGE_NONE && bin < bins)
                    atomicMin(&tab[1u + bin], (lt << PRUNE_KEY_SHIFT) | kk);
            }
            wave_lds_fence();
            {
                // running minimum over the bins: each lane owns a stretch
                const uint32_t per = (bins + lpr - 1u) >> lpr_log2;
                const uint32_t lo = 1u + q * per;
                const uint32_t hi = lo + per < bins + 1u ? lo + per : bins + 1u;
                uint32_t m = 0xFFFFFFFFu;
                for (uint32_t x = lo; x < hi; ++x) m = tab[x] < m ? tab[x] : m;
                // the minimum of all earlier stretches of the row: inclusive scan, moved
                // up a lane
                uint32_t before = segmented_scan<true>(m, q, lpr);
                before = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)before,
                                                               0x138 /* wave_shr:1 */, 0xF, 0xF, false);
                if (q == 0u) before = 0xFFFFFFFFu;
                for (uint32_t x = lo; x < hi; ++x) {
                    const uint32_t v0 = tab[x];
                    before = v0 < before ? v0 : before;
                    tab[x] = before;
                }
            }
            wave_lds_fence();
            for (uint32_t kk = q; kk < K; kk += lpr) {
                const uint32_t w0 = parked[kk], lt = w0 & 0xFFFFu;
                const uint32_t bin = (w0 >> 16) >> sh;
                bool keep = lt != STAGE_NONE && bin < bins;
                if (keep) {
                    // nothing strictly cheaper is as fast ...
                    keep = (tab[bin] >> PRUNE_KEY_SHIFT) > lt;
                    // ... and, where a bin is one cost, nothing as cheap is faster or
                    // equally fast with a smaller index
                    if (sh == 0u) keep = keep && tab[1u + bin] == ((lt << PRUNE_KEY_SHIFT) | kk);
                }
                if (!keep) parked[kk] = STAGE_NONE;
                if (keep) atomicAdd(&counts[lt >> BUCKET_SHIFT], 1u);
            }
            wave_lds_fence();
        }

        {
            // B: exclusive prefix over each row's buckets 0..nb, all rows of the wavefront
            // in one segmented scan: lane q of a row owns `per` consecutive buckets.  The
            // offset of bucket nb (which no candidate falls into) is the number of entries.
            const uint32_t per = (nb + lpr) >> lpr_log2;  // ceil((nb + 1) / lpr)
            const uint32_t lo = q * per;
            uint32_t sum = 0;
            for (uint32_t x = lo; x < lo + per && x <= nb; ++x) sum += counts[x];
            const uint32_t incl = segmented_scan<false>(sum, q, lpr);
            uint32_t run = incl - sum;
            for (uint32_t x = lo; x < lo + per && x <= nb; ++x) {
                const uint32_t v = counts[x];
                counts[x] = run;
                run += v;
            }
        }
        wave_lds_fence();

        if (!PRUNE && valid && part == 0u && tail_len > 0u) {
            // one run of slots for the cores beyond the cap of this batch size
            const uint32_t lt = tail_n[2u * nbat + j];
            tail_n[nbat + j] =
                lt != STAGE_NONE ? atomicAdd(&counts[lt >> BUCKET_SHIFT], tail_len) : 0xFFFFFFFFu;
        }
        wave_lds_fence();
        if (my_evals > 0u || (valid && worker && tail_len > 0u)) {
            // the LDS geometry the min-plus stage will use for this instance;
            // wide_shift() / narrow_shift() in one branch-free form:
            //   shift = base + (lt & 1) * step - (((lt + add) >> 1) << 2)
            const int cls = effective_class(T, class_map);
            const bool narrow = cls == NARROW_CLS;
            const uint32_t add = narrow ? 0u : 1u;
            const uint32_t step =
                narrow ? 4u * (NAR_COPY_DW - 1) : (uint32_t)wide_copy_bytes(cls_waves(cls));
            const uint32_t base = narrow ? 4u * NAR_CHUNK_DW : 0u;
            auto shift_of = [&](uint32_t lt) {
                return base + ((lt & 1u) ? step : 0u) - (((lt + add) >> 1) << 2);
            };
            StepEntry* const img = reinterpret_cast<StepEntry*>(image);
            // two singles per turn, so that their LDS round trips overlap
            auto place = [&](uint32_t e, uint32_t w0, uint32_t w1) {
                const uint32_t e1 = e + split;
                const uint32_t lt0 = w0 & 0xFFFFu, lt1 = w1 & 0xFFFFu;
                uint32_t slot0 = 0, slot1 = 0;
                if (lt0 != STAGE_NONE) slot0 = atomicAdd(&counts[lt0 >> BUCKET_SHIFT], 1u);
                if (lt1 != STAGE_NONE) slot1 = atomicAdd(&counts[lt1 >> BUCKET_SHIFT], 1u);
                if (lt0 != STAGE_NONE) {
                    StepEntry se;
                    se.shift = shift_of(lt0);
                    se.ck = (w0 >> 16) | (((c_lo + e - 1u) * nbat + j) << 16);
                    img[slot0] = se;
                }
                if (lt1 != STAGE_NONE) {
                    StepEntry se;
                    se.shift = shift_of(lt1);
                    se.ck = (w1 >> 16) | (((c_lo + e1 - 1u) * nbat + j) << 16);
                    img[slot1] = se;
                }
            };
            if constexpr (ME > 0) {
#pragma unroll
                for (int u = 0; u < ME; u += 2) {
                    const uint32_t e = part + (uint32_t)u * split;
                    if (e < my_evals) place(e, single[u], single[u + 1]);
                }
            } else {
                for (uint32_t e = part; e < my_evals; e += 2u * split)
                    place(e, parked[e * nbat + j],
                          e + split < my_evals ? parked[(e + split) * nbat + j] : STAGE_NONE);
            }
            if (!PRUNE && tail_len > 0u) {
                // The cores beyond the cap: one run of slots per batch size (reserved
                // above), the run's entries dealt to the parts in turn, so that the
                // lanes of a batch size write neighbouring slots at a time.
                const uint32_t slot0 = tail_n[nbat + j];
                if (slot0 != 0xFFFFFFFFu) {
                    const uint32_t lt = tail_n[2u * nbat + j];
                    const uint32_t n = tail_n[j];
                    const uint32_t c = c_lo + n_eval + part;  // this lane's first core
                    StepEntry se;
                    se.shift = shift_of(lt);
                    se.ck = __umul24(n, c) | (((c - 1u) * nbat + j) << 16);
                    const uint32_t per_turn = (n | (nbat << 16)) << split_log2;
                    for (uint32_t t = part; t < tail_len; t += split) {
                        img[slot0 + t] = se;
                        se.ck += per_turn;
                    }
                }
            }
        }
        wave_lds_fence();

        // The next rows' inputs have long arrived; taking them here, before any of
        // this group's stores is issued, keeps the wait for them (which counts every
        // memory operation issued before it) from waiting for stores.
        asm volatile("" ::"v"(next.T), "v"(next.lam), "v"(next.slo), "v"(next.n_given),
                     "v"(next.only), "v"(next.cf[0]), "v"(next.cf[1]), "v"(next.cf[2]),
                     "v"(next.cf[3]), "v"(next.cf[4]), "v"(next.cf[5]));
        if (live) {
            // D: every bucket's cursor now stands at the start of the next bucket, which
            // is what bcum holds: bcum[0] = 0, bcum[x + 1] = cursor[x]; two per store
            uint32_t* const bc = reinterpret_cast<uint32_t*>(bcum + (size_t)row * nbs);
            for (uint32_t y = q; 2u * y <= nb; y += lpr) {
                const uint32_t lo = y ? counts[2u * y - 1u] : 0u;
                const uint32_t hi = 2u * y < nb ? counts[2u * y] : 0u;  // the padding half, if any
                bc[y] = lo | (hi << 16);
            }
        }
        if (valid) {
            // the image goes to HBM front to back, two entries per lane and store
            // (an odd count takes one slot of padding along; the stretch has room)
            const uint32_t n_ent = counts[nb];
            const k1_u32x4* const src = reinterpret_cast<const k1_u32x4*>(image);
            k1_u32x4* const dst = reinterpret_cast<k1_u32x4*>(step_tab + (size_t)row * Kp);
            for (uint32_t x = q; 2u * x < n_ent; x += lpr) dst[x] = src[x];
        }
        wave_lds_fence();  // the next rows reuse this memory
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
    if ((uint32_t)L.N <= VALIDATE_SINGLE_MAX) {
        hipLaunchKernelGGL(k1_validate_single, dim3(1), dim3(VALIDATE_SINGLE_THREADS), 0, st,
                           d_coef, d_lambda, d_slo_us, d_r_fixed, opts.c_fixed, tmeta,
                           (int32_t*)(ws + L.ans_off), (int32_t*)(ws + L.order_off), ctrl,
                           (uint32_t)L.N, (uint32_t)L.S, p.r_max, p.c_max, (uint32_t)p.tick_us,
                           p.slo_max_us, p.coef_shared, cs);
    } else {
        hipLaunchKernelGGL(k1_reset_ctrl, dim3(1), dim3(64), 0, st, ctrl);
        hipLaunchKernelGGL(k1_validate, dim3((L.N + VALIDATE_THREADS - 1) / VALIDATE_THREADS),
                           dim3(VALIDATE_THREADS), 0, st, d_coef, d_lambda, d_slo_us, d_r_fixed,
                           opts.c_fixed, tmeta, (int32_t*)(ws + L.ans_off),
                           (int32_t*)(ws + L.order_off), ctrl, (uint32_t)L.N, (uint32_t)L.S,
                           p.r_max, p.c_max, (uint32_t)p.tick_us, p.slo_max_us, p.coef_shared, cs);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    const bool prune = (p.prune & THEMIS_PRUNE_DOMINATED) != 0;
    // Lanes per row: enough to give every batch size a lane, and beyond that enough
    // to leave a lane about sixteen candidates.  Fewer lanes per row spread the
    // per-row work (inputs, header, scan, set-up of the phases) over more
    // candidates; more lanes shorten the threads and let more wavefronts stay
    // resident, since a row's image and counters live in LDS (measured: sixteen per
    // lane is the best trade on the shapes of the numbered workloads).
    uint32_t lpr_log2 = 0;
    while ((1u << lpr_log2) < (uint32_t)p.n_batch) ++lpr_log2;
    while (lpr_log2 < 6 && ((uint32_t)p.c_max * (uint32_t)p.n_batch >> lpr_log2) > 16u) ++lpr_log2;
    // rows per wavefront must fit the LDS a workgroup may have (sized for the layout
    // that parks the singles in LDS)
    const uint32_t parked_row_bytes =
        k1_row((uint32_t)L.Kp, (uint32_t)p.c_max, (uint32_t)p.n_batch, (uint32_t)L.nb, false).words *
        (uint32_t)sizeof(uint32_t);
    while (lpr_log2 < 6 && (64u >> lpr_log2) * parked_row_bytes > 60u * 1024u) ++lpr_log2;
    uint32_t split_log2 = 0;
    while (((uint32_t)p.n_batch << (split_log2 + 1)) <= (1u << lpr_log2)) ++split_log2;
    // Where a lane then has at most sixteen singles (and nothing is pruned) they
    // stay in registers and the rows need no room for them.
    const uint32_t lane_singles = ((uint32_t)p.c_max + (1u << split_log2) - 1u) >> split_log2;
    const int me = prune || lane_singles > 16u ? 0 : lane_singles > 8u ? 16 : 8;
    const K1Row R = k1_row((uint32_t)L.Kp, (uint32_t)p.c_max, (uint32_t)p.n_batch, (uint32_t)L.nb,
                           me > 0);
    const uint32_t row_bytes = R.words * (uint32_t)sizeof(uint32_t);
    // row / S as the high half of row * ceil(2^32 / S): exact while rows * S < 2^32
    const uint64_t n_rows = (uint64_t)L.N * L.S;
    const uint32_t s_magic =
        L.S > 1 && n_rows * (uint64_t)L.S < (1ull << 32) ? (uint32_t)(((1ull << 32) + L.S - 1) / L.S) : 0u;
    // LDS of a workgroup: a reciprocal per core count, then per wavefront its rows
    const uint32_t rc_bytes = 8u * (((uint32_t)p.c_max + 1u) & ~1u);
    uint32_t waves = K1_WAVES;  // fewer when four wavefronts' rows do not fit
    auto lds_for = [&](uint32_t w) {
        return (size_t)rc_bytes + (size_t)w * ((64u >> lpr_log2) * row_bytes);
    };
    while (waves > 1 && lds_for(waves) > 150u * 1024u) --waves;
    if (lds_for(waves) > 150u * 1024u) return hipErrorInvalidValue;
    const uint32_t RW = 64u >> lpr_log2;
    const uint32_t rows = (uint32_t)L.N * L.S;
    const uint32_t n_groups = (rows + RW - 1) / RW;
    const size_t lds = lds_for(waves);
    // persistent workgroups: as many as stay resident, each wavefront walking the
    // row groups with a stride
    uint32_t per_cu = (uint32_t)(160u * 1024u / lds);
    if (per_cu > 32u / waves) per_cu = 32u / waves;
    if (per_cu < 1u) per_cu = 1u;
    uint32_t grid = (uint32_t)plan.cus * per_cu;
    if (grid > (n_groups + waves - 1) / waves) grid = (n_groups + waves - 1) / waves;
    auto launch = [&](auto kernel) -> hipError_t {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * waves), lds, st, d_coef,
                           d_lambda, d_slo_us, d_r_fixed, opts.c_fixed, (const int32_t*)tmeta,
                           (StepEntry*)(ws + L.step_off), (uint16_t*)(ws + L.bcum_off), bl, rows,
                           (uint32_t)L.S, (uint32_t)L.Kp, (uint32_t)p.c_max,
                           (uint32_t)p.r_max, (uint32_t)p.tick_us,
                           (1.0 / (double)p.tick_us) * (1.0 - 0x1p-45), p.coef_shared, lpr_log2,
                           split_log2, (uint32_t)L.nb, (uint32_t)L.nbs, plan.class_map,
                           opts.sparse, (uint32_t)opts.c_all, cs, s_magic, n_groups);
        return hipGetLastError();
    };
    const bool derive = d_r_fixed == nullptr;
    auto by_singles = [&](auto q_tag, auto d_tag) -> hipError_t {
        constexpr int Q = decltype(q_tag)::value;
        constexpr bool D = decltype(d_tag)::value;
        if (prune) return launch(&k1_candidates<Q, true, D, 0>);
        if (me == 8) return launch(&k1_candidates<Q, false, D, 8>);
        if (me == 16) return launch(&k1_candidates<Q, false, D, 16>);
        return launch(&k1_candidates<Q, false, D, 0>);
    };
    auto by_replicas = [&](auto q_tag) -> hipError_t {
        return derive ? by_singles(q_tag, std::true_type{}) : by_singles(q_tag, std::false_type{});
    };
    switch (p.queue_model) {
    case THEMIS_QUEUE_PER_REPLICA:
        return by_replicas(std::integral_constant<int, THEMIS_QUEUE_PER_REPLICA>{});
    case THEMIS_QUEUE_SHARED:
        return by_replicas(std::integral_constant<int, THEMIS_QUEUE_SHARED>{});
    case THEMIS_QUEUE_WORST_CASE:
        return by_replicas(std::integral_constant<int, THEMIS_QUEUE_WORST_CASE>{});
    default: return hipErrorInvalidValue;
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

// Stage 2 with the rows kept as step functions (option THEMIS_PRUNE_STEPS).
//
// Every row f[s][.] of the recurrence of Section 4.4 never increases with the
// budget, so it is a staircase: a short list of breakpoints (tau_j, v_j),
// f[s][t] = v_j for tau_j <= t < tau_{j+1}, F_INF below tau_0.  The row before
// the first model is the single breakpoint (0, 0).  For a model with
// candidates (lt_k, cost_k),
//
//     f[s][t] = min over k, j with lt_k + tau_j <= t of cost_k + v_j,
//
// that is: every pair (k, j) offers the value cost_k + v_j from budget
// lt_k + tau_j on, and the new row is the running minimum of the offers.  The
// pairs scatter their value into one dword per budget (an LDS atomic min), a
// min-scan over the budgets makes the row, and the cells where it drops are the
// next list.  The work per model is candidates x breakpoints (+ one pass over
// the budgets) instead of candidates x budgets, and the rows are bit for bit
// those of the sweeping kernel.  Of the last row only the answer is formed: the
// least cost over the pairs that fit T and, among those, the least budget, both
// as one packed minimum.
//
// One workgroup per instance, sized like the sweeping kernel's (64 threads per
// 1024 cells of its class group's longest rows).  Rows go to HBM as 16-bit
// cells for stage 3, as in the other forms.  A list that outgrows its LDS area
// is not written: for the following model every thread then scatters the
// breakpoints of its own stretch of the row, which it still holds in registers
// (slow when they bunch, but never wrong).
#include "instance_queue.h"
#include "themis_internal.h"

namespace themis {
namespace {

constexpr int STEP_LIST = 1024;  // breakpoints of a row kept as a list
constexpr int STEP_ENTS = 512;   // candidates of a model staged at a time
constexpr int STEP_RUN = 16;     // most cells a thread scans (1024 cells per wavefront)
constexpr int STEP_HDR = 64;     // dwords: queue slot, list length, answer, per-wavefront partials

// header dwords
enum { H_SLOT = 0, H_LEN = 1, H_KEY = 2, H_MIN = 8, H_CNT = 24 };

// Where the dword of budget c lives: one dword of padding per 32 budgets, so
// that the scans, in which lane l reads budget l * cells_per_thread + j, spread
// over the LDS banks instead of piling onto two of them.
__device__ __forceinline__ int cell_at(int c) { return c + (c >> 5); }
constexpr int STEP_CELLS_PER_WAVE = WIDE_CHUNK + WIDE_CHUNK / 32;  // dwords, padding included

__device__ __forceinline__ uint32_t wave_incl_min(uint32_t x, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(x, d, 64);
        if (lane >= d) x = o < x ? o : x;
    }
    return x;
}

__device__ __forceinline__ uint32_t wave_incl_sum(uint32_t x, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(x, d, 64);
        if (lane >= d) x += o;
    }
    return x;
}

__device__ __forceinline__ uint32_t wave_min(uint32_t x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(x, d, 64);
        x = o < x ? o : x;
    }
    return x;
}

__global__ __launch_bounds__(1024) void k2_steps(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum,
    const int32_t* __restrict__ tmeta, const int32_t* __restrict__ order,
    int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow, int32_t* __restrict__ ans, int N,
    int S, int Kp, int nbs, int row_stride, int cls, int low_cls)
{
    extern __shared__ uint32_t lds[];
    const int nt = (int)blockDim.x, nw = nt >> 6;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the layout stage 1 made the entries' shifts for (only their latency is used here)
    const int CSB = wide_copy_bytes(cls_waves(cls));
    uint32_t* const cell_min = lds;                      // one dword per budget, see cell_at()
    uint32_t* const hdr = lds + nw * STEP_CELLS_PER_WAVE;  // [STEP_HDR]
    uint32_t* const list = hdr + STEP_HDR;               // [STEP_LIST] tau << 16 | value
    uint32_t* const ent = list + STEP_LIST;              // [STEP_ENTS] lt << 16 | cost

    const int count = list_length(ctrl, cls, low_cls);
    int idx = -1;
    for (;;) {
        idx = next_index(reinterpret_cast<volatile uint32_t*>(hdr + H_SLOT),
                         ctrl + N_CLS + cls, count, idx);
        if (idx < 0) break;
        const int i = list_entry(ctrl, order, N, cls, low_cls, idx);
        const int T = as_constant(tmeta)[i];
        const int all = (T + BUCKET_CELLS) / BUCKET_CELLS;  // bcum index of "every feasible entry"
        // every thread scans STEP_RUN budgets; those at or beyond C hold F_INF, so
        // they never count as a drop and need no test of their own
        const int c0 = tid * STEP_RUN;

        // the row before the first model: zero from budget 0 on
        if (tid == 0) {
            list[0] = 0u;
            hdr[H_LEN] = 1u;
            hdr[H_KEY] = 0xFFFFFFFFu;
        }
        // this thread's stretch of the previous row and the value just below it;
        // only used when the list did not fit
        uint32_t f[STEP_RUN];
        uint32_t below = F_INF;
        bool own = false;  // uniform: scatter from the threads' own stretches
        lds_barrier();

        for (int s = S - 1; s >= 0; --s) {
            const size_t row = (size_t)i * S + s;
            const StepEntry* const grow = step_tab + row * Kp;
            const int n_all = as_constant(bcum + row * nbs)[all];
            const int J = (int)hdr[H_LEN];
            int jbits = 0;
            while ((1 << jbits) < J) ++jbits;

            // offers of the pairs (entry k of the staged part, breakpoint): value and
            // budget; `use` gets each pair that fits T
            auto pairs = [&](int cnt, auto use) {
                if (!own) {
                    for (int q = tid; q < (cnt << jbits); q += nt) {
                        const int j = q & ((1 << jbits) - 1);
                        if (j >= J) continue;
                        const uint32_t b = list[j], e = ent[q >> jbits];
                        const uint32_t t = (b >> 16) + (e >> 16);
                        if ((int)t <= T) use(t, (b & 0xFFFFu) + (e & 0xFFFFu));
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < STEP_RUN; ++j) {
                        const int cell = c0 + j;
                        if (f[j] < (j ? f[j - 1] : below)) {
                            for (int k = 0; k < cnt; ++k) {
                                const uint32_t e = ent[k];
                                const uint32_t t = (uint32_t)cell + (e >> 16);
                                if ((int)t <= T) use(t, f[j] + (e & 0xFFFFu));
                            }
                        }
                    }
                }
            };
            // stages entries [e0, e0 + cnt) of the row, latency decoded
            auto stage = [&](int e0, int cnt) {
                for (int x = tid; x < cnt; x += nt) {
                    const StepEntry se = grow[e0 + x];
                    ent[x] = (wide_lt_of_shift(se.shift, CSB) << 16) | (se.ck & 0xFFFFu);
                }
            };

            if (s == 0) {
                // the answer: least total, then least budget, as one packed minimum
                uint32_t key = 0xFFFFFFFFu;
                for (int e0 = 0; e0 < n_all; e0 += STEP_ENTS) {
                    const int cnt = n_all - e0 < STEP_ENTS ? n_all - e0 : STEP_ENTS;
                    if (e0) lds_barrier();  // the previous part has been used
                    stage(e0, cnt);
                    lds_barrier();
                    pairs(cnt, [&](uint32_t t, uint32_t v) {
                        const uint32_t c = (v << 16) | t;
                        key = c < key ? c : key;
                    });
                }
                key = wave_min(key);
                if (lane == 0) atomicMin(&hdr[H_KEY], key);
                lds_barrier();
                if (tid == 0) {
                    const uint32_t k = hdr[H_KEY];
                    const bool none = k == 0xFFFFFFFFu;
                    ans[2 * i] = none ? (int32_t)F_INF : (int32_t)(k >> 16);
                    ans[2 * i + 1] = none ? 0 : (int32_t)(k & 0xFFFFu);
                }
                break;
            }

            for (int x = tid; x < nw * STEP_CELLS_PER_WAVE; x += nt) cell_min[x] = F_INF;
            for (int e0 = 0; e0 < n_all; e0 += STEP_ENTS) {
                const int cnt = n_all - e0 < STEP_ENTS ? n_all - e0 : STEP_ENTS;
                if (e0) lds_barrier();
                stage(e0, cnt);
                lds_barrier();  // entries staged, cells initialised
                pairs(cnt, [&](uint32_t t, uint32_t v) { atomicMin(&cell_min[cell_at((int)t)], v); });
            }
            lds_barrier();

            // running minimum over the budgets: this thread's stretch, then the lanes,
            // then the wavefronts
            uint32_t run = F_INF;
#pragma unroll
            for (int j = 0; j < STEP_RUN; ++j) {
                const int cell = c0 + j;
                const uint32_t x = cell_min[cell_at(cell)];
                run = x < run ? x : run;
                f[j] = run;
            }
            const uint32_t incl = wave_incl_min(run, lane);
            below = __shfl_up(incl, 1, 64);
            if (lane == 0) below = F_INF;
            if (lane == 63) hdr[H_MIN + w] = incl;
            lds_barrier();
            for (int ww = 0; ww < w; ++ww) {
                const uint32_t o = hdr[H_MIN + ww];
                below = o < below ? o : below;
            }
            uint32_t drops = 0;
#pragma unroll
            for (int j = 0; j < STEP_RUN; ++j) {
                f[j] = f[j] < below ? f[j] : below;
                drops += f[j] < (j ? f[j - 1] : below) ? 1u : 0u;
            }
            // the row, for stage 3
            uint16_t* const out = frow + row * row_stride;
#pragma unroll
            for (int j = 0; j < STEP_RUN; j += 2) {
                const int cell = c0 + j;
                if (cell <= T) *reinterpret_cast<uint32_t*>(out + cell) = f[j] | (f[j + 1] << 16);
            }
            // where the list entries of this thread go
            const uint32_t isum = wave_incl_sum(drops, lane);
            if (lane == 63) hdr[H_CNT + w] = isum;
            lds_barrier();  // (also: every thread has read the list and the cells)
            uint32_t at = isum - drops, total = 0;
            for (int ww = 0; ww < nw; ++ww) {
                const uint32_t o = hdr[H_CNT + ww];
                if (ww < w) at += o;
                total += o;
            }
            own = total > (uint32_t)STEP_LIST;
            if (!own) {
#pragma unroll
                for (int j = 0; j < STEP_RUN; ++j) {
                    const int cell = c0 + j;
                    if (f[j] < (j ? f[j - 1] : below)) list[at++] = ((uint32_t)cell << 16) | f[j];
                }
            }
            if (tid == 0) hdr[H_LEN] = own ? 0u : total;
            lds_barrier();
        }
        lds_barrier();  // the answer has been read before the header is reused
    }
}

constexpr size_t LDS_PER_CU = 160 * 1024;

size_t steps_lds_bytes(int waves)
{
    return ((size_t)waves * STEP_CELLS_PER_WAVE + STEP_HDR + STEP_LIST + STEP_ENTS) *
           sizeof(uint32_t);
}

}  // namespace

// One launch for the class group whose longest rows are class `cls` (see
// make_plan); the instances of classes low .. cls are served.
hipError_t launch_steps_group(const Layout& L_, char* ws, hipStream_t st, int cls, int low,
                              int cus)
{
    const int nw = CLS_WAVES[cls];
    const size_t lds_bytes = steps_lds_bytes(nw);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k2_steps),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(LDS_PER_CU - 1024));
    if (e != hipSuccess) return e;
    int per_cu = (int)(LDS_PER_CU / lds_bytes);
    if (per_cu > 32 / nw) per_cu = 32 / nw;
    if (per_cu < 1) per_cu = 1;
    long long grid = (long long)cus * per_cu;
    if (grid > L_.N) grid = L_.N;
    hipLaunchKernelGGL(k2_steps, dim3((unsigned)grid), dim3(nw * 64), lds_bytes, st,
                       (const StepEntry*)(ws + L_.step_off), (const uint16_t*)(ws + L_.bcum_off),
                       (const int32_t*)(ws + L_.tmeta_off), (const int32_t*)(ws + L_.order_off),
                       (int32_t*)(ws + L_.ctrl_off), (uint16_t*)(ws + L_.frow_off),
                       (int32_t*)(ws + L_.ans_off), L_.N, L_.S, L_.Kp, L_.nbs, L_.row_stride, cls,
                       low);
    return hipGetLastError();
}

}  // namespace themis

// Stage 2: the min-plus recurrence over the latency-budget grid.
//
// Section 4.4 adds the pipeline's models one at a time and, for every budget,
// splits it between the current model and the rest.  With the candidate tables
// of stage 1 that is, for models s = S-1 .. 0 and budgets t = 0 .. T,
//
//     f[S][t] = 0
//     f[s][t] = min over candidates k with lt[s][k] <= t of
//               cost[s][k] + f[s+1][t - lt[s][k]]          (F_INF if none)
//
// (the suffix form: f[s][t] is the least cost of models s.. within t ticks, so
// that stage 3 can rebuild the choice forward from model 0).
//
// Mapping.  One workgroup per instance.  Lanes run over t and the candidate
// loop is wave-uniform: lt and cost live in SGPRs, and a candidate contributes
// f[s+1] shifted by lt, a unit-stride LDS read.  There is no cross-lane traffic
// and no argmin bookkeeping in the loop: only f is kept, and stage 3 recovers
// the argmin from the stored rows.
//
// f is 16 bits wide (totals are bounded by THEMIS_COST_LIMIT), so a dword holds
// two cells and one v_pk_add_u16 + one v_pk_min_u16 relax two cells.  On
// gfx950 the LDS delivers twice the bytes per clock to 64-bit reads that it
// does to 32-bit ones, but only at natural alignment (a misaligned ds_read is
// ~25x slower).  A shift by lt moves the row by an arbitrary number of 2-byte
// cells, so the previous row is kept in LDS once per residue of the shift:
//   wide kernel   4 copies, copy m shifted by m cells, ds_read_b64 (4 cells)
//   narrow kernel 2 copies, copy m shifted by m cells, ds_read_b32 (2 cells)
// and a candidate reads the copy with m = (-lt) mod 4 (resp. lt mod 2), always
// aligned.  New values stay in registers while the old row is being read.
//
// The row is cut into positions of 512 cells.  A candidate only reaches the
// positions whose last cell is >= lt, and stage 1 ordered every row of the
// candidate table by lt / 512, so the candidates that reach position p are the
// first bcum[p+1] entries of the row: the inner loops run over a prefix with no
// test per candidate.  Work per position therefore grows with p; to keep the
// wavefronts of an instance level, wavefront w takes position w from the
// bottom of the row and position npos-1-w from the top (the row folded in the
// middle).  A stretch of F_INF in front of every copy serves the reads that
// reach below t = 0, and doubles as the harmless target of the few entries
// that pad a batch of eight beyond the prefix.
//
// Scheduling.  Instances were grouped by row length in stage 1.  Every group is
// launched once, with a workgroup of exactly the wavefronts its rows need and
// just enough workgroups to fill the chip; the workgroups pull instances from
// the group's list through an atomic cursor until it is exhausted.
#include "themis_internal.h"

namespace themis {
namespace {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t pk_add(uint32_t a, uint32_t b)
{
    u16x2 r = __builtin_bit_cast(u16x2, a) + __builtin_bit_cast(u16x2, b);
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    u16x2 r = __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    return __builtin_bit_cast(uint32_t, r);
}

// Tables written by earlier kernels are read-only here.  Viewing them through
// the constant address space tells the compiler so (a workgroup barrier
// otherwise counts as a possible writer), which lets it fetch wave-uniform
// entries with scalar loads into SGPRs.
#define AS_CONST __attribute__((address_space(4)))

template <typename T>
__device__ __forceinline__ const AS_CONST T* as_constant(const T* p)
{
    return (const AS_CONST T*)(uintptr_t)p;
}

// Pull the next instance of this class, or -1 when the list is exhausted.
// Every wavefront of the workgroup gets the same answer.
__device__ __forceinline__ int next_instance(volatile uint32_t* slot, int32_t* cursor, int count,
                                             const int32_t* order)
{
    if (threadIdx.x == 0) *slot = (uint32_t)atomicAdd(cursor, 1);
    __syncthreads();
    const int idx = __builtin_amdgcn_readfirstlane((int)*slot);
    __syncthreads();  // slot may be rewritten by the next call
    if (idx >= count) return -1;
    return as_constant(order)[idx];
}

// Entries of the row that can reach a position whose last cell is `last_cell`.
__device__ __forceinline__ int prefix_count(const AS_CONST uint16_t* bc, int last_cell)
{
    return bc[(last_cell >> BUCKET_SHIFT) + 1];
}

// ------------------------------------------------------------------ wide kernel
constexpr int QP = 2;                 // quads (4 cells) per lane per position
constexpr int POSC = 64 * 4 * QP;     // cells per position
constexpr int PADB = WIDE_PAD_BYTES;  // bytes of F_INF in front of every copy
static_assert(POSC == BUCKET_CELLS, "a position is one bucket of the candidate order");
static_assert(WIDE_CHUNK == 2 * POSC, "a wavefront holds two positions");
static_assert(PADB == POSC * 2, "the pad is as long as one position");

// Sweep entries [k_begin, k_end) of a bucket-ordered row over the lane's lower
// position (DO_LO), upper position (DO_HI) or both.  k_begin and k_end are
// multiples of eight; entry k only counts for the lower position if k < n_lo
// and for the upper one if k < n_hi, otherwise its read is parked on the F_INF
// pad, where it changes nothing.
//
// The loop is software-pipelined by hand: the LDS reads of entry k+1 are
// issued before the arithmetic of entry k, into the other half of a double
// buffer, so a wavefront always has one entry's reads in flight while it
// works.  The scheduling barriers keep the compiler from undoing that order.
template <bool DO_LO, bool DO_HI>
__device__ __forceinline__ void sweep(uint32_t (&alo)[2 * QP], uint32_t (&ahi)[2 * QP],
                                      const char* ldsb, const AS_CONST u32x16* ep, int k_begin,
                                      int k_end, int n_lo, int n_hi, uint32_t byte_lo,
                                      uint32_t byte_hi, uint32_t park_lo, uint32_t park_hi)
{
    if (k_begin >= k_end) return;
    u32x2 blo[2][QP], bhi[2][QP];
    uint32_t bcost[2];

    // entry = (shift, cost2) as stage 1 prepared them
    auto issue = [&](uint32_t shift, uint32_t cost2, int k, int slot) {
        bcost[slot] = cost2;
        if (DO_LO) {
            const u32x2* src =
                reinterpret_cast<const u32x2*>(ldsb + (byte_lo + (k < n_lo ? shift : park_lo)));
#pragma unroll
            for (int q = 0; q < QP; ++q) blo[slot][q] = src[q * 64];
        }
        if (DO_HI) {
            const u32x2* src =
                reinterpret_cast<const u32x2*>(ldsb + (byte_hi + (k < n_hi ? shift : park_hi)));
#pragma unroll
            for (int q = 0; q < QP; ++q) bhi[slot][q] = src[q * 64];
        }
    };
    auto consume = [&](int slot) {
        const uint32_t c = bcost[slot];
        uint32_t t[4 * QP];
        // all the adds, then all the mins: no add feeds the instruction after it
#pragma unroll
        for (int q = 0; q < QP; ++q) {
            if (DO_LO) {
                t[4 * q] = pk_add(blo[slot][q].x, c);
                t[4 * q + 1] = pk_add(blo[slot][q].y, c);
            }
            if (DO_HI) {
                t[4 * q + 2] = pk_add(bhi[slot][q].x, c);
                t[4 * q + 3] = pk_add(bhi[slot][q].y, c);
            }
        }
#pragma unroll
        for (int q = 0; q < QP; ++q) {
            if (DO_LO) {
                alo[2 * q] = pk_min(alo[2 * q], t[4 * q]);
                alo[2 * q + 1] = pk_min(alo[2 * q + 1], t[4 * q + 1]);
            }
            if (DO_HI) {
                ahi[2 * q] = pk_min(ahi[2 * q], t[4 * q + 2]);
                ahi[2 * q + 1] = pk_min(ahi[2 * q + 1], t[4 * q + 3]);
            }
        }
    };

    u32x16 e = ep[k_begin >> 3];  // eight entries, one scalar load
    issue(e[0], e[1], k_begin, 0);
    for (int k0 = k_begin; k0 < k_end; k0 += 8) {
        // one batch ahead; past the prefix it fetches entries that get parked
        const u32x16 en = ep[(k0 >> 3) + 1];
#pragma unroll
        for (int z = 0; z < 8; ++z) {
            if (z < 7) {
                issue(e[2 * z + 2], e[2 * z + 3], k0 + z + 1, (z + 1) & 1);
            } else {
                // first touch of the batch fetched above: pinned here so that the
                // wait for that scalar load comes after seven entries of work
                uint32_t sh = en[0], c2 = en[1];
                asm volatile("" : "+s"(sh), "+s"(c2));
                issue(sh, c2, k0 + 8, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            consume(z & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        e = en;
    }
}

// Clamp a finished position, store it to the HBM row (cells <= T only).
__device__ __forceinline__ void finish_position(uint32_t (&acc)[2 * QP], uint16_t* out, int pos,
                                                int lane, int T)
{
#pragma unroll
    for (int q = 0; q < QP; ++q) {
        acc[2 * q] = pk_min(acc[2 * q], F_INF2);
        acc[2 * q + 1] = pk_min(acc[2 * q + 1], F_INF2);
        const int cell = 4 * (pos * (64 * QP) + q * 64 + lane);
        if (cell <= T) {
            u32x2 v;
            v.x = acc[2 * q];
            v.y = acc[2 * q + 1];
            *reinterpret_cast<u32x2*>(out + cell) = v;
        }
    }
}

// Write a finished position into the four shifted LDS copies.  `at` is the
// byte address of the lane's first quad in copy 0; copy m holds cell t at
// half-word (PADB/2 + t - m).  volatile: each store must stay a naturally
// aligned access of exactly this width (merged neighbours would be misaligned).
__device__ __forceinline__ void publish_position(const uint32_t (&acc)[2 * QP], char* at, int CSB)
{
#pragma unroll
    for (int q = 0; q < QP; ++q) {
        const uint32_t lo = acc[2 * q], hi = acc[2 * q + 1];         // cells c0 c1 | c2 c3
        const uint32_t mid = __builtin_amdgcn_alignbit(hi, lo, 16);  // c1 c2
        char* const p = at + q * 512;
        u32x2 v;
        v.x = lo;
        v.y = hi;
        *reinterpret_cast<volatile u32x2*>(p) = v;                                 // copy 0
        *reinterpret_cast<volatile uint16_t*>(p + CSB - 2) = (uint16_t)lo;         // copy 1
        *reinterpret_cast<volatile uint32_t*>(p + CSB) = mid;
        *reinterpret_cast<volatile uint16_t*>(p + CSB + 4) = (uint16_t)(hi >> 16);
        *reinterpret_cast<volatile uint32_t*>(p + 2 * CSB - 4) = lo;               // copy 2
        *reinterpret_cast<volatile uint32_t*>(p + 2 * CSB) = hi;
        *reinterpret_cast<volatile uint16_t*>(p + 3 * CSB - 6) = (uint16_t)lo;     // copy 3
        *reinterpret_cast<volatile uint32_t*>(p + 3 * CSB - 4) = mid;
        *reinterpret_cast<volatile uint16_t*>(p + 3 * CSB) = (uint16_t)(hi >> 16);
    }
}

__global__ __launch_bounds__(1024) void k2_minplus_wide(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum,
    const int32_t* __restrict__ tmeta, const int32_t* __restrict__ order,
    int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow, int N, int S, int Kp, int nbs,
    int row_stride, int cls)
{
    extern __shared__ uint32_t lds[];
    const int nwc = blockDim.x >> 6;             // wavefronts of this class
    const int CSB = wide_copy_bytes(nwc);        // bytes per copy: pad + two positions per wave
    char* const ldsb = reinterpret_cast<char*>(lds);
    volatile uint32_t* const slot = lds + CSB;   // one dword after the four copies

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int count = as_constant(ctrl)[cls];
    const int32_t* const my_order = order + (size_t)cls * N;

    for (;;) {
        const int i = next_instance(slot, ctrl + N_CLS + cls, count, my_order);
        if (i < 0) break;
        const int T = as_constant(tmeta)[i];
        const int npos = (T + POSC) / POSC;  // positions that hold cells 0..T
        const int pos_lo = w, pos_hi = npos - 1 - w;
        const bool has_lo = pos_lo <= pos_hi;  // an odd middle position is a "lo" without a "hi"
        const bool has_hi = pos_lo < pos_hi;
        // byte offset of this lane's first quad of each position inside a copy
        const uint32_t byte_lo = (uint32_t)(PADB + 8 * (pos_lo * (64 * QP) + lane));
        const uint32_t byte_hi = (uint32_t)(PADB + 8 * (pos_hi * (64 * QP) + lane));
        // offset that sends a lane's position read to the F_INF pad of copy 0
        const uint32_t park_lo = 0u - (uint32_t)(PADB + 8 * pos_lo * (64 * QP));
        const uint32_t park_hi = 0u - (uint32_t)(PADB + 8 * pos_hi * (64 * QP));

        // rows before the first model: cells t < 0 are F_INF, cells t >= 0 are 0
        for (int x = tid; x < CSB / 4; x += (int)blockDim.x) {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t h0 = 2 * x < PADB / 2 - m ? F_INF : 0u;
                const uint32_t h1 = 2 * x + 1 < PADB / 2 - m ? F_INF : 0u;
                lds[m * (CSB / 4) + x] = h0 | (h1 << 16);
            }
        }
        __syncthreads();

        for (int s = S - 1; s >= 0; --s) {
            uint32_t alo[2 * QP], ahi[2 * QP];
#pragma unroll
            for (int u = 0; u < 2 * QP; ++u) alo[u] = ahi[u] = 0xFFFFFFFFu;

            const size_t row = (size_t)i * S + s;
            const AS_CONST u32x16* ep =
                reinterpret_cast<const AS_CONST u32x16*>(as_constant(step_tab + row * Kp));
            const AS_CONST uint16_t* bc = as_constant(bcum + row * nbs);
            if (has_hi) {
                const int n_lo = prefix_count(bc, (pos_lo + 1) * POSC - 1);
                const int n_hi = prefix_count(bc, (pos_hi + 1) * POSC - 1);
                const int k_both = (n_lo + 7) & ~7;
                const int k_end = (n_hi + 7) & ~7;
                // entries that reach both positions, then those that reach only the upper one
                sweep<true, true>(alo, ahi, ldsb, ep, 0, k_both, n_lo, n_hi, byte_lo, byte_hi,
                                  park_lo, park_hi);
                sweep<false, true>(alo, ahi, ldsb, ep, k_both, k_end, n_lo, n_hi, byte_lo, byte_hi,
                                   park_lo, park_hi);
            } else if (has_lo) {
                // a lone middle position
                const int n_lo = prefix_count(bc, (pos_lo + 1) * POSC - 1);
                sweep<true, false>(alo, ahi, ldsb, ep, 0, (n_lo + 7) & ~7, n_lo, 0, byte_lo, byte_hi,
                                   park_lo, park_hi);
            }

            uint16_t* const out = frow + row * row_stride;
            if (has_lo) finish_position(alo, out, pos_lo, lane, T);
            if (has_hi) finish_position(ahi, out, pos_hi, lane, T);
            if (s == 0) break;  // nothing reads the LDS copies of the last row

            __syncthreads();  // every wavefront is done reading the previous row
            if (has_lo) publish_position(alo, ldsb + byte_lo, CSB);
            if (has_hi) publish_position(ahi, ldsb + byte_hi, CSB);
            __syncthreads();
        }
        __syncthreads();  // last row's reads are done before the LDS is re-initialised
    }
}

// ---------------------------------------------------------------- narrow kernel
// Rows of up to 32768 cells: 16 wavefronts, each a contiguous chunk of 16
// dwords (32 cells) per lane, two copies read with ds_read_b32.
constexpr int NAR_NW = NAR_WAVES;
constexpr int NAR_U = NAR_CHUNK_DW / 64;     // dwords per lane
constexpr int NAR_CHUNK = NAR_CHUNK_DW;      // dwords per wavefront
constexpr int NAR_PADW = NAR_CHUNK;          // F_INF dwords in front of each copy
constexpr int NAR_BOFF = NAR_COPY_DW;        // dwords per copy, pad included

__global__ __launch_bounds__(NAR_NW * 64) void k2_minplus_narrow(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum,
    const int32_t* __restrict__ tmeta, const int32_t* __restrict__ order,
    int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow, int N, int S, int Kp, int nbs,
    int row_stride)
{
    extern __shared__ uint32_t lds[];  // [A: pad + 16 chunks][B: pad + 16 chunks][slot]
    volatile uint32_t* const slot = lds + 2 * NAR_BOFF;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j0 = w * NAR_CHUNK;  // first dword of this wavefront's chunk
    const int count = as_constant(ctrl)[NARROW_CLS];
    const int32_t* const my_order = order + (size_t)NARROW_CLS * N;
    const int last_cell = 2 * (j0 + NAR_CHUNK) - 1;

    for (;;) {
        const int i = next_instance(slot, ctrl + N_CLS + NARROW_CLS, count, my_order);
        if (i < 0) break;
        const int T = as_constant(tmeta)[i];
        const int ndw = (T >> 1) + 1;  // dwords that hold cells 0..T
        const bool active = j0 < ndw;

        // copy A: dword j = cells (2j, 2j+1); copy B: dword j = cells (2j+1, 2j+2).
        // f[S][t] = 0 for t >= 0; pads F_INF; B's dword -1 is (cell -1, cell 0).
        for (int x = tid; x < NAR_BOFF; x += NAR_NW * 64) {
            lds[x] = x < NAR_PADW ? F_INF2 : 0u;
            lds[NAR_BOFF + x] = x < NAR_PADW - 1 ? F_INF2 : (x == NAR_PADW - 1 ? F_INF : 0u);
        }
        __syncthreads();

        for (int s = S - 1; s >= 0; --s) {
            uint32_t acc[NAR_U];
#pragma unroll
            for (int u = 0; u < NAR_U; ++u) acc[u] = 0xFFFFFFFFu;

            const size_t row = (size_t)i * S + s;
            if (active) {
                const AS_CONST StepEntry* ep = as_constant(step_tab + row * Kp);
                const int n = prefix_count(as_constant(bcum + row * nbs), last_cell > T ? T : last_cell);
                for (int k = 0; k < n; ++k) {
                    const uint32_t cost2 = ep[k].cost2;
                    // shift = byte offset of the aligned source of dword 0 (copy A or B)
                    const uint32_t* src = lds + ((ep[k].shift >> 2) + j0 + lane);
#pragma unroll
                    for (int u = 0; u < NAR_U; ++u)
                        acc[u] = pk_min(acc[u], pk_add(src[u * 64], cost2));
                }
            }

            uint32_t* const out = reinterpret_cast<uint32_t*>(frow + row * row_stride);
#pragma unroll
            for (int u = 0; u < NAR_U; ++u) {
                acc[u] = pk_min(acc[u], F_INF2);
                const int j = j0 + u * 64 + lane;
                if (j < ndw) out[j] = acc[u];
            }
            if (s == 0) break;

            __syncthreads();
            if (active) {
                volatile uint16_t* const b16 = reinterpret_cast<volatile uint16_t*>(lds + NAR_BOFF);
#pragma unroll
                for (int u = 0; u < NAR_U; ++u) {
                    const int j = j0 + u * 64 + lane;
                    lds[NAR_PADW + j] = acc[u];
                    // B[j-1].hi = cell 2j, B[j].lo = cell 2j+1; two aligned 16-bit stores
                    b16[2 * (NAR_PADW + j) - 1] = (uint16_t)(acc[u] & 0xFFFFu);
                    b16[2 * (NAR_PADW + j)] = (uint16_t)(acc[u] >> 16);
                }
            }
            __syncthreads();
        }
        __syncthreads();
    }
}

int cu_count()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        return 256;
    return n;
}

constexpr size_t LDS_PER_CU = 160 * 1024;

}  // namespace

hipError_t launch_minplus(const themis_problem_t&, const Layout& L_, char* ws, hipStream_t st)
{
    const StepEntry* w0 = (const StepEntry*)(ws + L_.step_off);
    const uint16_t* bcum = (const uint16_t*)(ws + L_.bcum_off);
    const int32_t* tmeta = (const int32_t*)(ws + L_.tmeta_off);
    const int32_t* order = (const int32_t*)(ws + L_.order_off);
    int32_t* ctrl = (int32_t*)(ws + L_.ctrl_off);
    uint16_t* frow = (uint16_t*)(ws + L_.frow_off);
    const int cus = cu_count();
    const int top = class_of_budget(L_.t_max);  // no instance can be in a higher class
    const int top_wide = top == NARROW_CLS ? N_WIDE_CLS - 1 : top;
    hipError_t e = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&k2_minplus_wide), hipFuncAttributeMaxDynamicSharedMemorySize,
        4 * (PADB + CLS_WAVES[top_wide] * WIDE_CHUNK * 2) + 16);
    if (e != hipSuccess) return e;

    // longest rows first: they take longest, so they should not start last
    if (top == NARROW_CLS) {
        size_t lds_bytes = (size_t)(2 * NAR_BOFF + 4) * sizeof(uint32_t);
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k2_minplus_narrow),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        int grid = L_.N < cus ? L_.N : cus;
        hipLaunchKernelGGL(k2_minplus_narrow, dim3(grid), dim3(NAR_NW * 64), lds_bytes, st, w0,
                           bcum, tmeta, order, ctrl, frow, L_.N, L_.S, L_.Kp, L_.nbs,
                           L_.row_stride);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int c = top_wide; c >= 0; --c) {
        const int nwc = CLS_WAVES[c];
        size_t lds_bytes = (size_t)4 * (PADB + nwc * WIDE_CHUNK * 2) + 16;
        int per_cu = (int)(LDS_PER_CU / lds_bytes);
        if (per_cu > 32 / nwc) per_cu = 32 / nwc;
        if (per_cu < 1) per_cu = 1;
        long long grid = (long long)cus * per_cu;
        if (grid > L_.N) grid = L_.N;
        hipLaunchKernelGGL(k2_minplus_wide, dim3((unsigned)grid), dim3(nwc * 64), lds_bytes, st, w0,
                           bcum, tmeta, order, ctrl, frow, L_.N, L_.S, L_.Kp, L_.nbs,
                           L_.row_stride, c);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace themis

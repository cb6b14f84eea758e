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
// Mapping.  One workgroup per instance, one wavefront per chunk of the row.
// Lanes run over t and the candidate loop is wave-uniform: lt and cost live in
// SGPRs, and a candidate contributes f[s+1] shifted by lt, a unit-stride LDS
// read.  There is no cross-lane traffic and no argmin bookkeeping in the loop:
// only f is kept, and stage 3 recovers the argmin from the stored rows.
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
// aligned.  Each wavefront owns a contiguous chunk of the row, keeps the new
// values in registers while the old row is being read, and skips candidates
// whose lt exceeds the chunk's last cell; one chunk of F_INF in front of every
// copy serves the reads that reach below t = 0.
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
typedef int32_t i32x16 __attribute__((ext_vector_type(16)));

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

// ------------------------------------------------------------------ wide kernel
constexpr int V = WIDE_V;          // quads per lane
constexpr int L = WIDE_CHUNK;      // cells per wavefront chunk (= 256 * V)

// value of half-word x of copy m before the first model: cells t < 0 are
// F_INF, cells t >= 0 are 0; cell t sits at half-word L + t - m.
__device__ __forceinline__ uint32_t init_half(int m, int x) { return x < L - m ? F_INF : 0u; }

__global__ __launch_bounds__(1024) void k2_minplus_wide(
    const CandEntry* __restrict__ cand, const int32_t* __restrict__ tmeta,
    const int32_t* __restrict__ order, int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow,
    int N, int S, int Kp, int row_stride, int cls)
{
    extern __shared__ uint32_t lds[];
    const int nwc = blockDim.x >> 6;            // wavefronts of this class
    const int CSB = (nwc + 1) * L * 2;          // bytes per copy (pad chunk + nwc chunks)
    char* const ldsb = reinterpret_cast<char*>(lds);
    volatile uint32_t* const slot = lds + CSB;  // one dword after the four copies

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int count = as_constant(ctrl)[cls];
    const int32_t* const my_order = order + (size_t)cls * N;
    // byte offset of this lane's first quad inside a copy's data area
    const uint32_t lane_byte = (uint32_t)(2 * L + 8 * (w * (L / 4) + lane));
    const uint32_t last_cell = (uint32_t)((w + 1) * L - 1);

    for (;;) {
        const int i = next_instance(slot, ctrl + N_CLS + cls, count, my_order);
        if (i < 0) break;
        const int T = as_constant(tmeta)[i];
        const bool active = w * L <= T;  // this wavefront's chunk holds cells <= T

        // rows before the first model
        for (int x = tid; x < CSB / 4; x += (int)blockDim.x) {
#pragma unroll
            for (int m = 0; m < 4; ++m)
                lds[m * (CSB / 4) + x] = init_half(m, 2 * x) | (init_half(m, 2 * x + 1) << 16);
        }
        __syncthreads();

        for (int s = S - 1; s >= 0; --s) {
            uint32_t acc[2 * V];
#pragma unroll
            for (int u = 0; u < 2 * V; ++u) acc[u] = 0xFFFFFFFFu;

            if (active) {
                const AS_CONST i32x16* ep =
                    reinterpret_cast<const AS_CONST i32x16*>(as_constant(cand + ((size_t)i * S + s) * Kp));
                for (int k0 = 0; k0 < Kp; k0 += 8) {
                    const i32x16 e = ep[k0 >> 3];  // eight (lt, cost) pairs, one scalar load
#pragma unroll
                    for (int z = 0; z < 8; ++z) {
                        const uint32_t lt = (uint32_t)e[2 * z];
                        if (lt > last_cell) continue;  // also skips infeasible (-1)
                        const uint32_t cost2 = (uint32_t)e[2 * z + 1] * 0x10001u;
                        const uint32_t m = (0u - lt) & 3u;   // copy whose shift aligns the read
                        const uint32_t h = (lt + 3u) >> 2;   // quads to step back
                        const uint32_t addr = lane_byte + m * (uint32_t)CSB - 8u * h;
                        const u32x2* src = reinterpret_cast<const u32x2*>(ldsb + addr);
#pragma unroll
                        for (int v = 0; v < V; ++v) {
                            const u32x2 r = src[v * 64];
                            acc[2 * v] = pk_min(acc[2 * v], pk_add(r.x, cost2));
                            acc[2 * v + 1] = pk_min(acc[2 * v + 1], pk_add(r.y, cost2));
                        }
                    }
                }
            }

            uint16_t* const out = frow + ((size_t)i * S + s) * row_stride;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                acc[2 * v] = pk_min(acc[2 * v], F_INF2);
                acc[2 * v + 1] = pk_min(acc[2 * v + 1], F_INF2);
                const int cell = 4 * (w * (L / 4) + v * 64 + lane);
                if (cell <= T) {
                    u32x2 q;
                    q.x = acc[2 * v];
                    q.y = acc[2 * v + 1];
                    *reinterpret_cast<u32x2*>(out + cell) = q;
                }
            }
            if (s == 0) break;  // nothing reads the LDS copies of the last row

            __syncthreads();  // every wavefront is done reading the previous row
            if (active) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const uint32_t lo = acc[2 * v], hi = acc[2 * v + 1];  // cells c0 c1 | c2 c3
                    const uint32_t mid = __builtin_amdgcn_alignbit(hi, lo, 16);  // c1 c2
                    char* const at = ldsb + lane_byte + v * 512;  // copy 0, this quad
                    // volatile: each store must stay a naturally aligned access of
                    // exactly this width (merged neighbours would be misaligned)
                    u32x2 q;
                    q.x = lo;
                    q.y = hi;
                    *reinterpret_cast<volatile u32x2*>(at) = q;                                // copy 0
                    *reinterpret_cast<volatile uint16_t*>(at + CSB - 2) = (uint16_t)lo;        // copy 1
                    *reinterpret_cast<volatile uint32_t*>(at + CSB) = mid;
                    *reinterpret_cast<volatile uint16_t*>(at + CSB + 4) = (uint16_t)(hi >> 16);
                    *reinterpret_cast<volatile uint32_t*>(at + 2 * CSB - 4) = lo;              // copy 2
                    *reinterpret_cast<volatile uint32_t*>(at + 2 * CSB) = hi;
                    *reinterpret_cast<volatile uint16_t*>(at + 3 * CSB - 6) = (uint16_t)lo;    // copy 3
                    *reinterpret_cast<volatile uint32_t*>(at + 3 * CSB - 4) = mid;
                    *reinterpret_cast<volatile uint16_t*>(at + 3 * CSB) = (uint16_t)(hi >> 16);
                }
            }
            __syncthreads();
        }
        __syncthreads();  // last row's reads are done before the LDS is re-initialised
    }
}

// ---------------------------------------------------------------- narrow kernel
// Rows of up to 32768 cells: 16 wavefronts, 16 dwords (32 cells) per lane, two
// copies read with ds_read_b32.
constexpr int NAR_NW = 16;
constexpr int NAR_U = 16;
constexpr int NAR_CHUNK = 64 * NAR_U;        // dwords per wavefront
constexpr int NAR_PADW = NAR_CHUNK;
constexpr int NAR_CAPW = NAR_NW * NAR_CHUNK; // dwords per copy
constexpr int NAR_BOFF = NAR_PADW + NAR_CAPW;

__global__ __launch_bounds__(NAR_NW * 64) void k2_minplus_narrow(
    const CandEntry* __restrict__ cand, const int32_t* __restrict__ tmeta,
    const int32_t* __restrict__ order, int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow,
    int N, int S, int Kp, int row_stride)
{
    extern __shared__ uint32_t lds[];  // [A: PADW + CAPW][B: PADW + CAPW][slot]
    volatile uint32_t* const slot = lds + 2 * NAR_BOFF;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j0 = w * NAR_CHUNK;  // first dword of this wavefront's chunk
    const int count = as_constant(ctrl)[NARROW_CLS];
    const int32_t* const my_order = order + (size_t)NARROW_CLS * N;
    const uint32_t last_cell = 2u * (uint32_t)(j0 + NAR_CHUNK) - 1u;

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

            if (active) {
                const AS_CONST i32x16* ep =
                    reinterpret_cast<const AS_CONST i32x16*>(as_constant(cand + ((size_t)i * S + s) * Kp));
                for (int k0 = 0; k0 < Kp; k0 += 8) {
                    const i32x16 e = ep[k0 >> 3];
#pragma unroll
                    for (int z = 0; z < 8; ++z) {
                        const uint32_t lt = (uint32_t)e[2 * z];
                        if (lt > last_cell) continue;
                        const uint32_t cost2 = (uint32_t)e[2 * z + 1] * 0x10001u;
                        const int h = (int)(lt >> 1);
                        // even lt: A[j - h]; odd lt: B[j - h - 1]
                        const int base = (lt & 1u) ? (NAR_BOFF + NAR_PADW - 1 - h) : (NAR_PADW - h);
                        const uint32_t* src = lds + (base + j0 + lane);
#pragma unroll
                        for (int u = 0; u < NAR_U; ++u)
                            acc[u] = pk_min(acc[u], pk_add(src[u * 64], cost2));
                    }
                }
            }

            uint32_t* const out =
                reinterpret_cast<uint32_t*>(frow + ((size_t)i * S + s) * row_stride);
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
    const CandEntry* cand = (const CandEntry*)(ws + L_.cand_off);
    const int32_t* tmeta = (const int32_t*)(ws + L_.tmeta_off);
    const int32_t* order = (const int32_t*)(ws + L_.order_off);
    int32_t* ctrl = (int32_t*)(ws + L_.ctrl_off);
    uint16_t* frow = (uint16_t*)(ws + L_.frow_off);
    const int cus = cu_count();
    const int top = class_of_budget(L_.t_max);  // no instance can be in a higher class

    const int top_wide = top == NARROW_CLS ? N_WIDE_CLS - 1 : top;
    hipError_t e = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&k2_minplus_wide), hipFuncAttributeMaxDynamicSharedMemorySize,
        4 * (CLS_WAVES[top_wide] + 1) * WIDE_CHUNK * 2 + 16);
    if (e != hipSuccess) return e;

    // longest rows first: they take longest, so they should not start last
    if (top == NARROW_CLS) {
        size_t lds_bytes = (size_t)(2 * NAR_BOFF + 4) * sizeof(uint32_t);
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k2_minplus_narrow),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        int grid = L_.N < cus ? L_.N : cus;
        hipLaunchKernelGGL(k2_minplus_narrow, dim3(grid), dim3(NAR_NW * 64), lds_bytes, st, cand,
                           tmeta, order, ctrl, frow, L_.N, L_.S, L_.Kp, L_.row_stride);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int c = top_wide; c >= 0; --c) {
        const int nwc = CLS_WAVES[c];
        size_t lds_bytes = (size_t)4 * (nwc + 1) * WIDE_CHUNK * 2 + 16;
        int per_cu = (int)(LDS_PER_CU / lds_bytes);
        if (per_cu > 32 / nwc) per_cu = 32 / nwc;
        if (per_cu < 1) per_cu = 1;
        long long grid = (long long)cus * per_cu;
        if (grid > L_.N) grid = L_.N;
        hipLaunchKernelGGL(k2_minplus_wide, dim3((unsigned)grid), dim3(nwc * 64), lds_bytes, st,
                           cand, tmeta, order, ctrl, frow, L_.N, L_.S, L_.Kp, L_.row_stride, c);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace themis

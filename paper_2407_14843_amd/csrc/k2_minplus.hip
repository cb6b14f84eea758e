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
// Mapping.  One workgroup of 8 wavefronts per instance.  Lanes run over t, the
// candidate loop is wave-uniform: lt and cost live in SGPRs, and a candidate
// contributes f[s+1] shifted by lt, a unit-stride LDS read.  No cross-lane
// traffic and no argmin bookkeeping in the loop: only f is kept, and stage 3
// recovers the argmin from the stored rows.
//
// f is 16 bits wide (totals are bounded by THEMIS_COST_LIMIT), two cells per
// dword, so one v_pk_add_u16 + one v_pk_min_u16 relax two cells for one LDS
// dword.  A shift by an odd lt would straddle dwords, so the previous row is
// kept twice in LDS: copy A holds cells (2j, 2j+1) in dword j, copy B holds
// cells (2j+1, 2j+2).  Even shifts read A, odd shifts read B, both aligned.
// Each wavefront owns a contiguous chunk of the row, keeps the new values in
// registers while the old row is being read, and skips candidates whose lt
// exceeds the chunk's last cell; a pad of F_INF one chunk long in front of
// each copy serves reads that reach below t = 0.
#include "themis_internal.h"

namespace themis {
namespace {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

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

constexpr int NW = 8;  // wavefronts per workgroup

// The candidate tables were written by an earlier kernel and are read-only
// here.  Viewing them through the constant address space tells the compiler so
// (a workgroup barrier otherwise counts as a possible writer), which lets it
// fetch the wave-uniform entries with scalar loads into SGPRs.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;

__device__ __forceinline__ const_i32_ptr as_constant(const int32_t* p)
{
    return (const_i32_ptr)(uintptr_t)p;
}

// U = dwords (pairs of cells) per lane.  Row capacity = NW*64*U dwords.
template <int U>
__global__ __launch_bounds__(NW * 64) void k2_minplus(
    const int32_t* __restrict__ lt_tab, const int32_t* __restrict__ cost_tab,
    const int32_t* __restrict__ tmeta, uint16_t* __restrict__ frow, int S, int K,
    int row_stride)
{
    constexpr int CHUNK = 64 * U;      // dwords per wavefront
    constexpr int PADW = CHUNK;        // F_INF dwords in front of each copy
    constexpr int CAPW = NW * CHUNK;   // dwords per copy
    extern __shared__ uint32_t lds[];  // [A: PADW + CAPW][B: PADW + CAPW]
    constexpr int BOFF = PADW + CAPW;

    const int i = blockIdx.x;
    const int T = as_constant(tmeta)[i];
    if (T < 0) return;  // invalid instance: stage 3 reports it

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j0 = w * CHUNK;           // first dword of this wavefront's chunk
    const int ndw = (T >> 1) + 1;       // dwords that hold cells 0..T
    const bool active = j0 < ndw;

    // f[S][t] = 0 for t >= 0; pads F_INF; B's dword -1 is (cell -1, cell 0).
    for (int x = tid; x < BOFF; x += NW * 64) {
        lds[x] = x < PADW ? F_INF2 : 0u;
        lds[BOFF + x] = x < PADW - 1 ? F_INF2 : (x == PADW - 1 ? F_INF : 0u);
    }
    __syncthreads();

    uint16_t* const b16 = reinterpret_cast<uint16_t*>(lds + BOFF);

    for (int s = S - 1; s >= 0; --s) {
        const const_i32_ptr ltp = as_constant(lt_tab + ((size_t)i * S + s) * K);
        const const_i32_ptr cop = as_constant(cost_tab + ((size_t)i * S + s) * K);
        uint32_t acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = 0xFFFFFFFFu;

        if (active) {
            const uint32_t last_cell = 2u * (uint32_t)(j0 + CHUNK) - 1u;
            for (int k = 0; k < K; ++k) {
                const uint32_t lt = (uint32_t)ltp[k];
                if (lt > last_cell) continue;  // also skips infeasible (-1)
                const uint32_t cost2 = (uint32_t)cop[k] * 0x10001u;
                const int h = (int)(lt >> 1);
                // even lt: A[j - h]; odd lt: B[j - h - 1]
                const int base = (lt & 1u) ? (BOFF + PADW - 1 - h) : (PADW - h);
                const uint32_t* src = lds + (base + j0 + lane);
#pragma unroll
                for (int u = 0; u < U; ++u)
                    acc[u] = pk_min(acc[u], pk_add(src[u * 64], cost2));
            }
        }

        uint32_t* __restrict__ out =
            reinterpret_cast<uint32_t*>(frow + ((size_t)i * S + s) * row_stride);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc[u] = pk_min(acc[u], F_INF2);
            const int j = j0 + u * 64 + lane;
            if (j < ndw) out[j] = acc[u];
        }
        if (s == 0) break;  // nothing reads the LDS copy of the last row

        __syncthreads();  // every wavefront is done reading the previous row
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * 64 + lane;
            lds[PADW + j] = acc[u];
            // B[j-1].hi = cell 2j, B[j].lo = cell 2j+1
            b16[2 * (PADW + j) - 1] = (uint16_t)(acc[u] & 0xFFFFu);
            b16[2 * (PADW + j)] = (uint16_t)(acc[u] >> 16);
        }
        __syncthreads();
    }
}

template <int U>
hipError_t launch_u(const Layout& L, char* ws, hipStream_t st)
{
    size_t lds_bytes = (size_t)2 * (64 * U + NW * 64 * U) * sizeof(uint32_t);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k2_minplus<U>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k2_minplus<U>, dim3(L.N), dim3(NW * 64), lds_bytes, st,
                       (const int32_t*)(ws + L.lt_off), (const int32_t*)(ws + L.cost_off),
                       (const int32_t*)(ws + L.tmeta_off), (uint16_t*)(ws + L.frow_off),
                       L.S, L.K, L.row_stride);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_minplus(const themis_problem_t&, const Layout& L, char* ws, hipStream_t st)
{
    // smallest U whose row capacity (NW*128*U cells) covers cells 0..t_max
    int cells = L.t_max + 1;
    if (cells <= NW * 128 * 1) return launch_u<1>(L, ws, st);
    if (cells <= NW * 128 * 2) return launch_u<2>(L, ws, st);
    if (cells <= NW * 128 * 4) return launch_u<4>(L, ws, st);
    if (cells <= NW * 128 * 8) return launch_u<8>(L, ws, st);
    if (cells <= NW * 128 * 16) return launch_u<16>(L, ws, st);
    if (cells <= NW * 128 * 32) return launch_u<32>(L, ws, st);
    return hipErrorInvalidValue;
}

}  // namespace themis

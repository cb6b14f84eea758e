// Solving every distinct instance once.
//
// A sweep over an arrival-rate trace (Section 6 drives the system with the
// per-second rates of one) hands the solver the same (rate, objective, replicas,
// profile) tuple again and again.  Equal inputs have equal answers, so only one
// instance per distinct tuple needs the three stages:
//   k6_fill     empties the hash table;
//   k6_dedupe   one thread per instance: hash the instance's input words,
//               insert the instance's index with open addressing (a compare
//               and swap per probe); the first index to take a slot is the
//               representative of its tuple, later ones with equal words
//               learn it from the slot.  Writes rep[i], the arrival rates of
//               the pass that follows (0 = switched off for every instance
//               that is not its own representative), and "invalid" into every
//               output, which the pass overwrites for the representatives
//               that pass the input check;
//   k6_scatter  after the pass: every other instance copies the outputs of
//               its representative.
// Which index of a tuple becomes the representative depends on the order the
// threads arrive in; the outputs do not, since equal inputs have one answer.
#include "themis_internal.h"

namespace themis {
namespace {

constexpr int32_t MEMO_EMPTY = -1;

__global__ __launch_bounds__(256) void k6_fill(int32_t* __restrict__ table, uint32_t slots)
{
    const uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g < slots) table[g] = MEMO_EMPTY;
}

struct MemoIn {
    const int32_t* coef;     // [N][S][cs], or [S][cs] when shared (then not part of the tuple)
    const int32_t* lambda;   // [N]
    const int32_t* slo_us;   // [N]
    const int32_t* r_fixed;  // [N][S] or null
    int S, cs, coef_shared;
};

__device__ __forceinline__ uint32_t mix(uint32_t h, uint32_t word)
{
    h ^= word;
    h *= 0x9E3779B1u;
    return h ^ (h >> 15);
}

__device__ uint32_t hash_of(const MemoIn& in, uint32_t i)
{
    uint32_t h = mix(mix(0x243F6A88u, (uint32_t)in.lambda[i]), (uint32_t)in.slo_us[i]);
    if (in.r_fixed)
        for (int s = 0; s < in.S; ++s) h = mix(h, (uint32_t)in.r_fixed[(size_t)i * in.S + s]);
    if (!in.coef_shared) {
        const int32_t* c = in.coef + (size_t)i * in.S * in.cs;
        for (int x = 0; x < in.S * in.cs; ++x) h = mix(h, (uint32_t)c[x]);
    }
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    return h ^ (h >> 13);
}

__device__ bool same_inputs(const MemoIn& in, uint32_t a, uint32_t b)
{
    bool same = in.lambda[a] == in.lambda[b] && in.slo_us[a] == in.slo_us[b];
    if (same && in.r_fixed)
        for (int s = 0; s < in.S; ++s)
            same = same && in.r_fixed[(size_t)a * in.S + s] == in.r_fixed[(size_t)b * in.S + s];
    if (same && !in.coef_shared) {
        const int32_t* ca = in.coef + (size_t)a * in.S * in.cs;
        const int32_t* cb = in.coef + (size_t)b * in.S * in.cs;
        for (int x = 0; x < in.S * in.cs; ++x) same = same && ca[x] == cb[x];
    }
    return same;
}

__global__ __launch_bounds__(256) void k6_dedupe(MemoIn in, int32_t* __restrict__ table,
                                                 uint32_t slots, int32_t* __restrict__ rep,
                                                 int32_t* __restrict__ lam_pass,
                                                 int32_t* __restrict__ status,
                                                 int32_t* __restrict__ cost,
                                                 int32_t* __restrict__ ticks,
                                                 int32_t* __restrict__ cfg, uint32_t N)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= N) return;
    const uint32_t h = hash_of(in, i);
    // The table has at least twice as many slots as there are instances, so a
    // probe sequence meets an empty slot (or an equal instance) long before it has
    // gone round; the bound makes the loop finite whatever the table holds.
    int32_t mine = (int32_t)i;
    for (uint32_t probe = 0; probe < slots; ++probe) {
        const uint32_t slot = (h + probe) & (slots - 1u);
        const int32_t seen = atomicCAS(&table[slot], MEMO_EMPTY, (int32_t)i);
        if (seen == MEMO_EMPTY) break;  // the slot is this instance's: it represents its tuple
        if ((uint32_t)seen < N && same_inputs(in, i, (uint32_t)seen)) {
            mine = seen;
            break;
        }
    }
    rep[i] = mine;
    lam_pass[i] = mine == (int32_t)i ? in.lambda[i] : 0;
    status[i] = THEMIS_INVALID;
    cost[i] = -1;
    ticks[i] = -1;
    for (int x = 0; x < 3 * in.S; ++x) cfg[(size_t)i * 3 * in.S + x] = 0;
}

__global__ __launch_bounds__(256) void k6_scatter(const int32_t* __restrict__ rep,
                                                  int32_t* __restrict__ status,
                                                  int32_t* __restrict__ cost,
                                                  int32_t* __restrict__ ticks,
                                                  int32_t* __restrict__ cfg, uint32_t N, int S)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= N) return;
    const uint32_t r = (uint32_t)rep[i];
    if (r == i || r >= N) return;
    // representatives are never written here, so reading theirs races with nothing
    status[i] = status[r];
    cost[i] = cost[r];
    ticks[i] = ticks[r];
    for (int x = 0; x < 3 * S; ++x) cfg[(size_t)i * 3 * S + x] = cfg[(size_t)r * 3 * S + x];
}

}  // namespace

hipError_t launch_memo_dedupe(const themis_problem_t& p, const Layout& L, const MemoLayout& M,
                              const int32_t* d_coef, const int32_t* d_lambda,
                              const int32_t* d_slo_us, const int32_t* d_r_fixed,
                              int32_t* d_status, int32_t* d_cost, int32_t* d_ticks,
                              int32_t* d_cfg, char* ws, hipStream_t st)
{
    int32_t* table = (int32_t*)(ws + M.table_off);
    hipLaunchKernelGGL(k6_fill, dim3((M.slots + 255u) / 256u), dim3(256), 0, st, table, M.slots);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    MemoIn in{};
    in.coef = d_coef;
    in.lambda = d_lambda;
    in.slo_us = d_slo_us;
    in.r_fixed = d_r_fixed;
    in.S = L.S;
    in.cs = p.profile_form == THEMIS_PROFILE_EQ1 ? 6 : 5;
    in.coef_shared = p.coef_shared;
    hipLaunchKernelGGL(k6_dedupe, dim3(((uint32_t)L.N + 255u) / 256u), dim3(256), 0, st, in, table,
                       M.slots, (int32_t*)(ws + M.rep_off), (int32_t*)(ws + M.lam_off), d_status,
                       d_cost, d_ticks, d_cfg, (uint32_t)L.N);
    return hipGetLastError();
}

hipError_t launch_memo_scatter(const Layout& L, const MemoLayout& M, int32_t* d_status,
                               int32_t* d_cost, int32_t* d_ticks, int32_t* d_cfg, const char* ws,
                               hipStream_t st)
{
    hipLaunchKernelGGL(k6_scatter, dim3(((uint32_t)L.N + 255u) / 256u), dim3(256), 0, st,
                       (const int32_t*)(ws + M.rep_off), d_status, d_cost, d_ticks, d_cfg,
                       (uint32_t)L.N, L.S);
    return hipGetLastError();
}

}  // namespace themis

// Workload-stability test of Section 5.1.3: the horizontal solve is run at the
// current and at the predicted arrival rate, and the workload counts as stable
// when both succeed with the same configuration for every model.  The two
// solves are ordinary passes of the three stages; this kernel compares what
// they left behind, one thread per instance.
#include "themis_internal.h"

namespace themis {
namespace {

__global__ __launch_bounds__(256) void k5_same_config(
    const int32_t* __restrict__ status_now, const int32_t* __restrict__ cfg_now,
    const int32_t* __restrict__ status_pred, const int32_t* __restrict__ cfg_pred,
    int32_t* __restrict__ stable, int N, int S)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    int same = (int)(status_now[i] == THEMIS_SOLVED) & (int)(status_pred[i] == THEMIS_SOLVED);
    const size_t at = (size_t)i * S * 3;
    for (int x = 0; x < 3 * S; ++x) same &= (int)(cfg_now[at + x] == cfg_pred[at + x]);
    stable[i] = same;
}

}  // namespace

hipError_t launch_same_config(const Layout& L, const int32_t* status_now, const int32_t* cfg_now,
                              const int32_t* status_pred, const int32_t* cfg_pred,
                              int32_t* stable, hipStream_t st)
{
    hipLaunchKernelGGL(k5_same_config, dim3((L.N + 255) / 256), dim3(256), 0, st, status_now,
                       cfg_now, status_pred, cfg_pred, stable, L.N, L.S);
    return hipGetLastError();
}

}  // namespace themis

// Regrouping generator as a kernel of its own (Sec. 3.1 "Shuffle-Exchange"; Algorithm 1:
// "randomly generate new groups depending on the seed").  One wavefront, one lane per
// worker; the same device function is what the step kernel evaluates in every wavefront.
#include "se_device.hpp"

namespace se {

__global__ __launch_bounds__(64) void se_plan_kernel(uint64_t seed, int64_t iter, int n, int m,
                                                     int32_t *group_of, int32_t *members)
{
    const int lane = (int)threadIdx.x;
    const uint32_t grp = wave_group_of(seed, iter, n, m, lane);
    if (lane < n) group_of[lane] = (int32_t)grp;
    if (members) {
        const int k = n / m;
        for (int g = 0; g < k; ++g) {
            const uint64_t mask = __ballot(grp == (uint32_t)g);
            if (grp == (uint32_t)g) {
                // position inside the group = number of members with a smaller id
                const int r = __popcll(mask & ((1ull << lane) - 1ull));
                members[g * m + r] = lane;
            }
        }
    }
}

hipError_t launch_plan(uint64_t seed, int64_t iter, int n, int m, int32_t *group_of_dev,
                       int32_t *members_dev, hipStream_t stream)
{
    hipLaunchKernelGGL(se_plan_kernel, dim3(1), dim3(64), 0, stream, seed, iter, n, m,
                       group_of_dev, members_dev);
    return hipGetLastError();
}

}  // namespace se

// Regrouping generator as a kernel of its own (Sec. 3.1 "Shuffle-Exchange"; Algorithm 1:
// "randomly generate new groups depending on the seed").  One wavefront, one lane per
// worker; the same device function is what the step kernel evaluates in every wavefront.
#include "se_device.hpp"

#include <atomic>

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

// ---- the regrouping without any allocation ---------------------------------------------------
// For callers that may not allocate device memory: the two result arrays are staged in a
// file-scope device array instead of a buffer from hipMalloc.  `scratch` names the array on the
// device; in host code the name is only a handle, so its device address is looked up once per
// device with hipGetSymbolAddress and that address is what the kernel and the copies are given.
constexpr int kPlanScratchInts = 2 * kMaxWorkers;          // group_of[64] then members[64]: 512 B
static __device__ __align__(256) int32_t scratch[kPlanScratchInts];

constexpr int kMaxDevices = 64;
static std::atomic<int32_t *> g_scratch_addr[kMaxDevices];   // per device ordinal; null = not looked up

static hipError_t scratch_of_current_device(int32_t **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    int32_t *addr = g_scratch_addr[dev].load();
    if (!addr) {
        e = hipGetSymbolAddress((void **)&addr, HIP_SYMBOL(scratch));   // this device's copy
        if (e != hipSuccess) return e;
        if (!addr) return hipErrorInvalidSymbol;
        g_scratch_addr[dev].store(addr);
    }
    *out = addr;
    return hipSuccess;
}

hipError_t plan_to_host_noalloc(uint64_t seed, int64_t iter, int n, int m, int32_t *group_of_host,
                                int32_t *members_host)
{
    if (n < 1 || n > kMaxWorkers) return hipErrorInvalidValue;     // the array holds 64 workers
    int32_t *dev = nullptr;
    hipError_t e = scratch_of_current_device(&dev);
    if (e != hipSuccess) return e;
    // every entry that is copied back is written by the kernel first: nothing to clear
    hipLaunchKernelGGL(se_plan_kernel, dim3(1), dim3(64), 0, nullptr, seed, iter, n, m, dev,
                       members_host ? dev + kMaxWorkers : nullptr);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = hipMemcpy(group_of_host, dev, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost);
    if (e == hipSuccess && members_host)
        e = hipMemcpy(members_host, dev + kMaxWorkers, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost);
    return e;
}

hipError_t launch_plan(uint64_t seed, int64_t iter, int n, int m, int32_t *group_of_dev,
                       int32_t *members_dev, hipStream_t stream)
{
    hipLaunchKernelGGL(se_plan_kernel, dim3(1), dim3(64), 0, stream, seed, iter, n, m,
                       group_of_dev, members_dev);
    return hipGetLastError();
}

}  // namespace se

// Measurement helper, not part of the method: a plain device-to-device copy of a known
// number of bytes.  It gives the profiler's HBM byte counters a reference reading
// (bytes read = bytes written = nbytes) and the bandwidth figures a practical ceiling.
#include "se_device.hpp"

namespace se {

__global__ __launch_bounds__(64) void se_calib_copy_kernel(const f32x4 *__restrict__ src,
                                                           f32x4 *__restrict__ dst, uint64_t nvec)
{
    const uint64_t i = (uint64_t)blockIdx.x * 64u + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

hipError_t launch_calib_copy(void *dst, const void *src, uint64_t nbytes, hipStream_t stream)
{
    const uint64_t nvec = nbytes / 16u;
    const uint64_t grid = (nvec + 63u) / 64u;
    hipLaunchKernelGGL(se_calib_copy_kernel, dim3((uint32_t)grid), dim3(64), 0, stream,
                       (const f32x4 *)src, (f32x4 *)dst, nvec);
    return hipGetLastError();
}

}  // namespace se

// Measurement helper, not part of the method: a plain device-to-device copy of a known
// number of bytes.  It gives the profiler's HBM byte counters a reference reading
// (bytes read = bytes written = nbytes) and the bandwidth figures a practical ceiling.
#include "se_device.hpp"

namespace se {

template <int NT>
__global__ __launch_bounds__(64) void se_calib_copy_kernel(const f32x4 *__restrict__ src,
                                                           f32x4 *__restrict__ dst, uint64_t nvec)
{
    const uint64_t i = (uint64_t)blockIdx.x * 64u + threadIdx.x;
    if (i >= nvec) return;
    const f32x4 v = ld<f32x4, NT>(src + i);
    if constexpr (NT == kStreamThrough) st_through(dst + (uint64_t)blockIdx.x * 64u, threadIdx.x * 16u, v);
    else st<f32x4, NT>(dst + i, v);
}

// One direction only, to tell what the memory system gives to reads and to writes apart from
// what it gives to their mix: every wavefront reads (MODE 1) or writes (MODE 2) four consecutive
// 1 KiB pieces (a wavefront that moves a single KiB in one direction is over before it has paid
// for its dispatch: 4.8 TB/s either way).  The reader folds what it read into a store that never
// happens, so that the loads stay.
template <int MODE>
__global__ __launch_bounds__(64) void se_calib_oneway_kernel(const f32x4 *__restrict__ src,
                                                             f32x4 *__restrict__ dst, uint64_t nvec)
{
    constexpr int kPieces = 4;
    const uint64_t base = (uint64_t)blockIdx.x * (64u * kPieces) + threadIdx.x;
    if constexpr (MODE == 1) {
        f32x4 v[kPieces];
#pragma unroll
        for (int r = 0; r < kPieces; ++r) {
            const uint64_t i = base + (uint64_t)r * 64u;
            v[r] = i < nvec ? ld<f32x4, kStream>(src + i) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
        f32x4 s = v[0];
#pragma unroll
        for (int r = 1; r < kPieces; ++r) s += v[r];
        if (s.x == 1.2345678e37f && s.y == -s.x) st<f32x4, kStream>(dst + base % nvec, s);
    } else {
#pragma unroll
        for (int r = 0; r < kPieces; ++r) {
            const uint64_t i = base + (uint64_t)r * 64u;
            if (i < nvec) st<f32x4, kStream>(dst + i, f32x4{1.0f, 2.0f, 3.0f, (float)r});
        }
    }
}

hipError_t launch_calib_oneway(void *dst, const void *src, uint64_t nbytes, int mode, hipStream_t stream)
{
    const uint64_t nvec = nbytes / 16u;
    const dim3 grid((uint32_t)((nvec + 255u) / 256u));
    // residency from a sweep: 24 workgroups per CU for the reader, 4 for the writer
    if (mode == 1)
        hipLaunchKernelGGL(se_calib_oneway_kernel<1>, grid, dim3(64), 6u * 1024u, stream, (const f32x4 *)src, (f32x4 *)dst, nvec);
    else
        hipLaunchKernelGGL(se_calib_oneway_kernel<2>, grid, dim3(64), 40u * 1024u, stream, (const f32x4 *)src, (f32x4 *)dst, nvec);
    return hipGetLastError();
}

// policy: the cache policy the step kernels use (se::Policy), so that the copy is a ceiling
// for the same kind of access
hipError_t launch_calib_copy(void *dst, const void *src, uint64_t nbytes, int policy,
                             hipStream_t stream)
{
    const uint64_t nvec = nbytes / 16u;
    const dim3 grid((uint32_t)((nvec + 63u) / 64u));
    // 6 KiB of unused LDS per one-wavefront workgroup keep about 24 of them resident per CU,
    // the measured optimum for this kernel (6.81 TB/s against 6.72 with no cap, 6.09 at 16)
    const uint32_t lds = 6u * 1024u;
    const f32x4 *s = (const f32x4 *)src;
    f32x4 *d = (f32x4 *)dst;
    switch (policy) {
    case kPlain: hipLaunchKernelGGL(se_calib_copy_kernel<kPlain>, grid, dim3(64), lds, stream, s, d, nvec); break;
    case kStream: hipLaunchKernelGGL(se_calib_copy_kernel<kStream>, grid, dim3(64), lds, stream, s, d, nvec); break;
    default: hipLaunchKernelGGL(se_calib_copy_kernel<kStreamThrough>, grid, dim3(64), lds, stream, s, d, nvec); break;
    }
    return hipGetLastError();
}

}  // namespace se

// Replica-consistency diagnostics (the quantity of the paper's divergence equation, Sec. 3.2,
// and of its "consistency of parameters" experiment, Sec. 4.2), in double precision:
//   out[0] += sum_e sum_i (x_i[e] - xbar[e])^2,  xbar[e] = (sum_i x_i[e]) / n   (Sec. 3.3)
//   out[1] += sum_e sum_i x_i[e]
// A lane owns a column at a time (rows re-read for the deviations; the second read is served
// by the caches), partial sums are reduced across the wavefront with lane shuffles, across
// the wavefronts of the workgroup through LDS, and one fp64 atomic per workgroup and output
// adds them to the caller's two doubles, which a one-lane kernel cleared before.
#include "se_device.hpp"

namespace se {

__global__ void se_clear2_kernel(double *out)
{
    out[0] = 0.0;
    out[1] = 0.0;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(256) void se_consensus_kernel(const float *__restrict__ x,
                                                           uint64_t pitch, uint64_t ncols, int n,
                                                           double *out)
{
    __shared__ double part[2][4];
    double dist = 0.0, total = 0.0;
    const double inv_n = 1.0 / (double)n;
    for (uint64_t e = (uint64_t)blockIdx.x * 256u + threadIdx.x; e < ncols;
         e += (uint64_t)gridDim.x * 256u) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) s += (double)x[(uint64_t)i * pitch + e];
        const double mean = s * inv_n;
        double d = 0.0;
        for (int i = 0; i < n; ++i) {
            const double t = (double)x[(uint64_t)i * pitch + e] - mean;
            d += t * t;
        }
        dist += d;
        total += s;
    }
    dist = wave_sum(dist);
    total = wave_sum(total);
    const int wave = (int)(threadIdx.x >> 6);
    if ((threadIdx.x & 63u) == 0) { part[0][wave] = dist; part[1][wave] = total; }
    __syncthreads();
    if (threadIdx.x == 0) {
        atomicAdd(out + 0, (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]));
        atomicAdd(out + 1, (part[1][0] + part[1][1]) + (part[1][2] + part[1][3]));
    }
}

hipError_t launch_consensus(const float *x, uint64_t pitch_elems, uint64_t ncols, int n,
                            double *out_dev, hipStream_t stream)
{
    hipLaunchKernelGGL(se_clear2_kernel, dim3(1), dim3(1), 0, stream, out_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || ncols == 0) return e;
    uint64_t grid = (ncols + 255u) / 256u;
    if (grid > 256u * 16u) grid = 256u * 16u;
    hipLaunchKernelGGL(se_consensus_kernel, dim3((uint32_t)grid), dim3(256), 0, stream, x,
                       pitch_elems, ncols, n, out_dev);
    return hipGetLastError();
}

}  // namespace se

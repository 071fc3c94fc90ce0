// Replica-consistency diagnostics (the quantity of the paper's divergence equation, Sec. 3.2,
// and of its "consistency of parameters" experiment, Sec. 4.2), in double precision:
//   out[0] += sum_e sum_i (x_i[e] - xbar[e])^2,  xbar[e] = (sum_i x_i[e]) / n   (Sec. 3.3)
//   out[1] += sum_e sum_i x_i[e]
//
// Every element is read once.  A lane owns VEC columns of a 64-lane tile and walks the n rows
// in batches of 8 loads; the squared deviations are taken about row 0 instead of the mean,
//   sum_i (x_i - xbar)^2 = sum_i d_i^2 - (sum_i d_i)^2 / n,   d_i = x_i - x_0,
// where every d_i is exact in double precision (a difference of two floats), the right-hand
// side cancels at most a factor n (x_0 is one of the samples), and identical rows give exactly
// zero.  Wavefronts stride over the tiles so that the tiles in flight are neighbours; partial
// sums are reduced across the wavefront with lane shuffles, across the four wavefronts of a
// workgroup through LDS, and added to the caller's two doubles with one fp64 atomic each per
// workgroup; a one-lane kernel clears them first.
#include "se_device.hpp"

namespace se {

constexpr uint32_t kConsensusWaves = 4;               // wavefronts per workgroup
constexpr uint32_t kConsensusMaxGrid = 256u * 2u;     // 8 wavefronts per CU
constexpr int kConsensusBatch = 8;

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

// x points at the first column of the range, nvec = columns / VEC, tiles = ceil(nvec / 64).
// Every wavefront strides over the tiles on its own (wavefront w of workgroup b takes tiles
// b + (4 i + w) * gridDim.x), so the tiles in flight are the same as with one-wavefront
// workgroups; the workgroup only exists to add its wavefronts' sums with one pair of atomics
// instead of four (an fp64 atomic on one address costs about 12 ns, and all workgroups arrive at
// the end together).
template <int VEC, bool NT>
__global__ __launch_bounds__(64 * kConsensusWaves) void se_consensus_kernel(
    const float *__restrict__ x, uint64_t pitch_bytes, uint32_t nvec, uint32_t tiles, int n, double *out)
{
    __shared__ double part[2][kConsensusWaves];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const double inv_n = 1.0 / (double)n;
    double dist = 0.0, total = 0.0;
    for (uint64_t tile = blockIdx.x + (uint64_t)wave * gridDim.x; tile < tiles;
         tile += (uint64_t)kConsensusWaves * gridDim.x) {
        const uint32_t c = (uint32_t)tile * 64u + lane;
        if (c >= nvec) continue;
        const char *col = (const char *)x + (uint64_t)c * (uint64_t)(VEC * 4);
        const Pack<VEC> x0 = load_f32<VEC, NT>(col);
        double s[VEC], sd[VEC], sd2[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) { s[q] = (double)x0.a[q]; sd[q] = 0.0; sd2[q] = 0.0; }
        for (int i = 1; i < n; i += kConsensusBatch) {
            Pack<VEC> X[kConsensusBatch];
#pragma unroll
            for (int b = 0; b < kConsensusBatch; ++b)
                if (i + b < n) X[b] = load_f32<VEC, NT>(col + (uint64_t)(i + b) * pitch_bytes);
#pragma unroll
            for (int b = 0; b < kConsensusBatch; ++b) {
                if (i + b < n) {
#pragma unroll
                    for (int q = 0; q < VEC; ++q) {
                        const double xi = (double)X[b].a[q];
                        const double d = xi - (double)x0.a[q];
                        s[q] += xi;
                        sd[q] += d;
                        sd2[q] = __builtin_fma(d, d, sd2[q]);
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
            const double dev2 = sd2[q] - sd[q] * sd[q] * inv_n;
            dist += dev2 < 0.0 ? 0.0 : dev2;          // rounding only; NaN passes through
            total += s[q];
        }
    }
    dist = wave_sum(dist);
    total = wave_sum(total);
    if (lane == 0) { part[0][wave] = dist; part[1][wave] = total; }
    __syncthreads();
    static_assert(kConsensusWaves == 4, "the sums below add four partials");
    if (threadIdx.x == 0) {
        atomicAdd(out + 0, (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]));
        atomicAdd(out + 1, (part[1][0] + part[1][1]) + (part[1][2] + part[1][3]));
    }
}

template <int VEC>
static hipError_t launch_part(const float *x, uint64_t pitch_elems, uint64_t ncols, int n,
                              double *out_dev, hipStream_t stream)
{
    if (ncols == 0) return hipSuccess;
    const uint32_t nvec = (uint32_t)(ncols / VEC);
    const uint32_t tiles = (nvec + 63u) / 64u;
    const uint32_t wgs = (tiles + kConsensusWaves - 1u) / kConsensusWaves;
    const uint32_t grid = wgs < kConsensusMaxGrid ? wgs : kConsensusMaxGrid;
    // streaming loads once the rows cannot stay in the 256 MiB Infinity Cache anyway
    const bool nt = (uint64_t)n * ncols * 4u >= ((uint64_t)192 << 20);
    if (nt)
        hipLaunchKernelGGL((se_consensus_kernel<VEC, true>), dim3(grid), dim3(64 * kConsensusWaves), 0, stream, x,
                           pitch_elems * 4u, nvec, tiles, n, out_dev);
    else
        hipLaunchKernelGGL((se_consensus_kernel<VEC, false>), dim3(grid), dim3(64 * kConsensusWaves), 0, stream, x,
                           pitch_elems * 4u, nvec, tiles, n, out_dev);
    return hipGetLastError();
}

// Columns [0, ncols) of n rows of pitch_elems floats: scalar head up to 16-byte alignment of
// row 0, 128-bit body, scalar tail; all three add into the same two doubles.  The other rows
// need not be 16-byte aligned (any pitch): a multi-dword global load is defined for every
// 4-byte aligned address, and the 4-column accessor promises the compiler no more than that.
hipError_t launch_consensus(const float *x, uint64_t pitch_elems, uint64_t ncols, int n,
                            double *out_dev, hipStream_t stream)
{
    hipLaunchKernelGGL(se_clear2_kernel, dim3(1), dim3(1), 0, stream, out_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || ncols == 0) return e;
    uint64_t head = (4u - ((uintptr_t)x / 4u) % 4u) % 4u;
    if (head > ncols) head = ncols;
    const uint64_t body = (ncols - head) / 4u * 4u;
    e = launch_part<1>(x, pitch_elems, head, n, out_dev, stream);
    if (e == hipSuccess) e = launch_part<4>(x + head, pitch_elems, body, n, out_dev, stream);
    if (e == hipSuccess)
        e = launch_part<1>(x + head + body, pitch_elems, ncols - head - body, n, out_dev, stream);
    return e;
}

}  // namespace se

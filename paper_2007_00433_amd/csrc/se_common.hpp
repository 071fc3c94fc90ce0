// Shared declarations of the HIP sources: kernel argument blocks and host launchers.
// gfx950 (CDNA4) only: 64-lane wavefronts are assumed throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace se {

constexpr int kMaxWorkers = 64;              // one lane per worker in the plan generator
constexpr uint32_t kLdsPerCu = 160 * 1024;   // gfx950 LDS per compute unit
constexpr int kSumBlock = 8;                 // members per block of the library's summation order

// What a step kernel computes per group (see se_step.hip for the passages).
enum Mode : int { kSesgd = 0, kGradAvg = 1, kAvgOnly = 2 };

// Arguments of the step kernels.  x, g, v point at the first column of the range the launch
// covers; rows are pitch_bytes apart; a lane owns `VEC` consecutive columns, `nvec` lane-columns
// per row in this launch, `tiles` tiles of 64 lane-columns.
struct StepArgs {
    float *x;
    const void *g;             // fp32 or bf16 bit patterns; unused in kAvgOnly
    float *v;                  // may be null (no momentum buffer)
    uint64_t seed;
    int64_t iter;
    uint64_t pitch_bytes;      // row distance of x and v in bytes (half of it for bf16 g)
    uint32_t lead;             // lane-columns at the start of the launch that are not touched (< 64)
    uint32_t nvec;             // lane-columns of the launch, the leading ones included
    uint32_t tiles;
    uint32_t coop_tiles;       // cooperative form: consecutive tiles one workgroup walks through
    int n, m, k;               // workers, rows reduced together, groups
    float neg_lr, mu, inv_m, wd;
    int mode;                  // Mode
};

// Cache policy of the row accesses: kPlain, kStream (non-temporal: the line is the first to be
// evicted), kStreamThrough (as kStream, and stores are written through the L2 to memory at
// once instead of waiting there as dirty lines: the `sc1` bit of the store).
enum Policy { kPlain = 0, kStream = 1, kStreamThrough = 2 };

struct LaunchShape {
    int vec;                // 4, 2 or 1 columns per lane
    bool bf16;              // gradient storage
    int policy;             // Policy of the row accesses
    uint32_t lds_bytes;     // dynamic LDS requested only to cap resident workgroups per CU
    int batch_rows;         // single-wavefront SESGD update: rows per batch of loads (0 = by group size)
};

// Split form: what the host decides per call.
struct SplitShape {
    float *scratch;         // library-owned device buffer of slots * chunk_tiles * 1 KiB
    uint32_t chunk_tiles;   // tiles per pair of launches
    uint32_t sub_tiles;     // tiles per sub-chunk of the finish launch
    int finish_rows;        // rows per wavefront of the finish launch: 1, 2, 4 when gradients are
                            // averaged, a multiple of 8 otherwise
    int reduce_batch;       // SESGD update: rows of a block loaded back to back in the first launch (2 or 8)
    uint32_t lds_reduce;    // dynamic LDS of the two launches, only to cap residency (0 = none)
    uint32_t lds_finish;
};

// single-wavefront form: grid (a.tiles, a.k)
hipError_t launch_step(const StepArgs &a, const LaunchShape &s, hipStream_t stream);
// cooperative form: a.m rows reduced together by ceil(a.m / 8) wavefronts per workgroup,
// grid (ceil(a.tiles / a.coop_tiles), a.k)
hipError_t launch_coop(const StepArgs &a, const LaunchShape &s, hipStream_t stream);
// split form (128-bit path only): two launches per chunk of sh.chunk_tiles tiles
hipError_t launch_split(const StepArgs &a, const LaunchShape &s, const SplitShape &sh, hipStream_t stream);
// the split form's buffer for `stream` on the current device, at least `bytes` long; null when
// none can be had (allocation failed, too many streams, or the stream is being captured)
float *split_scratch(hipStream_t stream, size_t bytes);
hipError_t launch_plan(uint64_t seed, int64_t iter, int n, int m, int32_t *group_of_dev,
                       int32_t *members_dev, hipStream_t stream);
// regrouping staged in the library's own file-scope device array (no allocation), results copied
// to host arrays of n ints; synchronous, default stream
hipError_t plan_to_host_noalloc(uint64_t seed, int64_t iter, int n, int m, int32_t *group_of_host,
                                int32_t *members_host);
hipError_t launch_consensus(const float *x, uint64_t pitch_elems, uint64_t ncols, int n,
                            double *out_dev, hipStream_t stream);
hipError_t launch_calib_copy(void *dst, const void *src, uint64_t nbytes, int policy,
                             hipStream_t stream);

// mode 1: read nbytes from src only; mode 2: write nbytes to dst only (a constant pattern)
hipError_t launch_calib_oneway(void *dst, const void *src, uint64_t nbytes, int mode, hipStream_t stream);

// Lets `kernel` request up to the whole LDS of a compute unit as dynamic shared memory; done
// once per device (bit per device ordinal in `done`).
inline hipError_t allow_full_lds(const void *kernel, std::atomic<uint64_t> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load() & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCu);
    if (e != hipSuccess) return e;
    done.fetch_or(bit);
    return hipSuccess;
}

}  // namespace se

// Shared declarations of the HIP sources: kernel argument blocks and host launchers.
// gfx950 (CDNA4) only: 64-lane wavefronts are assumed throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace se {

constexpr int kBlock = 256;        // threads per workgroup: 4 wavefronts
constexpr int kMaxWorkers = 64;    // one lane per worker in the plan generator
constexpr uint32_t kLdsPerCu = 160 * 1024;   // gfx950 LDS per compute unit

// Arguments of the fused SESGD step kernel.  Rows are `pitch` elements apart; a lane owns
// `VEC` consecutive columns, `nvec = pitch / VEC` lane-columns per row, `tiles` blocks of
// kBlock lane-columns per row.
struct StepArgs {
    float *x;
    const void *g;          // fp32 or bf16 bit patterns
    float *v;               // may be null (plain SGD)
    uint64_t seed;
    int64_t iter;
    uint64_t pitch_bytes;   // row distance of x and v in bytes
    uint32_t nvec;
    uint32_t tiles;            // tiles of `block` lane-columns per row
    uint32_t tiles_per_block;  // consecutive tiles one workgroup walks through
    uint32_t chunks;           // ceil(tiles / tiles_per_block): workgroups per group
    int n, m, k;
    float neg_lr, mu, inv_m;
    int group_major;        // block order: 1 = all chunks of a group, then the next group
};

struct RingArgs {
    float *x;
    const void *g;
    float *v;
    uint64_t pitch_bytes;
    uint32_t nvec;
    uint32_t tiles;
    int n;
    float neg_lr, mu, inv_n;
};

struct LaunchShape {
    int vec;                // 4, 2 or 1 columns per lane
    bool bf16;              // gradient storage
    int nontemporal;        // bit 0 loads, bit 1 stores
    uint32_t grid;          // workgroups
    int block;              // threads per workgroup of the step kernel: 64, 128 or 256
    uint32_t lds_bytes;     // dynamic LDS requested only to cap resident workgroups per CU
};

hipError_t launch_step(const StepArgs &a, const LaunchShape &s, hipStream_t stream);
hipError_t launch_ring(const RingArgs &a, const LaunchShape &s, hipStream_t stream);
// cooperative forms: a.m rows reduced together by ceil(a.m / 4) wavefronts per workgroup,
// a.tiles in tiles of 64 lane-columns, s.grid = a.tiles * a.k (a.k = 1 for the ring)
hipError_t launch_coop_step(const StepArgs &a, const LaunchShape &s, hipStream_t stream);
hipError_t launch_coop_ring(const StepArgs &a, const LaunchShape &s, hipStream_t stream);
hipError_t launch_plan(uint64_t seed, int64_t iter, int n, int m, int32_t *group_of_dev,
                       int32_t *members_dev, hipStream_t stream);

hipError_t launch_calib_copy(void *dst, const void *src, uint64_t nbytes, hipStream_t stream);

}  // namespace se

// Single-wavefront form of the step kernels: one 64-lane workgroup per (group, tile of 64
// lane-columns); a lane owns VEC consecutive columns of ALL member rows of its group, so the
// values to reduce never leave registers and the group mean needs no cross-lane traffic.
// A wavefront touches 64*VEC*4 contiguous bytes of each member row per access.
//
// The member list of group g is the bit mask ballot(group_of(lane) == g): iterating its set
// bits visits the members in ascending worker id; they are added up in the order the library
// documents (blocks of 8 members left to right, then the block sums left to right).  All of
// that is wave-uniform, so row bases live in scalar registers.
//
// Modes
//   kSesgd   Sec. 3.2 "Gradient Correction", the SESGD update equation; Algorithm 1 loop body:
//            local SGD/momentum step into x-hat, mean of x-hat over the group, mean written to
//            every member.
//   kGradAvg the uncorrected variant of Sec. 3.2 (the shuffle applied directly to the DSGD
//            equation): mean of the gradients over the group, then every member updates on its
//            own.  With one group of all n workers this is the Ring-SGD / DSGD step.
//   kAvgOnly mean of the parameters over the group, nothing else (Algorithm 1, last line, when
//            the group is all n workers).
#include "se_rows.hpp"

#include <atomic>

namespace se {

template <int VEC, bool BF16, bool HAS_V, bool HAS_WD, int NT, int MODE, int BMAX>
__global__ __launch_bounds__(64) void se_step_kernel(const StepArgs p)
{
    const int lane = (int)threadIdx.x;
    const uint64_t gpitch_bytes = BF16 ? p.pitch_bytes / 2 : p.pitch_bytes;
    // workgroup -> (group g = blockIdx.y, tile = blockIdx.x): all tiles of group 0 are
    // dispatched first, then group 1, ...
    const uint32_t g = blockIdx.y;
    // Regrouping for this iteration, redone by every wavefront: ~150 instructions next to
    // ~20 KiB of memory traffic.
    const uint64_t members = wave_members(p.seed, p.iter, p.n, p.m, g, lane);

    const uint32_t c = blockIdx.x * 64u + threadIdx.x;
    if (c < p.lead || c >= p.nvec) return;
    const uint32_t off = c * (uint32_t)(VEC * 4);
    const uint32_t goff = BF16 ? off / 2 : off;

    Pack<VEC> s;
#pragma unroll
    for (int q = 0; q < VEC; ++q) s.a[q] = 0.0f;
    uint64_t todo = members;

    if constexpr (MODE == kSesgd) {
#define SE_CALL(B, F, ACC) sesgd_batch<VEC, BF16, HAS_V, HAS_WD, NT, B, F>(p, todo, off, goff, gpitch_bytes, ACC)
        SE_SUM_MEMBER_BLOCKS(BMAX, p.m, VEC, s, SE_CALL);
#undef SE_CALL
    } else if constexpr (MODE == kGradAvg) {
#define SE_CALL(B, F, ACC) sum_batch<VEC, BF16, NT, false, B, F>(p, todo, goff, gpitch_bytes, ACC)
        SE_SUM_MEMBER_BLOCKS(8, p.m, VEC, s, SE_CALL);
#undef SE_CALL
    } else {
#define SE_CALL(B, F, ACC) sum_batch<VEC, false, NT, true, B, F>(p, todo, off, p.pitch_bytes, ACC)
        SE_SUM_MEMBER_BLOCKS(8, p.m, VEC, s, SE_CALL);
#undef SE_CALL
    }

    Pack<VEC> mean;
#pragma unroll
    for (int q = 0; q < VEC; ++q) mean.a[q] = s.a[q] * p.inv_m;
    todo = members;
    if constexpr (MODE == kGradAvg) {
#define SE_CALL(B, F) update_batch<VEC, HAS_V, HAS_WD, NT, B, F>(p, todo, off, mean)
        SE_FOR_MEMBER_BATCHES(BMAX, p.m, SE_CALL);
#undef SE_CALL
    } else {
        while (todo)
            store_f32<VEC, NT>((char *)p.x + next_row(todo) * p.pitch_bytes, off, mean);
    }
}

template <int VEC, bool BF16, bool HAS_V, bool HAS_WD, int NT, int MODE, int BMAX>
static hipError_t launch_one(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    auto kern = se_step_kernel<VEC, BF16, HAS_V, HAS_WD, NT, MODE, BMAX>;
    static std::atomic<uint64_t> allowed{0};
    if (s.lds_bytes > 0) {
        // the dynamic LDS is never touched: it only caps the resident workgroups per CU
        const hipError_t e = allow_full_lds((const void *)kern, allowed);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(a.tiles, (uint32_t)a.k), dim3(64), s.lds_bytes, stream, a);
    return hipGetLastError();
}

template <int VEC, bool BF16, int NT, int MODE, int BMAX>
static hipError_t launch_flags(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    const bool has_v = a.v != nullptr, has_wd = a.wd != 0.0f;
    if (has_v) return has_wd ? launch_one<VEC, BF16, true, true, NT, MODE, BMAX>(a, s, stream)
                             : launch_one<VEC, BF16, true, false, NT, MODE, BMAX>(a, s, stream);
    return has_wd ? launch_one<VEC, BF16, false, true, NT, MODE, BMAX>(a, s, stream)
                  : launch_one<VEC, BF16, false, false, NT, MODE, BMAX>(a, s, stream);
}

template <int VEC, bool BF16, int NT>
static hipError_t launch_mode(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    switch (a.mode) {
    case kSesgd: {
        // rows loaded back to back per batch (chosen by the caller from the group size)
        const int batch = s.batch_rows > 0 ? s.batch_rows : 8;
        if (batch >= 8) return launch_flags<VEC, BF16, NT, kSesgd, 8>(a, s, stream);
        if (batch >= 4) return launch_flags<VEC, BF16, NT, kSesgd, 4>(a, s, stream);
        if (batch >= 2) return launch_flags<VEC, BF16, NT, kSesgd, 2>(a, s, stream);
        return launch_flags<VEC, BF16, NT, kSesgd, 1>(a, s, stream);
    }
    case kGradAvg:
        // rows updated per batch in the second pass (the first pass adds the gradients up 8 rows at a time)
        if (s.batch_rows == 1) return launch_flags<VEC, BF16, NT, kGradAvg, 1>(a, s, stream);
        if (s.batch_rows == 2) return launch_flags<VEC, BF16, NT, kGradAvg, 2>(a, s, stream);
        return launch_flags<VEC, BF16, NT, kGradAvg, 8>(a, s, stream);
    default:
        if constexpr (BF16) return hipErrorInvalidValue;
        else return launch_one<VEC, false, false, false, NT, kAvgOnly, 8>(a, s, stream);
    }
}

template <int VEC, bool BF16>
static hipError_t launch_nt(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    switch (s.policy) {
    case kPlain: return launch_mode<VEC, BF16, kPlain>(a, s, stream);
    case kStream: return launch_mode<VEC, BF16, kStream>(a, s, stream);
    default: return launch_mode<VEC, BF16, kStreamThrough>(a, s, stream);
    }
}

hipError_t launch_step(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    if (s.bf16) {
        switch (s.vec) {
        case 4: return launch_nt<4, true>(a, s, stream);
        case 2: return launch_nt<2, true>(a, s, stream);
        default: return launch_nt<1, true>(a, s, stream);
        }
    }
    switch (s.vec) {
    case 4: return launch_nt<4, false>(a, s, stream);
    case 2: return launch_nt<2, false>(a, s, stream);
    default: return launch_nt<1, false>(a, s, stream);
    }
}

}  // namespace se

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
#include "se_device.hpp"

#include <atomic>

namespace se {

// ---- kSesgd: B members at once -------------------------------------------------------------
template <int VEC, bool BF16, bool HAS_V, bool HAS_WD, int NT, int B, bool FIRST>
__device__ __forceinline__ void sesgd_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                            uint32_t goff, uint64_t gpitch_bytes, Pack<VEC> &s)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) row[b] = next_row(todo);
    Pack<VEC> X[B], G[B], V[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        X[b] = load_f32<VEC, NT>((const char *)p.x + row[b] * p.pitch_bytes + off);
        G[b] = load_grad<VEC, BF16, NT>((const char *)p.g + row[b] * gpitch_bytes + goff);
        if constexpr (HAS_V)
            V[b] = load_f32<VEC, NT>((const char *)p.v + row[b] * p.pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        Pack<VEC> vn;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const float d = HAS_WD ? __builtin_fmaf(p.wd, X[b].a[c], G[b].a[c]) : G[b].a[c];
            vn.a[c] = HAS_V ? __builtin_fmaf(p.mu, V[b].a[c], d) : d;
            const float xhat = __builtin_fmaf(p.neg_lr, vn.a[c], X[b].a[c]);
            s.a[c] = (FIRST && b == 0) ? xhat : s.a[c] + xhat;
        }
        if constexpr (HAS_V)
            store_f32<VEC, NT>((char *)p.v + row[b] * p.pitch_bytes, off, vn);
    }
}

// ---- kGradAvg / kAvgOnly, pass 1: sum one array over B members ---------------------------------
template <int VEC, bool BF16, int NT, bool PARAMS, int B, bool FIRST>
__device__ __forceinline__ void sum_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                          uint64_t pitch_bytes, Pack<VEC> &s)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) row[b] = next_row(todo);
    Pack<VEC> A[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        if constexpr (PARAMS) A[b] = load_f32<VEC, NT>((const char *)p.x + row[b] * pitch_bytes + off);
        else A[b] = load_grad<VEC, BF16, NT>((const char *)p.g + row[b] * pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int c = 0; c < VEC; ++c)
            s.a[c] = (FIRST && b == 0) ? A[b].a[c] : s.a[c] + A[b].a[c];
}

// ---- kGradAvg, pass 2: every member updates with the group's mean gradient ---------------------
template <int VEC, bool HAS_V, bool HAS_WD, int NT, int B, bool FIRST>
__device__ __forceinline__ void update_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                             const Pack<VEC> &gbar)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) row[b] = next_row(todo);
    Pack<VEC> X[B], V[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        X[b] = load_f32<VEC, NT>((const char *)p.x + row[b] * p.pitch_bytes + off);
        if constexpr (HAS_V)
            V[b] = load_f32<VEC, NT>((const char *)p.v + row[b] * p.pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        Pack<VEC> vn, xn;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const float d = HAS_WD ? __builtin_fmaf(p.wd, X[b].a[c], gbar.a[c]) : gbar.a[c];
            vn.a[c] = HAS_V ? __builtin_fmaf(p.mu, V[b].a[c], d) : d;
            xn.a[c] = __builtin_fmaf(p.neg_lr, vn.a[c], X[b].a[c]);
        }
        if constexpr (HAS_V)
            store_f32<VEC, NT>((char *)p.v + row[b] * p.pitch_bytes, off, vn);
        store_f32<VEC, NT>((char *)p.x + row[b] * p.pitch_bytes, off, xn);
    }
}

// Applies CALL(B, FIRST) to all m members in batches of BMAX, then 4, 2, 1 (wave-uniform control
// flow throughout); FIRST is true for the first batch.  For passes that do not add anything up.
#define SE_FOR_MEMBER_BATCHES(BMAX, m, CALL)                                               \
    do {                                                                                   \
        int rem_ = (m);                                                                    \
        bool first_ = true;                                                                \
        if (rem_ >= BMAX) {                                                                \
            CALL(BMAX, true); rem_ -= BMAX; first_ = false;                                \
            while (rem_ >= BMAX) { CALL(BMAX, false); rem_ -= BMAX; }                      \
        }                                                                                  \
        if constexpr (BMAX > 4) { if (rem_ >= 4) {                                         \
            if (first_) { CALL(4, true); } else { CALL(4, false); } rem_ -= 4; first_ = false; } } \
        if constexpr (BMAX > 2) { if (rem_ >= 2) {                                         \
            if (first_) { CALL(2, true); } else { CALL(2, false); } rem_ -= 2; first_ = false; } } \
        if constexpr (BMAX > 1) { if (rem_ >= 1) {                                         \
            if (first_) { CALL(1, true); } else { CALL(1, false); } } }                    \
    } while (0)

// The library's summation order: the m members (ascending worker id) are cut into consecutive
// blocks of kSumBlock = 8, each block is added up left to right, then the block sums are added
// up left to right.  CALL(B, FIRST, acc) must add B members to acc, left to right, starting acc
// afresh when FIRST.  A full block is one batch of 8 (BMAX == 8) or two of 4; a shorter last
// block is walked in batches of 4, 2, 1.  The total lands in `total`.
constexpr int kSumBlock = 8;
#define SE_SUM_MEMBER_BLOCKS(BMAX, m, VEC_, total, CALL)                                   \
    do {                                                                                   \
        static_assert(BMAX == 8 || BMAX == 4, "batch size");                               \
        int rem_ = (m);                                                                    \
        bool first_block_ = true;                                                          \
        while (rem_ > 0) {                                                                 \
            Pack<VEC_> part_;                                                              \
            if (rem_ >= kSumBlock) {                                                       \
                if constexpr (BMAX == 8) { CALL(8, true, part_); }                         \
                else { CALL(4, true, part_); CALL(4, false, part_); }                      \
                rem_ -= kSumBlock;                                                         \
            } else {                                                                       \
                bool first_ = true;                                                        \
                if (rem_ >= 4) { CALL(4, true, part_); rem_ -= 4; first_ = false; }        \
                if (rem_ >= 2) {                                                           \
                    if (first_) { CALL(2, true, part_); } else { CALL(2, false, part_); }  \
                    rem_ -= 2; first_ = false; }                                           \
                if (rem_ >= 1) {                                                           \
                    if (first_) { CALL(1, true, part_); } else { CALL(1, false, part_); }  \
                    rem_ -= 1; }                                                           \
            }                                                                              \
            _Pragma("unroll")                                                              \
            for (int q_ = 0; q_ < VEC_; ++q_)                                              \
                total.a[q_] = first_block_ ? part_.a[q_] : total.a[q_] + part_.a[q_];      \
            first_block_ = false;                                                          \
        }                                                                                  \
    } while (0)

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
        SE_FOR_MEMBER_BATCHES(8, p.m, SE_CALL);
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
    case kSesgd:
        // deeper batches keep more rows in flight for large groups
        return a.m >= 8 ? launch_flags<VEC, BF16, NT, kSesgd, 8>(a, s, stream)
                        : launch_flags<VEC, BF16, NT, kSesgd, 4>(a, s, stream);
    case kGradAvg:
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

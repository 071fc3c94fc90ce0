// Fused SESGD step (Sec. 3.2 "Gradient Correction", the SESGD update equation;
// Algorithm 1 loop body): regroup, local SGD/momentum step into x-hat, mean of x-hat over
// the group, write the mean to every member -- one pass over the packed buffer.
//
// Work decomposition: a workgroup handles one group g and a run of consecutive tiles of
// BS lane-columns.  A lane owns VEC
// consecutive columns of ALL member rows of its group, so x-hat never leaves registers and
// the group mean needs no cross-lane traffic; a wavefront touches 64*VEC*4 contiguous
// bytes of each member row per access.  The member list of group g is the bit mask
// ballot(group_of(lane) == g): iterating its set bits visits the members in ascending
// worker id, which is the summation order the library documents.  All of that is
// wave-uniform, so row bases live in scalar registers and every row access is
// (scalar base) + (one shared 32-bit lane offset).
#include "se_device.hpp"

#include <atomic>

namespace se {

template <int VEC, bool BF16, bool HAS_V, bool NTL, bool NTS, int B>
__device__ __forceinline__ void member_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                             uint32_t goff, uint64_t gpitch_bytes,
                                             Pack<VEC> &s, bool first)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        row[b] = (uint64_t)__builtin_ctzll(todo);
        todo &= todo - 1;
    }
    Pack<VEC> X[B], G[B], V[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        X[b] = load_f32<VEC, NTL>((const char *)p.x + row[b] * p.pitch_bytes + off);
        G[b] = load_grad<VEC, BF16, NTL>((const char *)p.g + row[b] * gpitch_bytes + goff);
        if constexpr (HAS_V)
            V[b] = load_f32<VEC, NTL>((const char *)p.v + row[b] * p.pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        Pack<VEC> vn;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            vn.a[c] = HAS_V ? __builtin_fmaf(p.mu, V[b].a[c], G[b].a[c]) : G[b].a[c];
            const float xhat = __builtin_fmaf(p.neg_lr, vn.a[c], X[b].a[c]);
            s.a[c] = (first && b == 0) ? xhat : s.a[c] + xhat;
        }
        if constexpr (HAS_V)
            store_f32<VEC, NTS>((char *)p.v + row[b] * p.pitch_bytes + off, vn);
    }
}

template <int VEC, bool BF16, bool HAS_V, bool NTL, bool NTS, int BMAX, int BS>
__global__ __launch_bounds__(BS) void se_step_kernel(const StepArgs p)
{
    const int lane = (int)(threadIdx.x & 63u);
    // Regrouping for this iteration, redone by every wavefront (a few hundred integer
    // instructions, amortised over the tiles_per_block tiles the block walks through).
    const uint32_t grp = wave_group_of(p.seed, p.iter, p.n, p.m, lane);
    const uint64_t gpitch_bytes = BF16 ? p.pitch_bytes / 2 : p.pitch_bytes;

    // block -> (group g, run of consecutive tiles)
    uint32_t g, chunk;
    if (p.group_major) { g = blockIdx.x / p.chunks; chunk = blockIdx.x - g * p.chunks; }
    else               { chunk = blockIdx.x / (uint32_t)p.k; g = blockIdx.x - chunk * (uint32_t)p.k; }
    const uint64_t members = __ballot(grp == g);           // wave-uniform, m bits set
    const uint32_t tile0 = chunk * p.tiles_per_block;
    const uint32_t tile1 = min(tile0 + p.tiles_per_block, p.tiles);

    for (uint32_t tile = tile0; tile < tile1; ++tile) {
        const uint32_t c = tile * (uint32_t)BS + threadIdx.x;
        if (c >= p.nvec) break;
        const uint32_t off = c * (uint32_t)(VEC * 4);
        const uint32_t goff = BF16 ? off / 2 : off;

        Pack<VEC> s;
#pragma unroll
        for (int q = 0; q < VEC; ++q) s.a[q] = 0.0f;
        uint64_t todo = members;
        int rem = p.m;
        bool first = true;
        while (rem >= BMAX) {
            member_batch<VEC, BF16, HAS_V, NTL, NTS, BMAX>(p, todo, off, goff, gpitch_bytes, s, first);
            rem -= BMAX; first = false;
        }
        if constexpr (BMAX > 4) {
            if (rem >= 4) {
                member_batch<VEC, BF16, HAS_V, NTL, NTS, 4>(p, todo, off, goff, gpitch_bytes, s, first);
                rem -= 4; first = false;
            }
        }
        if constexpr (BMAX > 2) {
            if (rem >= 2) {
                member_batch<VEC, BF16, HAS_V, NTL, NTS, 2>(p, todo, off, goff, gpitch_bytes, s, first);
                rem -= 2; first = false;
            }
        }
        if constexpr (BMAX > 1) {
            if (rem >= 1)
                member_batch<VEC, BF16, HAS_V, NTL, NTS, 1>(p, todo, off, goff, gpitch_bytes, s, first);
        }

        Pack<VEC> mean;
#pragma unroll
        for (int q = 0; q < VEC; ++q) mean.a[q] = s.a[q] * p.inv_m;
        todo = members;
        while (todo) {
            const uint64_t row = (uint64_t)__builtin_ctzll(todo);
            todo &= todo - 1;
            store_f32<VEC, NTS>((char *)p.x + row * p.pitch_bytes + off, mean);
        }
    }
}

template <int VEC, bool BF16, bool HAS_V, int BMAX, int BS>
static hipError_t launch_bs(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    dim3 grid(s.grid), block(BS);
    const size_t lds = s.lds_bytes;
#define SE_LAUNCH(NTL, NTS)                                                                     \
    do {                                                                                        \
        auto kern = se_step_kernel<VEC, BF16, HAS_V, NTL, NTS, BMAX, BS>;                       \
        static std::atomic<bool> raised{false};                                                 \
        if (lds > 0 && !raised.load()) {                                                        \
            hipError_t e = hipFuncSetAttribute((const void *)kern,                              \
                                               hipFuncAttributeMaxDynamicSharedMemorySize,      \
                                               (int)kLdsPerCu);                                 \
            if (e != hipSuccess) return e;                                                      \
            raised.store(true);                                                                 \
        }                                                                                       \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, a);                                  \
    } while (0)
    switch (s.nontemporal & 3) {
    case 0: SE_LAUNCH(false, false); break;
    case 1: SE_LAUNCH(true, false); break;
    case 2: SE_LAUNCH(false, true); break;
    default: SE_LAUNCH(true, true); break;
    }
#undef SE_LAUNCH
    return hipGetLastError();
}

template <int VEC, bool BF16, bool HAS_V, int BMAX>
static hipError_t launch_nt(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    switch (s.block) {
    case 64: return launch_bs<VEC, BF16, HAS_V, BMAX, 64>(a, s, stream);
    case 128: return launch_bs<VEC, BF16, HAS_V, BMAX, 128>(a, s, stream);
    default: return launch_bs<VEC, BF16, HAS_V, BMAX, 256>(a, s, stream);
    }
}

template <int VEC, bool BF16>
static hipError_t launch_vec(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    const bool big = a.m >= 8;     // deeper batches keep more rows in flight for large groups
    if (a.v) return big ? launch_nt<VEC, BF16, true, 8>(a, s, stream)
                        : launch_nt<VEC, BF16, true, 4>(a, s, stream);
    return big ? launch_nt<VEC, BF16, false, 8>(a, s, stream)
               : launch_nt<VEC, BF16, false, 4>(a, s, stream);
}

hipError_t launch_step(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    if (s.bf16) {
        switch (s.vec) {
        case 4: return launch_vec<4, true>(a, s, stream);
        case 2: return launch_vec<2, true>(a, s, stream);
        default: return launch_vec<1, true>(a, s, stream);
        }
    }
    switch (s.vec) {
    case 4: return launch_vec<4, false>(a, s, stream);
    case 2: return launch_vec<2, false>(a, s, stream);
    default: return launch_vec<1, false>(a, s, stream);
    }
}

}  // namespace se

// Ring-SGD / DSGD baseline step (Sec. 3.2, the DSGD equation): what the ring all-reduce of
// Sec. 2.2 delivers to every worker is the mean gradient over all n workers; every worker
// then applies the same momentum/SGD update.  One pass: a lane sums its VEC columns of the
// n gradient rows in ascending worker id, scales by 1/n, then updates all n rows.
#include "se_device.hpp"

#include <atomic>

namespace se {

template <int VEC, bool BF16, bool HAS_V, bool NTL, bool NTS, int BS>
__global__ __launch_bounds__(BS) void se_ring_kernel(const RingArgs p)
{
    constexpr int GB = 8;     // gradient rows in flight per lane
    constexpr int UB = 4;     // parameter/momentum rows in flight per lane
    const uint64_t gpitch_bytes = BF16 ? p.pitch_bytes / 2 : p.pitch_bytes;

    for (uint32_t tile = blockIdx.x; tile < p.tiles; tile += gridDim.x) {
        const uint32_t c = tile * (uint32_t)BS + threadIdx.x;
        if (c >= p.nvec) break;
        const uint32_t off = c * (uint32_t)(VEC * 4);
        const uint32_t goff = BF16 ? off / 2 : off;

        Pack<VEC> s;
#pragma unroll
        for (int q = 0; q < VEC; ++q) s.a[q] = 0.0f;
        int i = 0;
        for (; i + GB <= p.n; i += GB) {
            Pack<VEC> G[GB];
#pragma unroll
            for (int b = 0; b < GB; ++b)
                G[b] = load_grad<VEC, BF16, NTL>((const char *)p.g + (uint64_t)(i + b) * gpitch_bytes + goff);
#pragma unroll
            for (int b = 0; b < GB; ++b)
#pragma unroll
                for (int q = 0; q < VEC; ++q)
                    s.a[q] = (i == 0 && b == 0) ? G[b].a[q] : s.a[q] + G[b].a[q];
        }
        for (; i < p.n; ++i) {
            const Pack<VEC> G = load_grad<VEC, BF16, NTL>((const char *)p.g + (uint64_t)i * gpitch_bytes + goff);
#pragma unroll
            for (int q = 0; q < VEC; ++q) s.a[q] = (i == 0) ? G.a[q] : s.a[q] + G.a[q];
        }
        Pack<VEC> gbar;
#pragma unroll
        for (int q = 0; q < VEC; ++q) gbar.a[q] = s.a[q] * p.inv_n;

        i = 0;
        for (; i + UB <= p.n; i += UB) {
            Pack<VEC> X[UB], V[UB];
#pragma unroll
            for (int b = 0; b < UB; ++b) {
                X[b] = load_f32<VEC, NTL>((const char *)p.x + (uint64_t)(i + b) * p.pitch_bytes + off);
                if constexpr (HAS_V)
                    V[b] = load_f32<VEC, NTL>((const char *)p.v + (uint64_t)(i + b) * p.pitch_bytes + off);
            }
#pragma unroll
            for (int b = 0; b < UB; ++b) {
                Pack<VEC> vn, xn;
#pragma unroll
                for (int q = 0; q < VEC; ++q) {
                    vn.a[q] = HAS_V ? __builtin_fmaf(p.mu, V[b].a[q], gbar.a[q]) : gbar.a[q];
                    xn.a[q] = __builtin_fmaf(p.neg_lr, vn.a[q], X[b].a[q]);
                }
                if constexpr (HAS_V)
                    store_f32<VEC, NTS>((char *)p.v + (uint64_t)(i + b) * p.pitch_bytes + off, vn);
                store_f32<VEC, NTS>((char *)p.x + (uint64_t)(i + b) * p.pitch_bytes + off, xn);
            }
        }
        for (; i < p.n; ++i) {
            const Pack<VEC> X = load_f32<VEC, NTL>((const char *)p.x + (uint64_t)i * p.pitch_bytes + off);
            Pack<VEC> V, vn, xn;
            if constexpr (HAS_V)
                V = load_f32<VEC, NTL>((const char *)p.v + (uint64_t)i * p.pitch_bytes + off);
#pragma unroll
            for (int q = 0; q < VEC; ++q) {
                vn.a[q] = HAS_V ? __builtin_fmaf(p.mu, V.a[q], gbar.a[q]) : gbar.a[q];
                xn.a[q] = __builtin_fmaf(p.neg_lr, vn.a[q], X.a[q]);
            }
            if constexpr (HAS_V)
                store_f32<VEC, NTS>((char *)p.v + (uint64_t)i * p.pitch_bytes + off, vn);
            store_f32<VEC, NTS>((char *)p.x + (uint64_t)i * p.pitch_bytes + off, xn);
        }
    }
}

template <int VEC, bool BF16, bool HAS_V, int BS>
static hipError_t launch_bs(const RingArgs &a, const LaunchShape &s, hipStream_t stream)
{
    dim3 grid(s.grid), block(BS);
    const size_t lds = s.lds_bytes;
#define SE_LAUNCH(NTL, NTS)                                                                     \
    do {                                                                                        \
        auto kern = se_ring_kernel<VEC, BF16, HAS_V, NTL, NTS, BS>;                             \
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

template <int VEC, bool BF16, bool HAS_V>
static hipError_t launch_nt(const RingArgs &a, const LaunchShape &s, hipStream_t stream)
{
    switch (s.block) {
    case 64: return launch_bs<VEC, BF16, HAS_V, 64>(a, s, stream);
    case 128: return launch_bs<VEC, BF16, HAS_V, 128>(a, s, stream);
    default: return launch_bs<VEC, BF16, HAS_V, 256>(a, s, stream);
    }
}

template <int VEC, bool BF16>
static hipError_t launch_vec(const RingArgs &a, const LaunchShape &s, hipStream_t stream)
{
    return a.v ? launch_nt<VEC, BF16, true>(a, s, stream) : launch_nt<VEC, BF16, false>(a, s, stream);
}

hipError_t launch_ring(const RingArgs &a, const LaunchShape &s, hipStream_t stream)
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

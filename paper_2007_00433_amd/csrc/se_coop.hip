// Cooperative form of the two steps for many rows per reduction (large groups, and the
// Ring-SGD baseline where all n rows are reduced): the rows of one reduction are split over
// the wavefronts of a workgroup, kRowsPerWave rows each, all wavefronts covering the same 64
// lane-columns.  Every lane issues all loads of its rows at once (one round trip to HBM),
// stages the values to be reduced in LDS, and after one barrier every wavefront walks the
// staged rows in ascending worker id -- the documented summation order, so the result is
// bit-identical to the single-wavefront kernel -- and finishes its own rows.
//
//   SESGD (Sec. 3.2, the SESGD update equation): stage x-hat, mean -> stored to own rows.
//   Ring-SGD (Sec. 3.2, the DSGD equation): stage g, mean gradient -> momentum/SGD update of
//   own rows (their x and v were loaded together with g).
#include "se_device.hpp"

#include <atomic>

namespace se {

constexpr int kRowsPerWave = 4;

template <int VEC, bool BF16, bool HAS_V, bool NTL, bool NTS, bool RING>
__global__ __launch_bounds__(1024) void se_coop_kernel(const StepArgs p)
{
    extern __shared__ float staged[];          // [rows][64 lanes][VEC]
    const int lane = (int)(threadIdx.x & 63u);
    const int wave = (int)(threadIdx.x >> 6);
    const uint64_t gpitch_bytes = BF16 ? p.pitch_bytes / 2 : p.pitch_bytes;

    uint32_t g, tile;
    uint64_t members;
    if constexpr (RING) {
        tile = blockIdx.x;
        members = p.n >= 64 ? ~0ull : ((1ull << p.n) - 1ull);
    } else {
        const uint32_t grp = wave_group_of(p.seed, p.iter, p.n, p.m, lane);
        if (p.group_major) { g = blockIdx.x / p.tiles; tile = blockIdx.x - g * p.tiles; }
        else               { tile = blockIdx.x / (uint32_t)p.k; g = blockIdx.x - tile * (uint32_t)p.k; }
        members = __ballot(grp == g);
    }
    const uint32_t c = tile * 64u + (uint32_t)lane;
    const bool valid = c < p.nvec;
    const uint32_t off = c * (uint32_t)(VEC * 4);
    const uint32_t goff = BF16 ? off / 2 : off;

    // this wavefront's rows: members number wave*kRowsPerWave .. +kRowsPerWave-1
    const int first = wave * kRowsPerWave;
    const int mine = min(kRowsPerWave, p.m - first);      // >= 1 by construction of the block
    uint64_t todo = members;
    for (int q = 0; q < first; ++q) todo &= todo - 1;
    uint64_t row[kRowsPerWave];
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        row[r] = todo ? (uint64_t)__builtin_ctzll(todo) : 0;
        todo &= todo - 1;
    }

    Pack<VEC> X[kRowsPerWave], G[kRowsPerWave], V[kRowsPerWave];
    if (valid) {
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            if (r < mine) {
                X[r] = load_f32<VEC, NTL>((const char *)p.x + row[r] * p.pitch_bytes + off);
                G[r] = load_grad<VEC, BF16, NTL>((const char *)p.g + row[r] * gpitch_bytes + goff);
                if constexpr (HAS_V)
                    V[r] = load_f32<VEC, NTL>((const char *)p.v + row[r] * p.pitch_bytes + off);
            }
        }
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            if (r < mine) {
                Pack<VEC> out;
                if constexpr (RING) {
                    out = G[r];
                } else {
                    Pack<VEC> vn;
#pragma unroll
                    for (int q = 0; q < VEC; ++q) {
                        vn.a[q] = HAS_V ? __builtin_fmaf(p.mu, V[r].a[q], G[r].a[q]) : G[r].a[q];
                        out.a[q] = __builtin_fmaf(p.neg_lr, vn.a[q], X[r].a[q]);
                    }
                    if constexpr (HAS_V)
                        store_f32<VEC, NTS>((char *)p.v + row[r] * p.pitch_bytes + off, vn);
                }
                store_f32<VEC, false>((char *)(staged + ((size_t)(first + r) * 64 + lane) * VEC), out);
            }
        }
    }
    __syncthreads();
    if (!valid) return;

    Pack<VEC> s = load_f32<VEC, false>((const char *)(staged + (size_t)lane * VEC));
    for (int r = 1; r < p.m; ++r) {
        const Pack<VEC> t = load_f32<VEC, false>((const char *)(staged + ((size_t)r * 64 + lane) * VEC));
#pragma unroll
        for (int q = 0; q < VEC; ++q) s.a[q] = s.a[q] + t.a[q];
    }
    Pack<VEC> mean;
#pragma unroll
    for (int q = 0; q < VEC; ++q) mean.a[q] = s.a[q] * p.inv_m;

#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        if (r < mine) {
            if constexpr (RING) {
                Pack<VEC> vn, xn;
#pragma unroll
                for (int q = 0; q < VEC; ++q) {
                    vn.a[q] = HAS_V ? __builtin_fmaf(p.mu, V[r].a[q], mean.a[q]) : mean.a[q];
                    xn.a[q] = __builtin_fmaf(p.neg_lr, vn.a[q], X[r].a[q]);
                }
                if constexpr (HAS_V)
                    store_f32<VEC, NTS>((char *)p.v + row[r] * p.pitch_bytes + off, vn);
                store_f32<VEC, NTS>((char *)p.x + row[r] * p.pitch_bytes + off, xn);
            } else {
                store_f32<VEC, NTS>((char *)p.x + row[r] * p.pitch_bytes + off, mean);
            }
        }
    }
}

template <int VEC, bool BF16, bool HAS_V, bool RING>
static hipError_t launch_nt(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    const int waves = (a.m + kRowsPerWave - 1) / kRowsPerWave;
    dim3 grid(s.grid), block(waves * 64);
    const size_t need = (size_t)a.m * 64 * VEC * sizeof(float);
    const size_t lds = need > s.lds_bytes ? need : s.lds_bytes;
#define SE_LAUNCH(NTL, NTS)                                                                     \
    do {                                                                                        \
        auto kern = se_coop_kernel<VEC, BF16, HAS_V, NTL, NTS, RING>;                           \
        static std::atomic<bool> raised{false};                                                 \
        if (!raised.load()) {                                                                   \
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

template <int VEC, bool BF16, bool RING>
static hipError_t launch_vec(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    return a.v ? launch_nt<VEC, BF16, true, RING>(a, s, stream)
               : launch_nt<VEC, BF16, false, RING>(a, s, stream);
}

template <bool RING>
static hipError_t launch_any(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    if (s.bf16) {
        switch (s.vec) {
        case 4: return launch_vec<4, true, RING>(a, s, stream);
        case 2: return launch_vec<2, true, RING>(a, s, stream);
        default: return launch_vec<1, true, RING>(a, s, stream);
        }
    }
    switch (s.vec) {
    case 4: return launch_vec<4, false, RING>(a, s, stream);
    case 2: return launch_vec<2, false, RING>(a, s, stream);
    default: return launch_vec<1, false, RING>(a, s, stream);
    }
}

// a.m rows are reduced together: the group size for SESGD, n for the ring baseline;
// a.tiles counts tiles of 64 lane-columns; s.grid = tiles * (groups or 1).
hipError_t launch_coop_step(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    return launch_any<false>(a, s, stream);
}

hipError_t launch_coop_ring(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    return launch_any<true>(a, s, stream);
}

}  // namespace se

// Cooperative form of the step kernels for many rows per reduction (large groups, and the
// Ring-SGD baseline where all n rows are reduced).  The library adds a group's values up in
// blocks of 8 members (ascending worker id, left to right) and then adds the block sums left to
// right; here every wavefront of a workgroup owns one such block: it issues all loads of its 8
// rows at once (one round trip to HBM), adds its block up in registers, stages the ONE block sum
// in LDS (1 KiB per wavefront), and after one barrier every wavefront adds the staged block sums
// in order -- the same tree, hence the same bits, as the single-wavefront form -- and finishes
// its own 8 rows.  A wavefront thus reads and writes 8 rows only, and a workgroup of ceil(m/8)
// wavefronts covers the same 64 lane-columns of all m rows.
//
//   kSesgd   (Sec. 3.2, the SESGD update equation): block sums of x-hat; mean -> own rows.
//   kGradAvg (Sec. 3.2, the DSGD equation applied per group; Ring-SGD when the group is all n
//            workers): block sums of g; mean gradient -> momentum/SGD update of own rows, whose
//            x and v were loaded together with g.
//   kAvgOnly (Algorithm 1, last line): block sums of x; mean -> own rows.
#include "se_device.hpp"

#include <atomic>

namespace se {

constexpr int kRowsPerWave = kSumBlock;   // one block of the summation order per wavefront

template <int VEC, bool BF16, bool HAS_V, bool HAS_WD, int NT, int MODE>
__global__ __launch_bounds__(64 * ((kMaxWorkers + kRowsPerWave - 1) / kRowsPerWave))
void se_coop_kernel(const StepArgs p)
{
    extern __shared__ float staged[];          // [wavefronts][VEC][64 lanes]: one block sum each
    const int lane = (int)(threadIdx.x & 63u);
    const int wave = (int)(threadIdx.x >> 6);
    const int blocks = (p.m + kRowsPerWave - 1) / kRowsPerWave;     // = wavefronts of the workgroup
    const uint64_t gpitch_bytes = BF16 ? p.pitch_bytes / 2 : p.pitch_bytes;

    const uint32_t g = blockIdx.y;
    const uint64_t members = wave_members(p.seed, p.iter, p.n, p.m, g, lane);

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

    // A workgroup walks through coop_tiles consecutive tiles.
    const uint32_t tile_end = min((blockIdx.x + 1u) * p.coop_tiles, p.tiles);
    for (uint32_t tile = blockIdx.x * p.coop_tiles; tile < tile_end; ++tile) {
        const uint32_t c = tile * 64u + (uint32_t)lane;
        const bool valid = c >= p.lead && c < p.nvec;
        const uint32_t off = c * (uint32_t)(VEC * 4);
        const uint32_t goff = BF16 ? off / 2 : off;

        Pack<VEC> X[kRowsPerWave], G[kRowsPerWave], V[kRowsPerWave];
        if (valid) {
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                if (r < mine) {
                    X[r] = load_f32<VEC, NT>((const char *)p.x + row[r] * p.pitch_bytes + off);
                    if constexpr (MODE != kAvgOnly) {
                        G[r] = load_grad<VEC, BF16, NT>((const char *)p.g + row[r] * gpitch_bytes + goff);
                        if constexpr (HAS_V)
                            V[r] = load_f32<VEC, NT>((const char *)p.v + row[r] * p.pitch_bytes + off);
                    }
                }
            }
            Pack<VEC> part;                    // this block's sum, members left to right
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                if (r < mine) {
                    Pack<VEC> out;
                    if constexpr (MODE == kGradAvg) {
                        out = G[r];
                    } else if constexpr (MODE == kAvgOnly) {
                        out = X[r];
                    } else {
                        Pack<VEC> vn;
#pragma unroll
                        for (int q = 0; q < VEC; ++q) {
                            const float d = HAS_WD ? __builtin_fmaf(p.wd, X[r].a[q], G[r].a[q]) : G[r].a[q];
                            vn.a[q] = HAS_V ? __builtin_fmaf(p.mu, V[r].a[q], d) : d;
                            out.a[q] = __builtin_fmaf(p.neg_lr, vn.a[q], X[r].a[q]);
                        }
                        if constexpr (HAS_V)
                            store_f32<VEC, NT>((char *)p.v + row[r] * p.pitch_bytes, off, vn);
                    }
#pragma unroll
                    for (int q = 0; q < VEC; ++q) part.a[q] = r == 0 ? out.a[q] : part.a[q] + out.a[q];
                }
            }
#pragma unroll
            for (int q = 0; q < VEC; ++q) staged[((size_t)wave * VEC + q) * 64 + lane] = part.a[q];
        }
        __syncthreads();
        if (valid) {
            Pack<VEC> s;
#pragma unroll
            for (int q = 0; q < VEC; ++q) s.a[q] = staged[(size_t)q * 64 + lane];
            for (int b = 1; b < blocks; ++b) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) s.a[q] = s.a[q] + staged[((size_t)b * VEC + q) * 64 + lane];
            }
            Pack<VEC> mean;
#pragma unroll
            for (int q = 0; q < VEC; ++q) mean.a[q] = s.a[q] * p.inv_m;

#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                if (r < mine) {
                    if constexpr (MODE == kGradAvg) {
                        Pack<VEC> vn, xn;
#pragma unroll
                        for (int q = 0; q < VEC; ++q) {
                            const float d = HAS_WD ? __builtin_fmaf(p.wd, X[r].a[q], mean.a[q]) : mean.a[q];
                            vn.a[q] = HAS_V ? __builtin_fmaf(p.mu, V[r].a[q], d) : d;
                            xn.a[q] = __builtin_fmaf(p.neg_lr, vn.a[q], X[r].a[q]);
                        }
                        if constexpr (HAS_V)
                            store_f32<VEC, NT>((char *)p.v + row[r] * p.pitch_bytes, off, vn);
                        store_f32<VEC, NT>((char *)p.x + row[r] * p.pitch_bytes, off, xn);
                    } else {
                        store_f32<VEC, NT>((char *)p.x + row[r] * p.pitch_bytes, off, mean);
                    }
                }
            }
        }
        // the staging area is rewritten by the next tile (uniform: every thread of the
        // workgroup runs the same number of tiles)
        if (tile + 1 < tile_end) __syncthreads();
    }
}

template <int VEC, bool BF16, bool HAS_V, bool HAS_WD, int NT, int MODE>
static hipError_t launch_one(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    const int waves = (a.m + kRowsPerWave - 1) / kRowsPerWave;     // <= 8 for m <= 64
    const size_t need = (size_t)waves * 64 * VEC * sizeof(float);  // <= 8 KiB
    const size_t lds = need > s.lds_bytes ? need : s.lds_bytes;
    auto kern = se_coop_kernel<VEC, BF16, HAS_V, HAS_WD, NT, MODE>;
    static std::atomic<uint64_t> allowed{0};
    const hipError_t e = allow_full_lds((const void *)kern, allowed);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((a.tiles + a.coop_tiles - 1) / a.coop_tiles, (uint32_t)a.k),
                       dim3(waves * 64), lds, stream, a);
    return hipGetLastError();
}

template <int VEC, bool BF16, int NT, int MODE>
static hipError_t launch_flags(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    const bool has_v = a.v != nullptr, has_wd = a.wd != 0.0f;
    if (has_v) return has_wd ? launch_one<VEC, BF16, true, true, NT, MODE>(a, s, stream)
                             : launch_one<VEC, BF16, true, false, NT, MODE>(a, s, stream);
    return has_wd ? launch_one<VEC, BF16, false, true, NT, MODE>(a, s, stream)
                  : launch_one<VEC, BF16, false, false, NT, MODE>(a, s, stream);
}

template <int VEC, bool BF16, int NT>
static hipError_t launch_mode(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
{
    switch (a.mode) {
    case kSesgd: return launch_flags<VEC, BF16, NT, kSesgd>(a, s, stream);
    case kGradAvg: return launch_flags<VEC, BF16, NT, kGradAvg>(a, s, stream);
    default:
        if constexpr (BF16) return hipErrorInvalidValue;
        else return launch_one<VEC, false, false, false, NT, kAvgOnly>(a, s, stream);
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

hipError_t launch_coop(const StepArgs &a, const LaunchShape &s, hipStream_t stream)
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

// Split form of the step kernels for reductions over many rows (groups of more than 8 workers,
// and the Ring-SGD baseline, which reduces all n rows).  A wavefront that owns all rows of a
// large group keeps dozens of row streams open at once; here no wavefront touches more than 8
// rows, and the launch order keeps the rows that are live on the chip at any moment few.  The
// work on a chunk of columns is cut into two launches that hand a small intermediate over
// through a library-owned device buffer (it is written and read back while still in the caches):
//
//   reduce   kGradAvg (Sec. 3.2, the DSGD equation; Ring-SGD when the group is all n workers):
//            one wavefront per (tile, group) adds the group's gradients up -- blocks of 8
//            members left to right, then the block sums left to right, the library's order --
//            and stores the mean gradient.
//            kAvgOnly (Algorithm 1, last line): the same over the group's parameters; the mean
//            parameters are stored.
//            kSesgd (Sec. 3.2, the SESGD update equation): one wavefront per (tile, group, block
//            of 8 members) does the local momentum/SGD step of its 8 rows, stores v, and stores
//            the block's sum of x-hat.
//   finish   kGradAvg: one wavefront per (tile, worker) updates that worker's v and x with the
//            stored mean gradient.  kAvgOnly: one wavefront per (tile, a few workers) writes the
//            stored mean into those workers' rows.
//            kSesgd: one wavefront per (tile, group, block) adds the group's stored block sums
//            left to right, scales by 1/m and writes the mean to its 8 rows.
//
// The finish launch walks its work in sub-chunks of `sub_tiles` tiles: all tiles of a sub-chunk
// for one worker (or block), then the same tiles for the next, so that the intermediate of a
// sub-chunk is re-read from cache while only a handful of rows are being streamed.  Results are
// bit-identical to the other two forms: same operations, same order.
#include "se_rows.hpp"

#include <atomic>
#include <mutex>

namespace se {

struct SplitArgs {
    StepArgs a;
    float *scratch;          // [slots][chunk_pitch] fp32; slot = group, or group * nb + block in kSesgd
    uint32_t tile0;          // first tile of this chunk (tiles are counted as in `a`)
    uint32_t tiles_c;        // tiles of this chunk
    uint32_t sub_tiles;      // tiles per sub-chunk of the finish launch
    uint32_t chunk_pitch;    // floats per slot
    int nb;                  // blocks of 8 members per group
    int finish_rows;         // rows one wavefront of the finish launch handles: 1, 2, 4 (kGradAvg) or
                             // a multiple of 8 (other modes)
    int finish_units;        // wavefronts per group and tile of the finish launch
};

constexpr int kVec = 4;      // the split form exists for the 128-bit path only

// members of `mask` from number `skip` on (ascending worker id)
__device__ __forceinline__ uint64_t skip_members(uint64_t mask, int skip)
{
    for (int q = 0; q < skip; ++q) mask &= mask - 1;
    return mask;
}

template <bool BF16, bool HAS_V, bool HAS_WD, int NT, int MODE, int BMAX>
__global__ __launch_bounds__(64) void se_split_reduce_kernel(const SplitArgs q)
{
    const StepArgs &p = q.a;
    const int lane = (int)threadIdx.x;
    const uint64_t gpitch_bytes = BF16 ? p.pitch_bytes / 2 : p.pitch_bytes;
    const uint32_t slot = blockIdx.y;
    constexpr bool kWholeGroup = MODE != kSesgd;          // one wavefront adds the whole group up
    const uint32_t g = kWholeGroup ? slot : slot / (uint32_t)q.nb;
    const int b = kWholeGroup ? 0 : (int)(slot - g * (uint32_t)q.nb);
    const uint64_t members = wave_members(p.seed, p.iter, p.n, p.m, g, lane);

    const uint32_t c = (q.tile0 + blockIdx.x) * 64u + threadIdx.x;
    if (c < p.lead || c >= p.nvec) return;
    const uint32_t off = c * (uint32_t)(kVec * 4);
    const uint32_t goff = BF16 ? off / 2 : off;

    Pack<kVec> s;
#pragma unroll
    for (int i = 0; i < kVec; ++i) s.a[i] = 0.0f;
    if constexpr (MODE == kGradAvg) {
        uint64_t todo = members;
#define SE_CALL(B, F, ACC) sum_batch<kVec, BF16, NT, false, B, F>(p, todo, goff, gpitch_bytes, ACC)
        SE_SUM_MEMBER_BLOCKS(8, p.m, kVec, s, SE_CALL);
#undef SE_CALL
#pragma unroll
        for (int i = 0; i < kVec; ++i) s.a[i] = s.a[i] * p.inv_m;
    } else if constexpr (MODE == kAvgOnly) {
        uint64_t todo = members;
#define SE_CALL(B, F, ACC) sum_batch<kVec, false, NT, true, B, F>(p, todo, off, p.pitch_bytes, ACC)
        SE_SUM_MEMBER_BLOCKS(8, p.m, kVec, s, SE_CALL);
#undef SE_CALL
#pragma unroll
        for (int i = 0; i < kVec; ++i) s.a[i] = s.a[i] * p.inv_m;
    } else {
        uint64_t todo = skip_members(members, b * kSumBlock);
        const int count = min(kSumBlock, p.m - b * kSumBlock);           // one block: a single partial
#define SE_CALL(B, F, ACC) sesgd_batch<kVec, BF16, HAS_V, HAS_WD, NT, B, F>(p, todo, off, goff, gpitch_bytes, ACC)
        SE_SUM_MEMBER_BLOCKS(BMAX, count, kVec, s, SE_CALL);
#undef SE_CALL
    }
    // plain store: the value is wanted again soon, from cache
    float *dst = q.scratch + (size_t)slot * q.chunk_pitch + ((size_t)blockIdx.x * 64u + threadIdx.x) * kVec;
    store_f32<kVec, kPlain>((char *)dst, 0u, s);
}

template <bool HAS_V, bool HAS_WD, int NT, int MODE>
__global__ __launch_bounds__(64) void se_split_finish_kernel(const SplitArgs q)
{
    const StepArgs &p = q.a;
    const int lane = (int)threadIdx.x;
    // work order: (sub-chunk, unit, tile inside the sub-chunk); a unit is `finish_rows`
    // consecutive members of one group
    const uint32_t units = (uint32_t)(p.k * q.finish_units);
    const uint32_t per_sub = units * q.sub_tiles;
    const uint32_t sub = blockIdx.x / per_sub;
    const uint32_t rem = blockIdx.x - sub * per_sub;
    const uint32_t unit = rem / q.sub_tiles;
    const uint32_t t = sub * q.sub_tiles + (rem - unit * q.sub_tiles);   // tile inside the chunk
    if (t >= q.tiles_c) return;
    const uint32_t g = unit / (uint32_t)q.finish_units;
    const int r0 = (int)(unit - g * (uint32_t)q.finish_units) * q.finish_rows;   // first member of the unit
    const int count = min(q.finish_rows, p.m - r0);
    const uint64_t members = wave_members(p.seed, p.iter, p.n, p.m, g, lane);
    const uint32_t c = (q.tile0 + t) * 64u + threadIdx.x;
    if (c < p.lead || c >= p.nvec) return;
    const uint32_t off = c * (uint32_t)(kVec * 4);
    const size_t scol = ((size_t)t * 64u + threadIdx.x) * kVec;
    uint64_t todo = skip_members(members, r0);

    if constexpr (MODE == kGradAvg) {
        const Pack<kVec> gbar = load_f32<kVec, kPlain>((const char *)(q.scratch + (size_t)g * q.chunk_pitch + scol));
#define SE_CALL(B, F) update_batch<kVec, HAS_V, HAS_WD, NT, B, F>(p, todo, off, gbar)
        SE_FOR_MEMBER_BATCHES(4, count, SE_CALL);
#undef SE_CALL
    } else if constexpr (MODE == kAvgOnly) {
        const Pack<kVec> mean = load_f32<kVec, kPlain>((const char *)(q.scratch + (size_t)g * q.chunk_pitch + scol));
        for (int i = 0; i < count; ++i)
            store_f32<kVec, NT>((char *)p.x + next_row(todo) * p.pitch_bytes, off, mean);
    } else {
        const float *part = q.scratch + (size_t)g * q.nb * q.chunk_pitch + scol;
        Pack<kVec> s = load_f32<kVec, kPlain>((const char *)part);
        for (int bb = 1; bb < q.nb; ++bb) {
            const Pack<kVec> u = load_f32<kVec, kPlain>((const char *)(part + (size_t)bb * q.chunk_pitch));
#pragma unroll
            for (int i = 0; i < kVec; ++i) s.a[i] = s.a[i] + u.a[i];
        }
        Pack<kVec> mean;
#pragma unroll
        for (int i = 0; i < kVec; ++i) mean.a[i] = s.a[i] * p.inv_m;
        for (int i = 0; i < count; ++i)
            store_f32<kVec, NT>((char *)p.x + next_row(todo) * p.pitch_bytes, off, mean);
    }
}

// ---- scratch: one buffer per (device, stream), grown on demand, kept until the process ends --
// Launches on one stream are ordered, so a buffer tied to the stream is never used by two steps
// at once; steps on different streams get different buffers.
namespace {
struct Slot { int dev; hipStream_t stream; float *ptr; size_t bytes; };
constexpr int kSlots = 16;
Slot g_slots[kSlots];
int g_nslots = 0;
std::mutex g_slot_mutex;
}  // namespace

float *split_scratch(hipStream_t stream, size_t bytes)
{
    // Never while the stream is being captured into a graph: an allocation is not allowed then,
    // and a buffer tied to the capturing stream would not be tied to the graph's replays.  The
    // caller records the one-launch form instead.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return nullptr;
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    std::lock_guard<std::mutex> lock(g_slot_mutex);
    Slot *slot = nullptr;
    for (int i = 0; i < g_nslots; ++i)
        if (g_slots[i].dev == dev && g_slots[i].stream == stream) slot = &g_slots[i];
    if (slot && slot->bytes >= bytes) return slot->ptr;
    if (!slot) {
        if (g_nslots == kSlots) return nullptr;
        slot = &g_slots[g_nslots];
        *slot = Slot{dev, stream, nullptr, 0};
    }
    float *fresh = nullptr;
    if (hipMalloc((void **)&fresh, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (slot->ptr) {
        // the old buffer may still be read by launches in flight on this stream
        if (hipStreamSynchronize(stream) != hipSuccess || hipFree(slot->ptr) != hipSuccess) (void)hipGetLastError();
    }
    slot->ptr = fresh;
    slot->bytes = bytes;
    if (slot == &g_slots[g_nslots]) ++g_nslots;
    return fresh;
}

template <typename K> static hipError_t cap_residency(K kern, std::atomic<uint64_t> &allowed, uint32_t lds)
{
    return lds > 0 ? allow_full_lds((const void *)kern, allowed) : hipSuccess;
}

template <bool BF16, bool HAS_V, bool HAS_WD, int NT, int MODE, int BMAX>
static hipError_t launch_chunks(const StepArgs &a, const SplitShape &sh, hipStream_t stream)
{
    auto reduce = se_split_reduce_kernel<BF16, HAS_V, HAS_WD, NT, MODE, BMAX>;
    auto finish = se_split_finish_kernel<HAS_V, HAS_WD, NT, MODE>;
    static std::atomic<uint64_t> allowed_r{0}, allowed_f{0};
    hipError_t e = cap_residency(reduce, allowed_r, sh.lds_reduce);
    if (e == hipSuccess) e = cap_residency(finish, allowed_f, sh.lds_finish);
    if (e != hipSuccess) return e;

    SplitArgs q;
    q.a = a;
    q.scratch = sh.scratch;
    q.nb = (a.m + kSumBlock - 1) / kSumBlock;
    q.sub_tiles = sh.sub_tiles;
    const uint32_t slots = MODE == kSesgd ? (uint32_t)(a.k * q.nb) : (uint32_t)a.k;
    q.finish_rows = sh.finish_rows;
    q.finish_units = (a.m + sh.finish_rows - 1) / sh.finish_rows;
    const uint32_t units = (uint32_t)(a.k * q.finish_units);
    q.chunk_pitch = sh.chunk_tiles * 64u * kVec;
    for (uint32_t tile0 = 0; tile0 < a.tiles; tile0 += sh.chunk_tiles) {
        q.tile0 = tile0;
        q.tiles_c = a.tiles - tile0 < sh.chunk_tiles ? a.tiles - tile0 : sh.chunk_tiles;
        hipLaunchKernelGGL(reduce, dim3(q.tiles_c, slots), dim3(64), sh.lds_reduce, stream, q);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        const uint32_t subs = (q.tiles_c + q.sub_tiles - 1) / q.sub_tiles;
        hipLaunchKernelGGL(finish, dim3(subs * units * q.sub_tiles), dim3(64), sh.lds_finish, stream, q);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <bool BF16, int NT, int MODE>
static hipError_t launch_flags(const StepArgs &a, const SplitShape &sh, hipStream_t stream)
{
    const bool has_v = a.v != nullptr, has_wd = a.wd != 0.0f;
    if constexpr (MODE == kSesgd) {
        // rows of a block whose loads are issued back to back in the first launch
        if (sh.reduce_batch < 2) {
            if (has_v) return has_wd ? launch_chunks<BF16, true, true, NT, MODE, 1>(a, sh, stream)
                                     : launch_chunks<BF16, true, false, NT, MODE, 1>(a, sh, stream);
            return has_wd ? launch_chunks<BF16, false, true, NT, MODE, 1>(a, sh, stream)
                          : launch_chunks<BF16, false, false, NT, MODE, 1>(a, sh, stream);
        }
        if (sh.reduce_batch < 8) {
            if (has_v) return has_wd ? launch_chunks<BF16, true, true, NT, MODE, 2>(a, sh, stream)
                                     : launch_chunks<BF16, true, false, NT, MODE, 2>(a, sh, stream);
            return has_wd ? launch_chunks<BF16, false, true, NT, MODE, 2>(a, sh, stream)
                          : launch_chunks<BF16, false, false, NT, MODE, 2>(a, sh, stream);
        }
    }
    if (has_v) return has_wd ? launch_chunks<BF16, true, true, NT, MODE, 8>(a, sh, stream)
                             : launch_chunks<BF16, true, false, NT, MODE, 8>(a, sh, stream);
    return has_wd ? launch_chunks<BF16, false, true, NT, MODE, 8>(a, sh, stream)
                  : launch_chunks<BF16, false, false, NT, MODE, 8>(a, sh, stream);
}

template <bool BF16, int NT>
static hipError_t launch_mode(const StepArgs &a, const SplitShape &sh, hipStream_t stream)
{
    switch (a.mode) {
    case kSesgd: return launch_flags<BF16, NT, kSesgd>(a, sh, stream);
    case kGradAvg: return launch_flags<BF16, NT, kGradAvg>(a, sh, stream);
    default:
        if constexpr (BF16) return hipErrorInvalidValue;
        else return launch_chunks<false, false, false, NT, kAvgOnly, 8>(a, sh, stream);
    }
}

hipError_t launch_split(const StepArgs &a, const LaunchShape &s, const SplitShape &sh, hipStream_t stream)
{
    if (s.vec != kVec || !sh.scratch || sh.chunk_tiles == 0 || sh.sub_tiles == 0) return hipErrorInvalidValue;
    const int fr = sh.finish_rows;
    if (a.mode == kSesgd ? (fr < kSumBlock || fr % kSumBlock != 0) : a.mode == kGradAvg ? (fr != 1 && fr != 2 && fr != 4) : (fr < 1 || fr > kMaxWorkers))
        return hipErrorInvalidValue;
    if (s.bf16) {
        switch (s.policy) {
        case kPlain: return launch_mode<true, kPlain>(a, sh, stream);
        case kStream: return launch_mode<true, kStream>(a, sh, stream);
        default: return launch_mode<true, kStreamThrough>(a, sh, stream);
        }
    }
    switch (s.policy) {
    case kPlain: return launch_mode<false, kPlain>(a, sh, stream);
    case kStream: return launch_mode<false, kStream>(a, sh, stream);
    default: return launch_mode<false, kStreamThrough>(a, sh, stream);
    }
}

}  // namespace se

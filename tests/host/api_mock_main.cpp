// Host-only harness for the C ABI: se_api.cpp is linked against mock launchers that never
// touch a device but check, for every launch the API would make, that the argument block is
// consistent with what the kernels assume (alignment of every row at the first column, column
// count, tile and grid arithmetic), and record which columns each launch covers.  main() then
// drives the entry points with fake addresses of every alignment class and with layer ranges
// at arbitrary boundaries, and verifies that the launches tile the requested columns exactly
// once.  Built with -fsanitize=address,undefined by tests/test_host_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_2007_00433_amd/csrc/se_common.hpp"
#include "../../include/sesgd.h"
#include "../../include/sesgd_tuning.h"

namespace {

struct Rec { uintptr_t x, g, v; uint64_t cols; int vec; bool coop, bf16; int mode, m, k; uint32_t tiles; };
std::vector<Rec> g_recs;
int g_failures = 0;

#define EXPECT(cond)                                                                          \
    do { if (!(cond)) { std::printf("FAIL %s:%d: %s\n", __FILE__, __LINE__, #cond); ++g_failures; } } while (0)

hipError_t record(const se::StepArgs &a, const se::LaunchShape &s, bool coop)
{
    // 128-bit bodies: row 0 of the parameters on 16 bytes, every other row on 4 at least
    const uintptr_t fa = s.vec == 4 ? 4u : (uintptr_t)s.vec * 4u;
    const uintptr_t ga = s.vec == 4 ? 4u : (uintptr_t)s.vec * (s.bf16 ? 2u : 4u);
    EXPECT(s.vec == 1 || s.vec == 2 || s.vec == 4);
    EXPECT((uintptr_t)a.x % ((uintptr_t)s.vec * 4u) == 0);
    EXPECT(a.pitch_bytes % fa == 0);
    if (a.v) EXPECT((uintptr_t)a.v % fa == 0);
    if (a.mode != se::kAvgOnly) { EXPECT(a.g != nullptr); EXPECT((uintptr_t)a.g % ga == 0); }
    EXPECT(a.nvec > 0 && a.lead < 64u && a.lead < a.nvec);
    if (a.lead) { EXPECT(s.vec == 4); EXPECT((uintptr_t)a.x % 1024u == 0); }   // only to reach a 1 KiB boundary
    EXPECT((uint64_t)a.nvec * (uint64_t)s.vec * 4u <= a.pitch_bytes);      // stays inside a row
    EXPECT(a.tiles == (a.nvec + 63u) / 64u);
    EXPECT(a.m >= 1 && a.m <= a.n && a.n <= se::kMaxWorkers && a.k * a.m == a.n);
    EXPECT(a.inv_m == 1.0f / (float)a.m);
    EXPECT(s.lds_bytes <= se::kLdsPerCu);
    if (coop) {
        EXPECT((size_t)((a.m + 7) / 8) * 64 * s.vec * 4 <= 8u * 1024u);    // one staged block sum per wavefront
        EXPECT((a.m + 7) / 8 <= 8);                                        // <= 512 threads
        EXPECT(a.coop_tiles >= 1);
    }
    // what the launch touches: the columns behind the leading, switched-off lanes
    const uint64_t skip = (uint64_t)a.lead * (uint64_t)s.vec;
    g_recs.push_back({(uintptr_t)a.x + skip * 4u, a.g ? (uintptr_t)a.g + skip * (s.bf16 ? 2u : 4u) : 0,
                      a.v ? (uintptr_t)a.v + skip * 4u : 0, (uint64_t)(a.nvec - a.lead) * (uint64_t)s.vec,
                      s.vec, coop, s.bf16, a.mode, a.m, a.k, a.tiles});
    return hipSuccess;
}

}  // namespace

namespace se {
hipError_t launch_step(const StepArgs &a, const LaunchShape &s, hipStream_t) { return record(a, s, false); }
hipError_t launch_coop(const StepArgs &a, const LaunchShape &s, hipStream_t) { return record(a, s, true); }
static size_t g_scratch_bytes = 0;      // what the last split_scratch call asked for
static int g_split_launches = 0;
static SplitShape g_last_split;
hipError_t launch_split(const StepArgs &a, const LaunchShape &s, const SplitShape &sh, hipStream_t)
{
    ++g_split_launches;
    g_last_split = sh;
    EXPECT(s.vec == 4 && a.m > 8 && sh.scratch != nullptr);
    // the buffer holds one 1 KiB piece per tile of a chunk and slot (group, or group and block of 8)
    const size_t slots = a.mode == se::kSesgd ? (size_t)a.k * (size_t)((a.m + 7) / 8) : (size_t)a.k;
    EXPECT(g_scratch_bytes == (size_t)sh.chunk_tiles * slots * 1024u);
    EXPECT(g_scratch_bytes <= ((size_t)129 << 20) || sh.chunk_tiles == sh.sub_tiles);
    EXPECT(a.mode == se::kSesgd ? (sh.finish_rows >= 8 && sh.finish_rows % 8 == 0)
           : a.mode == se::kGradAvg ? (sh.finish_rows == 1 || sh.finish_rows == 2 || sh.finish_rows == 4)
                                    : (sh.finish_rows >= 1 && sh.finish_rows <= 64));
    // chunks of equal size cover all tiles; the finish launch's grid stays far below 2^31
    const uint64_t nchunks = ((uint64_t)a.tiles + sh.chunk_tiles - 1) / sh.chunk_tiles;
    EXPECT(nchunks * sh.chunk_tiles < (uint64_t)a.tiles + nchunks * 8u * (sh.chunk_tiles / sh.sub_tiles) + 8u);
    EXPECT((uint64_t)sh.chunk_tiles * 64u < ((uint64_t)1 << 31));
    EXPECT(sh.sub_tiles >= 8 && sh.sub_tiles % 8 == 0 && sh.chunk_tiles >= sh.sub_tiles && sh.chunk_tiles % sh.sub_tiles == 0);
    EXPECT(sh.lds_reduce <= se::kLdsPerCu && sh.lds_finish <= se::kLdsPerCu);
    return record(a, s, false);
}
float *split_scratch(hipStream_t, size_t bytes)
{
    static float dummy;
    EXPECT(bytes > 0 && bytes <= ((size_t)4096 << 20));
    g_scratch_bytes = bytes;
    return &dummy;
}
hipError_t launch_plan(uint64_t, int64_t, int, int, int32_t *, int32_t *, hipStream_t) { return hipSuccess; }
hipError_t plan_to_host_noalloc(uint64_t, int64_t, int, int, int32_t *, int32_t *) { return hipSuccess; }
hipError_t launch_consensus(const float *, uint64_t, uint64_t, int, double *, hipStream_t) { return hipSuccess; }
hipError_t launch_calib_copy(void *, const void *, uint64_t, int, hipStream_t) { return hipSuccess; }
hipError_t launch_calib_oneway(void *, const void *, uint64_t, int, hipStream_t) { return hipSuccess; }
}  // namespace se

// The launches recorded since `from` must cover columns [c0, c1) of the row that starts at
// `base`, in order, without gap or overlap.
static void expect_exact_cover(size_t from, uintptr_t base, int64_t c0, int64_t c1)
{
    uintptr_t next = base + (uintptr_t)c0 * 4u;
    for (size_t i = from; i < g_recs.size(); ++i) {
        EXPECT(g_recs[i].x == next);
        next += g_recs[i].cols * 4u;
    }
    EXPECT(next == base + (uintptr_t)c1 * 4u);
}

int main()
{
    const uintptr_t X = 0x100000000ull, G = 0x200000000ull, V = 0x300000000ull;
    int calls = 0;
    for (int wide = 0; wide < 2; ++wide)
    for (int sx = 0; sx < 4; ++sx) for (int sg = 0; sg < 4; ++sg) for (int sv = 0; sv < 4; ++sv)
    for (int bf16 = 0; bf16 < 2; ++bf16) for (int64_t pitch : {1, 2, 3, 4, 5, 63, 64, 66, 257, 4096, 4099}) {
        EXPECT(se_set_tuning("unaligned_wide", wide) == SE_OK);
        int64_t offs[4] = {0, pitch / 3, pitch / 3 + (pitch > 7 ? 5 : 0), pitch};
        float *x = (float *)(X + 4u * sx);
        void *g = (void *)(G + (bf16 ? 2u : 4u) * sg);
        float *v = (float *)(V + 4u * sv);
        for (int first = 0; first <= 3; ++first) for (int last = first; last <= 3; ++last) {
            for (int n : {1, 4, 16, 64}) for (int m : {1, 4, 16, 64}) {
                if (m > n) continue;
                const size_t from = g_recs.size();
                const int rc = se_step_ex(x, g, bf16, (n & 4) ? v : nullptr, offs, 3, first, last, n, m, 7,
                                          0.1f, (n & 4) ? 0.9f : 0.0f, 1e-4f, (m & 4) ? SE_FLAG_GRAD_AVG : 0u, nullptr);
                EXPECT(rc == SE_OK);
                expect_exact_cover(from, (uintptr_t)x, offs[first], offs[last]);
                ++calls;
            }
        }
        const size_t from = g_recs.size();
        EXPECT(se_global_average(x, offs, 3, 16, nullptr) == SE_OK);
        expect_exact_cover(from, (uintptr_t)x, 0, pitch);
        EXPECT(se_ring_step(x, (const float *)(G + 4u * sg), v, offs, 3, 16, 0.1f, 0.9f, nullptr) == SE_OK);
    }
    // rows that are only 4-byte aligned: a 128-bit body with at most 3 scalar columns on either side
    {
        int64_t offs[2] = {0, 25557033};
        for (int bf16 = 0; bf16 < 2; ++bf16) {
            const size_t from = g_recs.size();
            EXPECT(se_step_ex((float *)(X + 4u), (const void *)G, bf16, (float *)(V + 8u), offs, 1, 0, 1, 16, 4, 0,
                              0.1f, 0.9f, 0.0f, 0u, nullptr) == SE_OK);
            uint64_t wide_cols = 0;
            for (size_t i = from; i < g_recs.size(); ++i) if (g_recs[i].vec == 4) wide_cols += g_recs[i].cols;
            if (bf16) EXPECT(wide_cols == 0);                 // odd pitch: bf16 rows start on odd 2-byte addresses
            else EXPECT(wide_cols >= 25557033u - 6u);
        }
    }
    // the aligned, padded case is a single 128-bit launch
    {
        int64_t offs[2] = {0, 25557056};
        const size_t from = g_recs.size();
        EXPECT(se_step((float *)X, (const float *)G, (float *)V, offs, 1, 16, 4, 0, 0.1f, 0.9f, nullptr) == SE_OK);
        EXPECT(g_recs.size() == from + 1 && g_recs[from].vec == 4 && !g_recs[from].coop &&
               g_recs[from].tiles == (25557056u / 4 + 63) / 64);
        EXPECT(se_ring_step((float *)X, (const float *)G, (float *)V, offs, 1, 16, 0.1f, 0.9f, nullptr) == SE_OK);
        EXPECT(!g_recs.back().coop && g_recs.back().mode == se::kGradAvg && g_recs.back().m == 16 && g_recs.back().k == 1);
    }
    // large reductions take the split form by themselves from 2 GiB per call, and on request
    // for any size that streams; every shape of it is checked in the launch_split stand-in
    {
        const int before = se::g_split_launches;
        const uintptr_t X = (uintptr_t)1 << 40, G = (uintptr_t)2 << 40, V = (uintptr_t)3 << 40;   // 1 TiB apart
        for (int64_t pitch : {(int64_t)25558016, (int64_t)109483008, (int64_t)138357760, (int64_t)4 * 8191 * 64, (int64_t)1024}) {
            int64_t offs[3] = {0, pitch / 8 * 4 + 256, pitch};
            for (int n : {16, 32, 64}) for (int m : {16, 32, 64}) {
                if (m > n) continue;
                for (int forced = 0; forced < 2; ++forced) for (int first = 0; first < 2; ++first) {
                    EXPECT(se_set_tuning("split", forced ? 1 : -1) == SE_OK);
                    EXPECT(se_set_tuning("cache_resident_mib", forced ? 0 : 512) == SE_OK);
                    EXPECT(se_set_tuning("split_sub_tiles", forced && first ? 8 : 0) == SE_OK);
                    EXPECT(se_set_tuning("split_scratch_mib", forced && !first ? 1 : 128) == SE_OK);
                    const size_t from = g_recs.size();
                    EXPECT(se_step_ex((float *)X, (const void *)G, m == 32, (float *)V, offs, 2, first, 2, n, m, 3, 0.1f, 0.9f, 0.0f,
                                      (n == 32) ? SE_FLAG_GRAD_AVG : 0u, nullptr) == SE_OK);
                    expect_exact_cover(from, X, offs[first], offs[2]);
                    EXPECT(g_recs.size() == from + 1);            // one record per call: no head or tail pieces here
                }
            }
        }
        EXPECT(se::g_split_launches > before + 60);
        // the parameter average of many workers: split from 3 GiB per call, an eighth of the
        // workers (2 to 8 rows) per wavefront of the pass that writes the mean
        se_set_tuning("split", -1); se_set_tuning("cache_resident_mib", 512);
        se_set_tuning("split_sub_tiles", 0); se_set_tuning("split_scratch_mib", 128);
        for (int n : {8, 9, 16, 24, 64}) for (int64_t pitch : {(int64_t)1 << 20, (int64_t)25558016, (int64_t)109483008}) {
            int64_t offs[2] = {0, pitch};
            const int launches = se::g_split_launches;
            const size_t from = g_recs.size();
            EXPECT(se_global_average((float *)X, offs, 1, n, nullptr) == SE_OK);
            expect_exact_cover(from, X, 0, pitch);
            const bool expected = n > 8 && (uint64_t)n * (uint64_t)pitch * 8u >= ((uint64_t)3 << 30);
            EXPECT((se::g_split_launches == launches + 1) == expected);
            if (expected) {
                const int eighth = (n + 7) / 8;
                EXPECT(se::g_last_split.finish_rows == (eighth < 2 ? 2 : eighth));
                EXPECT(se::g_last_split.lds_finish > 0 && se::g_last_split.lds_reduce > 0);
            }
        }
        se_set_tuning("split", -1); se_set_tuning("cache_resident_mib", 512);
        se_set_tuning("split_sub_tiles", 0); se_set_tuning("split_scratch_mib", 128);
    }
    // error paths write nothing and launch nothing
    {
        int64_t offs[2] = {0, 100};
        const size_t from = g_recs.size();
        EXPECT(se_step((float *)X, (const float *)G, nullptr, offs, 1, 6, 4, 0, 0.1f, 0.0f, nullptr) == SE_ERR_DIVISIBILITY);
        EXPECT(se_step((float *)X, (const float *)X, nullptr, offs, 1, 4, 2, 0, 0.1f, 0.0f, nullptr) == SE_ERR_LAYOUT);
        EXPECT(se_step_ex((float *)X, (const void *)G, 0, nullptr, offs, 1, 0, 2, 4, 2, 0, 0.1f, 0.0f, 0.0f, 0u, nullptr) == SE_ERR_ARG);
        EXPECT(g_recs.size() == from);
    }
    std::printf("%d calls, %zu launches checked, %d failures\n", calls, g_recs.size(), g_failures);
    return g_failures ? 1 : 0;
}

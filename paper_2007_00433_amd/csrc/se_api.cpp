// C ABI of the SESGD step library (see include/sesgd.h): argument validation on the host,
// choice of the launch shape, kernel launch on the caller's stream.  No torch types, no
// CPU fallback: every step of the method runs in the HIP kernels.
#include "se_common.hpp"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>

#include "../../include/sesgd.h"
#include "../../include/sesgd_tuning.h"

namespace {

std::atomic<uint64_t> g_seed{0};
std::atomic<int> g_nontemporal{2};         // se::Policy of the row accesses of launches that stream from HBM
std::atomic<int> g_max_blocks_per_cu{-1}; // resident workgroups per CU (0 = no cap, -1 = chosen per launch)
std::atomic<int> g_cooperative{0};        // LDS-staged form: 0 never, 1 always (and no split form then)
std::atomic<int> g_coop_tiles{0};         // cooperative form: consecutive tiles per workgroup (0 = by group size)
std::atomic<int> g_cache_resident_mib{512};  // calls moving fewer MiB per step run faster with plain accesses (256 MiB Infinity Cache)
std::atomic<int> g_split{-1};             // split form for more than 8 rows per group: 0 never, 1 always, -1 where it measured faster
std::atomic<int> g_split_scratch_mib{128}; // size of the split form's intermediate buffer
std::atomic<int> g_split_sub_tiles{0};    // tiles per sub-chunk of the split form's finish launch (0 = by mode)
std::atomic<int> g_split_cap_reduce{-1};  // resident workgroups per CU of the two launches (0 = no cap, -1 = default)
std::atomic<int> g_split_cap_finish{-1};
std::atomic<int> g_split_finish_rows{0};  // rows per wavefront of the finish launch (0 = default)
std::atomic<int> g_batch_rows{0};         // member rows whose loads are issued back to back (0 = chosen per launch)
std::atomic<int> g_unaligned_wide{1};     // 128-bit accesses also for rows that are only 4-byte aligned

thread_local char t_last_error[256] = "";

int hip_fail(const char *what, hipError_t e)
{
    std::snprintf(t_last_error, sizeof t_last_error, "%s: %s", what, hipGetErrorString(e));
    return SE_ERR_HIP;
}

bool overlaps(const void *a, uint64_t abytes, const void *b, uint64_t bbytes)
{
    if (!a || !b || abytes == 0 || bbytes == 0) return false;
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

// Everything that can be rejected without touching the device.  grads may be NULL only when
// grad_bytes == 0 (calls that take no gradients).
int validate(const void *params, const void *grads, const void *momentum,
             const int64_t *layer_offsets, int num_layers, int n, int group_size, int64_t iter,
             float mu, int grad_bytes, int64_t *pitch_out)
{
    if (n < 1 || group_size < 1 || group_size > n || iter < 0 || num_layers < 0) return SE_ERR_ARG;
    if (n % group_size != 0) return SE_ERR_DIVISIBILITY;
    if (!params || !layer_offsets || (grad_bytes && !grads)) return SE_ERR_NULL;
    if (!momentum && mu != 0.0f) return SE_ERR_NULL;
    if (layer_offsets[0] != 0) return SE_ERR_LAYOUT;
    for (int l = 0; l < num_layers; ++l)
        if (layer_offsets[l + 1] < layer_offsets[l]) return SE_ERR_LAYOUT;
    const int64_t pitch = layer_offsets[num_layers];
    if (n > SE_MAX_WORKERS || pitch >= ((int64_t)1 << 30)) return SE_ERR_UNSUPPORTED;
    const uintptr_t px = (uintptr_t)params, pg = (uintptr_t)grads, pv = (uintptr_t)momentum;
    if (px % 4 || pv % 4 || (grad_bytes && pg % (uintptr_t)grad_bytes)) return SE_ERR_LAYOUT;
    const uint64_t fbytes = (uint64_t)n * (uint64_t)pitch * 4u;
    const uint64_t gbytes = (uint64_t)n * (uint64_t)pitch * (uint64_t)grad_bytes;
    if (overlaps(params, fbytes, grads, gbytes) || overlaps(params, fbytes, momentum, fbytes) ||
        overlaps(grads, gbytes, momentum, fbytes))
        return SE_ERR_LAYOUT;
    *pitch_out = pitch;
    return SE_OK;
}

struct Job {
    float *x;
    const void *g;
    float *v;
    int grad_bytes;          // 4, 2, or 0 when the mode reads no gradients
    int64_t pitch;
    int n, m;
    int64_t iter;
    float lr, mu, wd;
    int mode;
    hipStream_t stream;
};

// Launch shape of the one-launch forms on buffers that stream from HBM, from sweeps on MI355X
// (ResNet-50-, VGG-16- and BERT-sized rows; fp32 and bf16 gradients; with and without a momentum
// buffer; 4 to 64 workers; all group sizes up to 8).
//
// Rows per batch: a wavefront issues the loads of `batch` member rows (x, g, v of each) back to
// back, then does their arithmetic and stores.  One row at a time measured 1-3 % faster for
// groups of up to 4 than all rows at once, two at a time for groups of 5 to 8: fewer rows open
// per wavefront at a time.  The same holds for the update pass of gradient averaging.
int auto_batch_rows(const Job &j, bool streams, uint64_t launch_bytes)
{
    if (j.mode == se::kAvgOnly) return 8;
    // Buffers small enough for plain accesses: all rows of a small group at once is 0-5 % faster.
    // Launches over few columns (a layer range) are over before the order of the rows matters;
    // there one round trip for all rows is what counts (161 per-tensor launches of the
    // ResNet-50 shape: 566 against 530 steps/s).
    // Reductions over more than 8 rows out of the cache: two rows at a time (ResNet-20-sized rows,
    // 16 workers: ring 5.9 -> 6.2 TB/s, one group of 16 6.05 -> 6.5).
    if (!streams && j.m > 8) return 2;
    if (!streams || launch_bytes < ((uint64_t)64 << 20)) return j.mode == se::kSesgd && j.m < 8 ? 4 : 8;
    if (j.m > 8) return j.mode == se::kGradAvg ? 1 : 8;
    return j.m <= 4 ? 1 : 2;
}

// Resident workgroups per CU.  What the sweeps have in common is the amount of loads in flight
// per CU: about 48 KiB for singleton groups, 32 KiB for pairs, 25-28 KiB for larger groups (36 KiB
// for groups of 5, whose batches are 2 + 2 + 1 rows, and for gradient averaging over 3, 5 or 6
// rows), whatever the bytes per row (momentum buffer
// or not, fp32 or bf16 gradients, 128-, 64- or 32-bit accesses): 16 / 11 / 8 workgroups for
// groups of 1 / 2 / 4 with momentum and fp32 gradients, 10 for groups of 4 with bf16 gradients,
// 24 / 16 / 13 without a momentum buffer, 4 to 6 for groups of 8 two rows at a time.  Fewer
// starve the memory system, more scatter the tiles in flight and lose DRAM locality.
int auto_blocks_per_cu(const Job &j, int batch, int vec)
{
    if (j.mode == se::kAvgOnly) return j.m <= 2 ? 12 : j.m <= 4 ? 8 : 4;   // 4 workers: 6.65 TB/s with 8, 4.90 with 4
    if (j.m > 8) return j.mode == se::kGradAvg ? 6 : 2;
    if (batch > j.m) batch = j.m;
    const int row_bytes = 64 * vec * (4 + j.grad_bytes + (j.v ? 4 : 0));
    if (batch >= 4) {
        // all rows of the group at once (small launches, or on request): about 72 KiB in flight
        const int all = 72 * 1024 / (batch * row_bytes);
        return all < 4 ? 4 : all > 16 ? 16 : all;
    }
    int target_kib = j.m == 1 ? 48 : j.m == 2 ? 32 : j.m <= 4 ? 25 : j.m == 5 ? 36 : 28;
    if (j.mode == se::kGradAvg && (j.m == 3 || j.m == 5 || j.m == 6)) target_kib = 36;
    const int target = target_kib * 1024;
    const int cap = (target + batch * row_bytes / 2) / (batch * row_bytes);
    return cap < 2 ? 2 : cap > 24 ? 24 : cap;
}

// Shape of the split form for one range of columns.  False when its intermediate buffer cannot
// be had (the stream is being captured into a graph, or the allocation failed): the caller then
// launches the one-launch form.
bool split_shape(const Job &j, const se::StepArgs &a, se::SplitShape *out)
{
    const uint32_t nb = (uint32_t)((j.m + se::kSumBlock - 1) / se::kSumBlock);
    const uint32_t slots = j.mode == se::kSesgd ? (uint32_t)a.k * nb : (uint32_t)a.k;
    se::SplitShape sh;
    // Sub-chunks of 4096 tiles (4 MiB of every row) measured best when one mean gradient is
    // re-read per row, 256-2048 tiles alike and 4096 5 % slower when 8 block sums are.
    uint64_t sub_target = (uint64_t)g_split_sub_tiles.load() / 8u * 8u;
    if (sub_target == 0) sub_target = j.mode == se::kSesgd ? 2048u : 4096u;
    // Chunks as large as the buffer allows, all of the same size, each cut into sub-chunks of
    // the same size (a short last sub-chunk would switch rows every few tiles).
    const uint64_t budget = (uint64_t)g_split_scratch_mib.load() << 20;
    uint64_t max_chunk = budget / ((uint64_t)slots * 1024u);         // 1 KiB per slot and tile
    if (max_chunk < 8u) max_chunk = 8u;
    const uint64_t all = ((uint64_t)a.tiles + 7u) / 8u * 8u;
    const uint64_t nchunks = (all + max_chunk - 1u) / max_chunk;
    const uint64_t chunk_target = (all + nchunks - 1u) / nchunks;
    const uint64_t nsub = (chunk_target + sub_target - 1u) / sub_target;
    sh.sub_tiles = (uint32_t)(((chunk_target + nsub - 1u) / nsub + 7u) / 8u * 8u);
    const uint64_t chunk = (uint64_t)sh.sub_tiles * nsub;
    sh.chunk_tiles = (uint32_t)chunk;
    sh.scratch = se::split_scratch(j.stream, (size_t)(chunk * slots * 1024u));
    if (!sh.scratch) return false;
    int fr = g_split_finish_rows.load();
    if (j.mode == se::kGradAvg) fr = fr >= 4 ? 4 : fr >= 2 ? 2 : 1;
    else if (j.mode == se::kAvgOnly) {
        // rows one wavefront writes the mean to: an eighth of the group (2 to 8) measured best
        const int eighth = (j.m + 7) / 8;
        if (fr < 1) fr = eighth < 2 ? 2 : eighth > 8 ? 8 : eighth;
    }
    else fr = fr < 8 ? 8 : fr / 8 * 8;
    sh.finish_rows = fr;
    sh.reduce_batch = g_batch_rows.load() > 0 ? g_batch_rows.load() : 1;
    // Resident workgroups per CU, from sweeps on the ResNet-50, VGG-16 and BERT shapes: the
    // mean-gradient pass has 8 KiB or less in flight per wavefront and wants 12 or more, the
    // one-row update 24; the 8-row SESGD pass, walked one row at a time like the single-wavefront
    // form, 7 (10 with bf16 gradients; all 8 rows at once with 4 to 6 workgroups measured 1-4 %
    // slower), the pass that writes the mean 16.  Without a momentum buffer a row is a third
    // shorter: twice as many in the 8-row pass and 8 in the pass that writes the mean (6.19
    // against 5.45 TB/s), 32 in the one-row update.
    int cr = g_split_cap_reduce.load(), cf = g_split_cap_finish.load();
    if (cr < 0) cr = j.mode != se::kSesgd ? (j.v ? 12 : 10) : (j.grad_bytes == 2 ? 10 : 7) * (j.v ? 1 : 2);
    if (cf < 0) cf = j.mode != se::kSesgd ? (j.v ? 24 : 32) : (j.v ? 16 : 8);
    if (j.mode == se::kAvgOnly) {
        // The parameter average: 6 workgroups in the pass that adds the rows up (8 at a time); in
        // the pass that writes the mean about 48 rows in flight per CU (64 beyond 32 workers),
        // whatever the rows per wavefront.  9 to 64 workers: 6.25-6.6 TB/s (ResNet-50-sized rows).
        if (g_split_cap_reduce.load() < 0) cr = 6;
        if (g_split_cap_finish.load() < 0) {
            cf = (j.m > 32 ? 64 : 48) / fr;
            cf = cf < 2 ? 2 : cf > 32 ? 32 : cf;
        }
    }
    sh.lds_reduce = cr > 0 ? (se::kLdsPerCu / (uint32_t)cr) & ~1023u : 0u;
    sh.lds_finish = cf > 0 ? (se::kLdsPerCu / (uint32_t)cf) & ~1023u : 0u;
    *out = sh;
    return true;
}

// One launch over columns [c0, c1) with `vec` columns per lane; (c1 - c0) % vec == 0 and every
// row of every buffer is vec-aligned at column c0 (for vec == 4, 4-byte alignment of the other
// rows is enough when row 0 of the parameters is 16-byte aligned there).
hipError_t launch_columns(const Job &j, int64_t c0, int64_t c1, int vec)
{
    if (c1 <= c0) return hipSuccess;
    se::StepArgs a;
    // A wavefront moves 1 KiB of each row per access, and 1 KiB-aligned pieces measure 3-4 %
    // faster (25 % when the pieces do not even start on a 128-byte line).  A 128-bit launch that
    // starts in the middle of such a piece (a layer range) is therefore started at the piece's
    // beginning, with the lanes before c0 switched off.  Where that would reach in front of the
    // row (a base address that is not 1 KiB aligned), a long range is split instead: the
    // columns up to the next boundary first, the aligned rest after them.
    int64_t lead_cols = 0;
    if (vec == 4) {
        lead_cols = (int64_t)(((uintptr_t)j.x / 4u + (uintptr_t)c0) % 256u);
        if (lead_cols > c0) {
            const int64_t head = 256 - lead_cols;
            if (c1 - c0 >= 65536) {
                const hipError_t e = launch_columns(j, c0, c0 + head, vec);   // short: not split again
                return e != hipSuccess ? e : launch_columns(j, c0 + head, c1, vec);
            }
            lead_cols = 0;
        }
    }
    const int64_t s0 = c0 - lead_cols;
    a.x = j.x + s0;
    a.g = j.g ? (const void *)((const char *)j.g + s0 * j.grad_bytes) : nullptr;
    a.v = j.v ? j.v + s0 : nullptr;
    a.seed = g_seed.load();
    a.iter = j.iter;
    a.pitch_bytes = (uint64_t)j.pitch * 4u;
    a.lead = (uint32_t)(lead_cols / vec);
    a.nvec = (uint32_t)((c1 - s0) / vec);
    a.tiles = (a.nvec + 63u) / 64u;
    const int coop_tiles = g_coop_tiles.load();
    a.coop_tiles = coop_tiles > 0 ? (uint32_t)coop_tiles : (j.m > 32 ? 4u : 1u);
    a.n = j.n; a.m = j.m; a.k = j.n / j.m;
    a.neg_lr = -j.lr; a.mu = j.mu; a.inv_m = 1.0f / (float)j.m; a.wd = j.wd;
    a.mode = j.mode;

    se::LaunchShape s;
    s.vec = vec;
    s.bf16 = j.grad_bytes == 2;
    // Streaming accesses and a residency cap pay off when the buffers stream from HBM; buffers
    // that fit the Infinity Cache as a whole are faster with plain accesses and no cap.  The
    // whole rows count, not the columns of this launch: a caller that steps layer by layer
    // still walks through all of them between two visits of the same layer.
    const uint64_t per_elem = 8u + (uint64_t)j.grad_bytes + (j.v ? 8u : 0u);
    const uint64_t moved = (uint64_t)j.n * (uint64_t)j.pitch * per_elem;
    const bool streams = moved >= ((uint64_t)g_cache_resident_mib.load() << 20);
    s.policy = streams ? g_nontemporal.load() : se::kPlain;
    s.batch_rows = g_batch_rows.load();
    if (s.batch_rows <= 0)
        s.batch_rows = auto_batch_rows(j, streams, (uint64_t)j.n * (uint64_t)(c1 - c0) * per_elem);
    // The LDS-staged form (one block of 8 rows per wavefront, block sums staged in LDS) measured
    // slower than the single-wavefront form for every group size (0.5-7 %) and than the split
    // form for large ones; it runs only when asked for.
    const int coop = g_cooperative.load();
    const bool use_coop = coop > 0;
    int cap = g_max_blocks_per_cu.load();
    if (cap < 0) cap = !streams ? 0 : use_coop ? 8 : auto_blocks_per_cu(j, s.batch_rows, vec);
    s.lds_bytes = cap > 0 ? (se::kLdsPerCu / (uint32_t)cap) & ~1023u : 0u;
    // Split form: two launches per chunk of columns with an intermediate in a library-owned
    // buffer; for reductions over more than 8 rows on the 128-bit path.  Measured on MI355X it
    // beats the one-launch forms by 6-20 % for the gradient-averaging modes (the Ring-SGD
    // baseline) and the SESGD update once a launch moves about 2 GiB, by 5-20 % for the parameter
    // average of 16 to 64 workers from about 3 GiB, and it does not depend on where the driver
    // happened to place the buffers.
    const int split = g_split.load();
    const uint64_t launch_bytes = (uint64_t)j.n * (uint64_t)(c1 - c0) * per_elem;
    const bool split_pays = launch_bytes >= (j.mode == se::kAvgOnly ? (uint64_t)3 << 30 : (uint64_t)1 << 31);
    if (vec == 4 && streams && j.m > se::kSumBlock && coop <= 0 &&
        (split > 0 || (split < 0 && split_pays))) {
        se::SplitShape sh;
        if (split_shape(j, a, &sh)) return se::launch_split(a, s, sh, j.stream);
    }
    if (use_coop) return se::launch_coop(a, s, j.stream);
    return se::launch_step(a, s, j.stream);
}

// Columns [c0, c1) of every row: the widest body the rows allow plus scalar head and tail columns.
hipError_t launch_range(const Job &j, int64_t c0, int64_t c1)
{
    if (c1 <= c0) return hipSuccess;
    const int gb = j.grad_bytes ? j.grad_bytes : 4;
    const uintptr_t ex = (uintptr_t)j.x / 4u;                       // base addresses in elements
    const uintptr_t ev = j.v ? (uintptr_t)j.v / 4u : ex;
    const uintptr_t eg = j.g ? (uintptr_t)j.g / (uintptr_t)gb : ex;
    for (int vec = 4; vec > 1; vec >>= 1) {
        const uintptr_t v = (uintptr_t)vec;
        if (j.pitch % vec != 0 || ex % v != ev % v || ex % v != eg % v) {
            // Rows that do not line up on 16 bytes (a pitch that is no multiple of 4 elements,
            // bases at different offsets) still take 128-bit accesses when each starts on a
            // 4-byte boundary, which is all a multi-dword global access needs: fp32 rows always
            // do, bf16 gradient rows when the pitch and their first column are even.  Measured
            // against the 64- and 32-bit bodies these rows would otherwise get: see the tuning
            // header.  Row 0 of the parameters is brought to a 16-byte boundary first.
            const bool g16 = j.g && j.grad_bytes == 2;
            const int64_t head = (int64_t)((4u - (ex + (uintptr_t)c0) % 4u) % 4u);
            const bool dword_rows = !g16 || (j.pitch % 2 == 0 && (eg + (uintptr_t)(c0 + head)) % 2u == 0);
            if (vec == 4 && g_unaligned_wide.load() > 0 && dword_rows && c1 - (c0 + head) >= 4) {
                const int64_t a = c0 + head, b = a + (c1 - a) / 4 * 4;
                hipError_t e = launch_columns(j, c0, a, 1);
                if (e == hipSuccess) e = launch_columns(j, a, b, 4);
                if (e == hipSuccess) e = launch_columns(j, b, c1, 1);
                return e;
            }
            continue;
        }
        const int64_t head = (int64_t)((v - (ex + (uintptr_t)c0) % v) % v);   // columns up to alignment
        const int64_t a = c0 + head;
        if (a >= c1) break;
        const int64_t b = a + (c1 - a) / vec * vec;
        if (b <= a) continue;
        hipError_t e = launch_columns(j, c0, a, 1);
        if (e == hipSuccess) e = launch_columns(j, a, b, vec);
        if (e == hipSuccess) e = launch_columns(j, b, c1, 1);
        return e;
    }
    return launch_columns(j, c0, c1, 1);
}

int run(const char *what, float *params, const void *grads, int grad_bytes, float *momentum,
        const int64_t *layer_offsets, int num_layers, int first_layer, int last_layer,
        int n, int group_size, int64_t iter, float lr, float mu, float wd, int mode, void *stream)
{
    int64_t pitch = 0;
    const int rc = validate(params, grads, momentum, layer_offsets, num_layers, n, group_size,
                            iter, mu, grad_bytes, &pitch);
    if (rc != SE_OK) return rc;
    if (first_layer < 0 || last_layer < first_layer || last_layer > num_layers) return SE_ERR_ARG;
    Job j;
    j.x = params; j.g = grads; j.v = momentum; j.grad_bytes = grad_bytes;
    j.pitch = pitch; j.n = n; j.m = group_size; j.iter = iter;
    j.lr = lr; j.mu = mu; j.wd = wd; j.mode = mode; j.stream = (hipStream_t)stream;
    const hipError_t e = launch_range(j, layer_offsets[first_layer], layer_offsets[last_layer]);
    return e == hipSuccess ? SE_OK : hip_fail(what, e);
}

int plan_check(int n, int group_size, int64_t iter, const void *group_of)
{
    if (n < 1 || group_size < 1 || group_size > n || iter < 0) return SE_ERR_ARG;
    if (n % group_size != 0) return SE_ERR_DIVISIBILITY;
    if (!group_of) return SE_ERR_NULL;
    if (n > SE_MAX_WORKERS) return SE_ERR_UNSUPPORTED;
    return SE_OK;
}

struct Knob { const char *name; std::atomic<int> *value; int lo, hi; };
Knob kKnobs[] = {
    {"max_blocks_per_cu", &g_max_blocks_per_cu, -1, 32},
    {"nontemporal", &g_nontemporal, 0, 2},
    {"cooperative", &g_cooperative, 0, 1},
    {"coop_tiles", &g_coop_tiles, 0, 4096},
    {"cache_resident_mib", &g_cache_resident_mib, 0, 1 << 20},
    {"split", &g_split, -1, 1},
    {"split_scratch_mib", &g_split_scratch_mib, 1, 4096},
    {"split_sub_tiles", &g_split_sub_tiles, 0, 1 << 24},
    {"split_cap_reduce", &g_split_cap_reduce, -1, 32},
    {"split_cap_finish", &g_split_cap_finish, -1, 32},
    {"split_finish_rows", &g_split_finish_rows, 0, 64},
    {"batch_rows", &g_batch_rows, 0, 8},
    {"unaligned_wide", &g_unaligned_wide, 0, 1},
};

}  // namespace

extern "C" {

int se_plan(int n, int group_size, int64_t iter, int32_t *group_of, int32_t *members)
{
    const int rc = plan_check(n, group_size, iter, group_of);
    if (rc != SE_OK) return rc;
    int32_t *dev = nullptr;
    hipError_t e = hipMalloc((void **)&dev, sizeof(int32_t) * 2u * (size_t)n);
    if (e != hipSuccess) return hip_fail("se_plan hipMalloc", e);
    e = se::launch_plan(g_seed.load(), iter, n, group_size, dev, members ? dev + n : nullptr, nullptr);
    if (e == hipSuccess) e = hipMemcpy(group_of, dev, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost);
    if (e == hipSuccess && members)
        e = hipMemcpy(members, dev + n, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost);
    const hipError_t ef = hipFree(dev);
    if (e != hipSuccess) return hip_fail("se_plan", e);
    if (ef != hipSuccess) return hip_fail("se_plan hipFree", ef);
    return SE_OK;
}

int se_plan_noalloc(int n, int group_size, int64_t iter, int32_t *group_of, int32_t *members)
{
    const int rc = plan_check(n, group_size, iter, group_of);      // n > 64 is SE_ERR_UNSUPPORTED
    if (rc != SE_OK) return rc;
    const hipError_t e = se::plan_to_host_noalloc(g_seed.load(), iter, n, group_size, group_of, members);
    return e == hipSuccess ? SE_OK : hip_fail("se_plan_noalloc", e);
}

int se_plan_device(int n, int group_size, int64_t iter, int32_t *group_of_dev,
                   int32_t *members_dev, void *stream)
{
    const int rc = plan_check(n, group_size, iter, group_of_dev);
    if (rc != SE_OK) return rc;
    const hipError_t e = se::launch_plan(g_seed.load(), iter, n, group_size, group_of_dev,
                                         members_dev, (hipStream_t)stream);
    return e == hipSuccess ? SE_OK : hip_fail("se_plan_device launch", e);
}

int se_step(float *params, const float *grads, float *momentum, const int64_t *layer_offsets,
            int num_layers, int n, int group_size, int64_t iter, float lr, float mu, void *stream)
{
    return run("se_step launch", params, grads, 4, momentum, layer_offsets, num_layers, 0,
               num_layers, n, group_size, iter, lr, mu, 0.0f, se::kSesgd, stream);
}

int se_step_bf16g(float *params, const uint16_t *grads_bf16, float *momentum,
                  const int64_t *layer_offsets, int num_layers, int n, int group_size,
                  int64_t iter, float lr, float mu, void *stream)
{
    return run("se_step_bf16g launch", params, grads_bf16, 2, momentum, layer_offsets, num_layers,
               0, num_layers, n, group_size, iter, lr, mu, 0.0f, se::kSesgd, stream);
}

int se_step_ex(float *params, const void *grads, int grads_are_bf16, float *momentum,
               const int64_t *layer_offsets, int num_layers, int first_layer, int last_layer,
               int n, int group_size, int64_t iter, float lr, float mu, float weight_decay,
               unsigned flags, void *stream)
{
    if (flags & ~(unsigned)SE_FLAG_GRAD_AVG) return SE_ERR_ARG;
    return run("se_step_ex launch", params, grads, grads_are_bf16 ? 2 : 4, momentum, layer_offsets,
               num_layers, first_layer, last_layer, n, group_size, iter, lr, mu, weight_decay,
               (flags & SE_FLAG_GRAD_AVG) ? se::kGradAvg : se::kSesgd, stream);
}

// Ring-SGD is the gradient-averaging form with a single group of all n workers.
int se_ring_step(float *params, const float *grads, float *momentum, const int64_t *layer_offsets,
                 int num_layers, int n, float lr, float mu, void *stream)
{
    return run("se_ring_step launch", params, grads, 4, momentum, layer_offsets, num_layers, 0,
               num_layers, n, n < 1 ? 1 : n, 0, lr, mu, 0.0f, se::kGradAvg, stream);
}

int se_ring_step_bf16g(float *params, const uint16_t *grads_bf16, float *momentum,
                       const int64_t *layer_offsets, int num_layers, int n, float lr, float mu,
                       void *stream)
{
    return run("se_ring_step_bf16g launch", params, grads_bf16, 2, momentum, layer_offsets,
               num_layers, 0, num_layers, n, n < 1 ? 1 : n, 0, lr, mu, 0.0f, se::kGradAvg, stream);
}

int se_global_average(float *params, const int64_t *layer_offsets, int num_layers, int n,
                      void *stream)
{
    return run("se_global_average launch", params, nullptr, 0, nullptr, layer_offsets, num_layers,
               0, num_layers, n, n < 1 ? 1 : n, 0, 0.0f, 0.0f, 0.0f, se::kAvgOnly, stream);
}

int se_consensus(const float *params, const int64_t *layer_offsets, int num_layers, int n,
                 double *out_dev, void *stream)
{
    int64_t pitch = 0;
    const int rc = validate(params, nullptr, nullptr, layer_offsets, num_layers, n, 1, 0, 0.0f, 0,
                            &pitch);
    if (rc != SE_OK) return rc;
    if (!out_dev) return SE_ERR_NULL;
    if ((uintptr_t)out_dev % 8 ||
        overlaps(params, (uint64_t)n * (uint64_t)pitch * 4u, out_dev, 16))
        return SE_ERR_LAYOUT;
    const hipError_t e = se::launch_consensus(params, (uint64_t)pitch, (uint64_t)pitch, n, out_dev,
                                              (hipStream_t)stream);
    return e == hipSuccess ? SE_OK : hip_fail("se_consensus launch", e);
}

int se_comm_model(const int64_t *layer_offsets, int num_layers, int elem_bytes, int n, int groups,
                  double bandwidth, double latency, double *ring_seconds, double *sesgd_seconds,
                  int64_t *ring_handshakes, int64_t *sesgd_handshakes)
{
    if (num_layers < 0 || elem_bytes < 1 || n < 1 || groups < 1 || !(bandwidth > 0.0) ||
        !(latency >= 0.0))
        return SE_ERR_ARG;
    if (n % groups != 0) return SE_ERR_DIVISIBILITY;
    if (!layer_offsets) return SE_ERR_NULL;
    if (layer_offsets[0] != 0) return SE_ERR_LAYOUT;
    for (int l = 0; l < num_layers; ++l)
        if (layer_offsets[l + 1] < layer_offsets[l]) return SE_ERR_LAYOUT;
    const int m = n / groups;
    double ring = 0.0, se_t = 0.0;
    for (int l = 0; l < num_layers; ++l) {
        const double bytes = (double)(layer_offsets[l + 1] - layer_offsets[l]) * (double)elem_bytes;
        ring += 2.0 * (double)(n - 1) * (bytes / ((double)n * bandwidth) + latency);
        se_t += 2.0 * (double)(m - 1) * (bytes / ((double)m * bandwidth) + latency);
    }
    if (ring_seconds) *ring_seconds = ring;
    if (sesgd_seconds) *sesgd_seconds = se_t;
    if (ring_handshakes) *ring_handshakes = (int64_t)num_layers * 2 * (n - 1);
    if (sesgd_handshakes) *sesgd_handshakes = (int64_t)num_layers * 2 * (m - 1);
    return SE_OK;
}

int se_layer_buckets(const int64_t *layer_offsets, int num_layers, int64_t min_elements,
                     int32_t *first_layer, int capacity, int *num_ranges)
{
    if (num_layers < 0 || min_elements < 1 || capacity < 0) return SE_ERR_ARG;
    if (!layer_offsets || !num_ranges || (capacity > 0 && !first_layer)) return SE_ERR_NULL;
    if (layer_offsets[0] != 0) return SE_ERR_LAYOUT;
    for (int l = 0; l < num_layers; ++l)
        if (layer_offsets[l + 1] < layer_offsets[l]) return SE_ERR_LAYOUT;
    // back to front: a range is closed as soon as it holds min_elements, the front-most range
    // takes what is left; first a count, so that nothing is written when it does not fit
    for (int pass = 0; pass < 2; ++pass) {
        int count = 0, end = num_layers;
        for (int l = num_layers - 1; l >= 0; --l) {
            if (layer_offsets[end] - layer_offsets[l] >= min_elements || l == 0) {
                if (pass == 1) first_layer[count] = (int32_t)l;
                ++count;
                end = l;
            }
        }
        if (pass == 0) {
            *num_ranges = count;
            if (count > capacity) return SE_ERR_ARG;
        }
    }
    return SE_OK;
}

int se_calib_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (nbytes < 0) return SE_ERR_ARG;
    if (!dst || !src) return SE_ERR_NULL;
    if ((uintptr_t)dst % 16 || (uintptr_t)src % 16 || nbytes % 16 || nbytes >= ((int64_t)1 << 37) ||
        overlaps(dst, (uint64_t)nbytes, src, (uint64_t)nbytes))
        return SE_ERR_LAYOUT;
    if (nbytes == 0) return SE_OK;
    const hipError_t e = se::launch_calib_copy(dst, src, (uint64_t)nbytes, g_nontemporal.load(),
                                               (hipStream_t)stream);
    return e == hipSuccess ? SE_OK : hip_fail("se_calib_copy launch", e);
}

int se_calib_oneway(void *dst, const void *src, int64_t nbytes, int direction, void *stream)
{
    if (nbytes < 0 || (direction != 1 && direction != 2)) return SE_ERR_ARG;
    if (!dst || !src) return SE_ERR_NULL;
    if ((uintptr_t)dst % 16 || (uintptr_t)src % 16 || nbytes % 16 || nbytes >= ((int64_t)1 << 37) ||
        overlaps(dst, (uint64_t)nbytes, src, (uint64_t)nbytes))
        return SE_ERR_LAYOUT;
    if (nbytes == 0) return SE_OK;
    const hipError_t e = se::launch_calib_oneway(dst, src, (uint64_t)nbytes, direction, (hipStream_t)stream);
    return e == hipSuccess ? SE_OK : hip_fail("se_calib_oneway launch", e);
}

int se_set_seed(uint64_t seed) { g_seed.store(seed); return SE_OK; }
uint64_t se_get_seed(void) { return g_seed.load(); }

int64_t se_pitch(int64_t P)
{
    if (P < 0) return -1;
    return (P + 1023) / 1024 * 1024;
}

int64_t se_step_bytes(int64_t columns, int n, int grad_elem_bytes, int has_momentum)
{
    if (columns < 0 || n < 0 || (grad_elem_bytes != 2 && grad_elem_bytes != 4)) return -1;
    return (int64_t)n * columns * (8 + grad_elem_bytes + (has_momentum ? 8 : 0));
}

int se_set_tuning(const char *name, int value)
{
    if (!name) return SE_ERR_NULL;
    for (const Knob &k : kKnobs) {
        if (std::strcmp(name, k.name)) continue;
        if (value < k.lo || value > k.hi) return SE_ERR_ARG;
        k.value->store(value);
        return SE_OK;
    }
    return SE_ERR_ARG;
}

int se_get_tuning(const char *name)
{
    if (!name) return SE_ERR_NULL;
    for (const Knob &k : kKnobs)
        if (!std::strcmp(name, k.name)) return k.value->load();
    return SE_ERR_ARG;
}

const char *se_strerror(int code)
{
    switch (code) {
    case SE_OK: return "success";
    case SE_ERR_ARG: return "invalid argument (n, group_size, iter, layer range, flags or a size out of range)";
    case SE_ERR_DIVISIBILITY: return "n is not a multiple of group_size (only equal groups are defined)";
    case SE_ERR_NULL: return "a required pointer is NULL (momentum may be NULL only when mu == 0)";
    case SE_ERR_LAYOUT: return "bad layout (layer offsets not monotone from 0, buffers overlap or are misaligned)";
    case SE_ERR_UNSUPPORTED: return "unsupported size (more than 64 workers, or rows of 2^30 elements or more)";
    case SE_ERR_HIP: return "a HIP call failed (see se_last_error)";
    default: return "unknown error code";
    }
}

const char *se_last_error(void) { return t_last_error; }

}  // extern "C"

// C ABI of the SESGD step library (see include/sesgd.h): argument validation on the host,
// choice of the launch shape, kernel launch on the caller's stream.  No torch types, no
// CPU fallback: every step of the method runs in the HIP kernels.
#include "se_common.hpp"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/sesgd.h"

namespace {

std::atomic<uint64_t> g_seed{0};
std::atomic<int> g_blocks_per_cu{0};     // ring kernel: grid-stride blocks per CU (0 = one per tile)
std::atomic<int> g_group_major{1};
std::atomic<int> g_nontemporal{3};
std::atomic<int> g_block_threads{64};
std::atomic<int> g_tiles_per_block{1};
std::atomic<int> g_max_blocks_per_cu{8};
std::atomic<int> g_coop_min_rows{8};      // rows reduced together from which the LDS form is used (0 = never)  // step kernel: resident workgroups per CU (0 = no cap)

thread_local char t_last_error[256] = "";

int hip_fail(const char *what, hipError_t e)
{
    std::snprintf(t_last_error, sizeof t_last_error, "%s: %s", what, hipGetErrorString(e));
    return SE_ERR_HIP;
}

int compute_units()
{
    static std::mutex mu;
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

bool overlaps(const void *a, uint64_t abytes, const void *b, uint64_t bbytes)
{
    if (!a || !b || abytes == 0 || bbytes == 0) return false;
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

struct Layout {
    int64_t pitch;
    int vec;
};

// Everything that can be rejected without touching the device.
int validate(const void *params, const void *grads, const void *momentum,
             const int64_t *layer_offsets, int num_layers, int n, int group_size, int64_t iter,
             float mu, int grad_bytes, Layout *out)
{
    if (n < 1 || group_size < 1 || group_size > n || iter < 0 || num_layers < 0) return SE_ERR_ARG;
    if (n % group_size != 0) return SE_ERR_DIVISIBILITY;
    if (!params || !grads || !layer_offsets) return SE_ERR_NULL;
    if (!momentum && mu != 0.0f) return SE_ERR_NULL;
    if (layer_offsets[0] != 0) return SE_ERR_LAYOUT;
    for (int l = 0; l < num_layers; ++l)
        if (layer_offsets[l + 1] < layer_offsets[l]) return SE_ERR_LAYOUT;
    const int64_t pitch = layer_offsets[num_layers];
    if (n > SE_MAX_WORKERS || pitch >= ((int64_t)1 << 30)) return SE_ERR_UNSUPPORTED;
    const uintptr_t px = (uintptr_t)params, pg = (uintptr_t)grads, pv = (uintptr_t)momentum;
    if (px % 4 || pv % 4 || pg % (uintptr_t)grad_bytes) return SE_ERR_LAYOUT;
    const uint64_t fbytes = (uint64_t)n * (uint64_t)pitch * 4u;
    const uint64_t gbytes = (uint64_t)n * (uint64_t)pitch * (uint64_t)grad_bytes;
    if (overlaps(params, fbytes, grads, gbytes) || overlaps(params, fbytes, momentum, fbytes) ||
        overlaps(grads, gbytes, momentum, fbytes))
        return SE_ERR_LAYOUT;
    // widest access for which every row of every buffer starts aligned
    int vec = 1;
    for (int cand = 4; cand > 1; cand >>= 1) {
        const uintptr_t fa = (uintptr_t)cand * 4u, ga = (uintptr_t)cand * (uintptr_t)grad_bytes;
        if (pitch % cand == 0 && px % fa == 0 && pv % fa == 0 && pg % ga == 0) { vec = cand; break; }
    }
    out->pitch = pitch;
    out->vec = vec;
    return SE_OK;
}

uint32_t grid_for(uint64_t ntasks)
{
    const int bpc = g_blocks_per_cu.load();
    uint64_t grid = ntasks;
    if (bpc > 0) {
        const uint64_t cap = (uint64_t)compute_units() * (uint64_t)bpc;
        if (grid > cap) grid = cap;
    }
    if (grid > 0x7FFFFFFFull) grid = 0x7FFFFFFFull;
    return (uint32_t)grid;
}

int step_impl(float *params, const void *grads, float *momentum, const int64_t *layer_offsets,
              int num_layers, int n, int group_size, int64_t iter, float lr, float mu,
              void *stream, int grad_bytes)
{
    Layout lay;
    const int rc = validate(params, grads, momentum, layer_offsets, num_layers, n, group_size,
                            iter, mu, grad_bytes, &lay);
    if (rc != SE_OK) return rc;
    if (lay.pitch == 0) return SE_OK;

    se::StepArgs a;
    a.x = params; a.g = grads; a.v = momentum;
    a.seed = g_seed.load(); a.iter = iter;
    a.pitch_bytes = (uint64_t)lay.pitch * 4u;
    se::LaunchShape s;
    s.vec = lay.vec; s.bf16 = grad_bytes == 2; s.nontemporal = g_nontemporal.load();
    s.block = g_block_threads.load();
    const int cap = g_max_blocks_per_cu.load();
    s.lds_bytes = cap > 0 ? (se::kLdsPerCu / (uint32_t)cap) & ~1023u : 0u;

    a.nvec = (uint32_t)(lay.pitch / lay.vec);
    a.tiles = (a.nvec + (uint32_t)s.block - 1) / (uint32_t)s.block;
    a.tiles_per_block = (uint32_t)g_tiles_per_block.load();
    a.chunks = (a.tiles + a.tiles_per_block - 1) / a.tiles_per_block;
    a.n = n; a.m = group_size; a.k = n / group_size;
    a.neg_lr = -lr; a.mu = mu; a.inv_m = 1.0f / (float)group_size;
    a.group_major = g_group_major.load();
    s.grid = a.chunks * (uint32_t)a.k;        // < 2^30 / 64 * 64 workgroups
    const int coop = g_coop_min_rows.load();
    hipError_t e;
    if (coop > 0 && group_size >= coop) {
        a.tiles = (a.nvec + 63u) / 64u;
        s.grid = a.tiles * (uint32_t)a.k;
        e = se::launch_coop_step(a, s, (hipStream_t)stream);
    } else {
        e = se::launch_step(a, s, (hipStream_t)stream);
    }
    return e == hipSuccess ? SE_OK : hip_fail("se_step launch", e);
}

int ring_impl(float *params, const void *grads, float *momentum, const int64_t *layer_offsets,
              int num_layers, int n, float lr, float mu, void *stream, int grad_bytes)
{
    Layout lay;
    const int rc = validate(params, grads, momentum, layer_offsets, num_layers, n, 1, 0, mu,
                            grad_bytes, &lay);
    if (rc != SE_OK) return rc;
    if (lay.pitch == 0) return SE_OK;

    se::RingArgs a;
    a.x = params; a.g = grads; a.v = momentum;
    a.pitch_bytes = (uint64_t)lay.pitch * 4u;
    se::LaunchShape s;
    s.vec = lay.vec; s.bf16 = grad_bytes == 2; s.nontemporal = g_nontemporal.load();
    s.block = g_block_threads.load();
    const int cap = g_max_blocks_per_cu.load();
    s.lds_bytes = cap > 0 ? (se::kLdsPerCu / (uint32_t)cap) & ~1023u : 0u;
    a.nvec = (uint32_t)(lay.pitch / lay.vec);
    a.tiles = (a.nvec + (uint32_t)s.block - 1) / (uint32_t)s.block;
    a.n = n;
    a.neg_lr = -lr; a.mu = mu; a.inv_n = 1.0f / (float)n;
    s.grid = grid_for(a.tiles);
    const int coop = g_coop_min_rows.load();
    hipError_t e;
    if (coop > 0 && n >= coop) {
        se::StepArgs c;
        c.x = params; c.g = grads; c.v = momentum;
        c.seed = 0; c.iter = 0;
        c.pitch_bytes = a.pitch_bytes; c.nvec = a.nvec;
        c.tiles = (a.nvec + 63u) / 64u; c.tiles_per_block = 1; c.chunks = c.tiles;
        c.n = n; c.m = n; c.k = 1;
        c.neg_lr = -lr; c.mu = mu; c.inv_m = a.inv_n;
        c.group_major = 1;
        s.grid = c.tiles;
        e = se::launch_coop_ring(c, s, (hipStream_t)stream);
    } else {
        e = se::launch_ring(a, s, (hipStream_t)stream);
    }
    return e == hipSuccess ? SE_OK : hip_fail("se_ring_step launch", e);
}

int plan_check(int n, int group_size, int64_t iter, const void *group_of)
{
    if (n < 1 || group_size < 1 || group_size > n || iter < 0) return SE_ERR_ARG;
    if (n % group_size != 0) return SE_ERR_DIVISIBILITY;
    if (!group_of) return SE_ERR_NULL;
    if (n > SE_MAX_WORKERS) return SE_ERR_UNSUPPORTED;
    return SE_OK;
}

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
    return step_impl(params, grads, momentum, layer_offsets, num_layers, n, group_size, iter,
                     lr, mu, stream, 4);
}

int se_step_bf16g(float *params, const uint16_t *grads_bf16, float *momentum,
                  const int64_t *layer_offsets, int num_layers, int n, int group_size,
                  int64_t iter, float lr, float mu, void *stream)
{
    return step_impl(params, grads_bf16, momentum, layer_offsets, num_layers, n, group_size,
                     iter, lr, mu, stream, 2);
}

int se_ring_step(float *params, const float *grads, float *momentum, const int64_t *layer_offsets,
                 int num_layers, int n, float lr, float mu, void *stream)
{
    return ring_impl(params, grads, momentum, layer_offsets, num_layers, n, lr, mu, stream, 4);
}

int se_ring_step_bf16g(float *params, const uint16_t *grads_bf16, float *momentum,
                       const int64_t *layer_offsets, int num_layers, int n, float lr, float mu,
                       void *stream)
{
    return ring_impl(params, grads_bf16, momentum, layer_offsets, num_layers, n, lr, mu, stream, 2);
}

int se_calib_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (nbytes < 0) return SE_ERR_ARG;
    if (!dst || !src) return SE_ERR_NULL;
    if ((uintptr_t)dst % 16 || (uintptr_t)src % 16 || nbytes % 16 || nbytes >= ((int64_t)1 << 37) ||
        overlaps(dst, (uint64_t)nbytes, src, (uint64_t)nbytes))
        return SE_ERR_LAYOUT;
    if (nbytes == 0) return SE_OK;
    const hipError_t e = se::launch_calib_copy(dst, src, (uint64_t)nbytes, (hipStream_t)stream);
    return e == hipSuccess ? SE_OK : hip_fail("se_calib_copy launch", e);
}

int se_set_seed(uint64_t seed) { g_seed.store(seed); return SE_OK; }
uint64_t se_get_seed(void) { return g_seed.load(); }

int64_t se_pitch(int64_t P)
{
    if (P < 0) return -1;
    return (P + 63) / 64 * 64;
}

int64_t se_step_bytes(int64_t pitch, int n, int grad_elem_bytes, int has_momentum)
{
    if (pitch < 0 || n < 0 || (grad_elem_bytes != 2 && grad_elem_bytes != 4)) return -1;
    return (int64_t)n * pitch * (8 + grad_elem_bytes + (has_momentum ? 8 : 0));
}

int se_set_tuning(const char *name, int value)
{
    if (!name) return SE_ERR_NULL;
    if (!std::strcmp(name, "grid_blocks_per_cu")) {
        if (value < 0 || value > 4096) return SE_ERR_ARG;
        g_blocks_per_cu.store(value); return SE_OK;
    }
    if (!std::strcmp(name, "group_major")) {
        if (value < 0 || value > 1) return SE_ERR_ARG;
        g_group_major.store(value); return SE_OK;
    }
    if (!std::strcmp(name, "block_threads")) {
        if (value != 64 && value != 128 && value != 256) return SE_ERR_ARG;
        g_block_threads.store(value); return SE_OK;
    }
    if (!std::strcmp(name, "tiles_per_block")) {
        if (value < 1 || value > 65536) return SE_ERR_ARG;
        g_tiles_per_block.store(value); return SE_OK;
    }
    if (!std::strcmp(name, "max_blocks_per_cu")) {
        if (value < 0 || value > 32) return SE_ERR_ARG;
        g_max_blocks_per_cu.store(value); return SE_OK;
    }
    if (!std::strcmp(name, "coop_min_rows")) {
        if (value < 0 || value > 65) return SE_ERR_ARG;
        g_coop_min_rows.store(value); return SE_OK;
    }
    if (!std::strcmp(name, "nontemporal")) {
        if (value < 0 || value > 3) return SE_ERR_ARG;
        g_nontemporal.store(value); return SE_OK;
    }
    return SE_ERR_ARG;
}

int se_get_tuning(const char *name)
{
    if (!name) return SE_ERR_NULL;
    if (!std::strcmp(name, "grid_blocks_per_cu")) return g_blocks_per_cu.load();
    if (!std::strcmp(name, "group_major")) return g_group_major.load();
    if (!std::strcmp(name, "nontemporal")) return g_nontemporal.load();
    if (!std::strcmp(name, "block_threads")) return g_block_threads.load();
    if (!std::strcmp(name, "tiles_per_block")) return g_tiles_per_block.load();
    if (!std::strcmp(name, "max_blocks_per_cu")) return g_max_blocks_per_cu.load();
    if (!std::strcmp(name, "coop_min_rows")) return g_coop_min_rows.load();
    return SE_ERR_ARG;
}

const char *se_strerror(int code)
{
    switch (code) {
    case SE_OK: return "success";
    case SE_ERR_ARG: return "invalid argument (n, group_size, iter or num_layers out of range)";
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

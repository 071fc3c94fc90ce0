/* Plain C user of the C ABI: no Python, no torch.  Allocates with the HIP runtime, runs
 * se_plan / se_plan_noalloc / se_step / se_ring_step / se_step_ex (ranges from se_layer_buckets) /
 * se_global_average / se_consensus on a small
 * ragged problem and compares every result with the CPU oracle (linked in from oracle/, which
 * is why this program lives with the tests).  Exit status 0 = all equal.
 * Built by __graft_entry__.build(); run by tests/test_gpu_c_abi.py on the GPU machine. */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/sesgd.h"
#include "../../oracle/se_oracle.c"

#define HIPCHECK(call)                                                                   \
    do { hipError_t e_ = (call); if (e_ != hipSuccess) {                                 \
        fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define SECHECK(call)                                                                    \
    do { int rc_ = (call); if (rc_ != SE_OK) {                                           \
        fprintf(stderr, "%s -> %d (%s) %s\n", #call, rc_, se_strerror(rc_), se_last_error()); return 3; } } while (0)

static uint32_t lcg_state = 12345u;
static float draw(float scale)
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((float)(int32_t)(lcg_state >> 8) / 8388608.0f - 1.0f) * scale;
}

static int same_bits(const float *a, const float *b, size_t count, const char *what)
{
    if (memcmp(a, b, count * sizeof(float)) != 0) {
        fprintf(stderr, "MISMATCH in %s\n", what);
        return 1;
    }
    return 0;
}

int main(void)
{
    enum { N = 12, M = 4, L = 4 };
    const int64_t offs[L + 1] = {0, 37, 37, 1061, 2500};     /* ragged, one empty layer */
    const int64_t pitch = offs[L];
    const size_t count = (size_t)N * (size_t)pitch, bytes = count * sizeof(float);
    float *hx = malloc(bytes), *hv = malloc(bytes), *hg = malloc(bytes), *back = malloc(bytes);
    float *dx, *dv, *dg;
    double *dout, hout[2], want[2];
    int32_t group_of[N], members[N], o_group_of[N], o_members[N];
    int bad = 0, t;
    size_t i;

    for (i = 0; i < count; ++i) { hx[i] = draw(0.05f); hv[i] = draw(0.01f); }
    HIPCHECK(hipMalloc((void **)&dx, bytes));
    HIPCHECK(hipMalloc((void **)&dv, bytes));
    HIPCHECK(hipMalloc((void **)&dg, bytes));
    HIPCHECK(hipMalloc((void **)&dout, 2 * sizeof(double)));
    HIPCHECK(hipMemcpy(dx, hx, bytes, hipMemcpyHostToDevice));
    HIPCHECK(hipMemcpy(dv, hv, bytes, hipMemcpyHostToDevice));
    SECHECK(se_set_seed(42));

    for (t = 0; t < 4; ++t) {
        for (i = 0; i < count; ++i) hg[i] = draw(0.01f);
        HIPCHECK(hipMemcpy(dg, hg, bytes, hipMemcpyHostToDevice));
        SECHECK(se_plan(N, M, t, group_of, members));
        if (oracle_plan(42, N, M, t, NULL, NULL, o_group_of, o_members) != 0) return 4;
        if (memcmp(group_of, o_group_of, sizeof group_of) || memcmp(members, o_members, sizeof members)) {
            fprintf(stderr, "MISMATCH in plan, iter %d\n", t);
            ++bad;
        }
        SECHECK(se_plan_noalloc(N, M, t, group_of, members));       /* the form that allocates nothing */
        if (memcmp(group_of, o_group_of, sizeof group_of) || memcmp(members, o_members, sizeof members)) {
            fprintf(stderr, "MISMATCH in plan (no allocation), iter %d\n", t);
            ++bad;
        }
        switch (t) {
        case 0:
            SECHECK(se_step(dx, dg, dv, offs, L, N, M, t, 0.1f, 0.9f, NULL));
            if (oracle_step(hx, hg, 0, hv, pitch, 0, pitch, N, M, 42, t, 0.1f, 0.9f)) return 4;
            break;
        case 1:
            SECHECK(se_ring_step(dx, dg, dv, offs, L, N, 0.1f, 0.9f, NULL));
            if (oracle_ring_step(hx, hg, 0, hv, pitch, 0, pitch, N, 0.1f, 0.9f)) return 4;
            break;
        case 2: {    /* layer ranges of at least 1000 elements, back to front; weight decay */
            int32_t first[L];
            int ranges = -1, r, end = L;
            SECHECK(se_layer_buckets(offs, L, 1000, first, L, &ranges));
            if (ranges != 3 || first[0] != 3 || first[1] != 2 || first[2] != 0) {
                fprintf(stderr, "MISMATCH in layer buckets: %d ranges\n", ranges);
                ++bad;
            }
            for (r = 0; r < ranges; ++r) {
                SECHECK(se_step_ex(dx, dg, 0, dv, offs, L, first[r], end, N, M, t, 0.1f, 0.9f, 5e-4f, 0u, NULL));
                end = first[r];
            }
            if (oracle_step_ex(hx, hg, 0, hv, pitch, 0, pitch, N, M, 42, t, 0.1f, 0.9f, 5e-4f, 0u)) return 4;
            break;
        }
        default:     /* the uncorrected variant */
            SECHECK(se_step_ex(dx, dg, 0, dv, offs, L, 0, L, N, M, t, 0.1f, 0.9f, 0.0f, SE_FLAG_GRAD_AVG, NULL));
            if (oracle_step_ex(hx, hg, 0, hv, pitch, 0, pitch, N, M, 42, t, 0.1f, 0.9f, 0.0f, 1u)) return 4;
            break;
        }
        HIPCHECK(hipDeviceSynchronize());
        HIPCHECK(hipMemcpy(back, dx, bytes, hipMemcpyDeviceToHost));
        bad += same_bits(back, hx, count, "params");
        HIPCHECK(hipMemcpy(back, dv, bytes, hipMemcpyDeviceToHost));
        bad += same_bits(back, hv, count, "momentum");
    }

    SECHECK(se_consensus(dx, offs, L, N, dout, NULL));
    HIPCHECK(hipMemcpy(hout, dout, sizeof hout, hipMemcpyDeviceToHost));
    if (oracle_consensus(hx, pitch, 0, pitch, N, want)) return 4;
    if (hout[0] < want[0] * (1 - 1e-10) || hout[0] > want[0] * (1 + 1e-10) ||
        hout[1] < want[1] - 1e-9 || hout[1] > want[1] + 1e-9) {
        fprintf(stderr, "MISMATCH in consensus: %.17g %.17g vs %.17g %.17g\n", hout[0], hout[1], want[0], want[1]);
        ++bad;
    }
    SECHECK(se_global_average(dx, offs, L, N, NULL));
    if (oracle_global_average(hx, pitch, 0, pitch, N)) return 4;
    HIPCHECK(hipMemcpy(back, dx, bytes, hipMemcpyDeviceToHost));
    bad += same_bits(back, hx, count, "global average");
    if (se_step(dx, dg, dv, offs, L, N, 5, 0, 0.1f, 0.9f, NULL) != SE_ERR_DIVISIBILITY) ++bad;

    HIPCHECK(hipFree(dx)); HIPCHECK(hipFree(dv)); HIPCHECK(hipFree(dg)); HIPCHECK(hipFree(dout));
    free(hx); free(hv); free(hg); free(back);
    printf("c_abi_check: %d mismatches\n", bad);
    return bad ? 1 : 0;
}

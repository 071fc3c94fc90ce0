/* Runs every oracle function on exactly-sized heap buffers so that an out-of-bounds access,
 * an uninitialised index or signed overflow trips AddressSanitizer / UBSan.
 * Built by tests/test_host_sanitizers.py. */
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/se_oracle.c"

int main(void)
{
    int fails = 0, n, m;
    for (n = 1; n <= 64; n += (n < 8 ? 1 : 7)) {
        for (m = 1; m <= n; ++m) {
            int64_t pitch = 37, e;
            float *x, *v, *g;
            uint16_t *gb;
            int32_t *go, *mem, *rank;
            uint32_t *keys;
            double out[2];
            if (n % m) continue;
            x = malloc(sizeof(float) * n * pitch); v = malloc(sizeof(float) * n * pitch);
            g = malloc(sizeof(float) * n * pitch); gb = malloc(sizeof(uint16_t) * n * pitch);
            go = malloc(sizeof(int32_t) * n); mem = malloc(sizeof(int32_t) * n);
            rank = malloc(sizeof(int32_t) * n); keys = malloc(sizeof(uint32_t) * n);
            for (e = 0; e < n * pitch; ++e) { x[e] = 0.01f * (float)(e % 97); v[e] = 0.0f; g[e] = 0.001f * (float)(e % 13); gb[e] = (uint16_t)(0x3A00 + e % 64); }
            fails += oracle_plan(3, n, m, 1234567890123LL, keys, rank, go, mem) != 0;
            fails += oracle_step(x, g, 0, v, pitch, 0, pitch, n, m, 3, 5, 0.1f, 0.9f) != 0;
            fails += oracle_step(x, gb, 1, NULL, pitch, 3, 30, n, m, 3, 6, 0.1f, 0.0f) != 0;
            fails += oracle_ring_step(x, g, 0, v, pitch, 0, pitch, n, 0.1f, 0.9f) != 0;
            fails += oracle_step_ex(x, gb, 1, v, pitch, 1, pitch, n, m, 3, 7, 0.1f, 0.9f, 1e-4f, 1u) != 0;
            fails += oracle_step_ex(x, g, 0, v, pitch, 0, pitch - 1, n, m, 3, 8, 0.1f, 0.9f, 1e-4f, 0u) != 0;
            fails += oracle_global_average(x, pitch, 0, pitch, n) != 0;
            fails += oracle_consensus(x, pitch, 0, pitch, n, out) != 0;
            fails += out[0] != 0.0;
            free(x); free(v); free(g); free(gb); free(go); free(mem); free(rank); free(keys);
        }
    }
    fails += oracle_plan(0, 64, 8, INT64_MAX, NULL, NULL, (int32_t[64]){0}, NULL) != 0;
    fails += oracle_plan(0, 6, 4, 0, NULL, NULL, (int32_t[8]){0}, NULL) != ORACLE_ERR_DIVISIBILITY;
    printf("oracle sanitizer run: %d failures\n", fails);
    return fails ? 1 : 0;
}

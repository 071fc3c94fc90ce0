/*
 * CPU oracle for the Shuffle-Exchange SGD (SESGD) step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU library computes.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg, and
 * by nothing else.  It shares no code, header, table or constant generator with the
 * HIP sources and must never be linked into, or called from, the product path.
 *
 * Every function evaluates the paper's definition directly, one element at a time,
 * in fp32 with a fixed evaluation order, round-to-nearest-even, no contraction other
 * than the two explicit fmaf() calls, no flush-to-zero.  Build with
 *     gcc -O2 -ffp-contract=off -shared -fPIC
 *
 * What follows the paper and what is this build's convention:
 *   - Regrouping (Sec. 3.1 "Shuffle-Exchange"; Algorithm 1, the "randomly generate new
 *     groups depending on the seed" step): the paper fixes only that every worker derives
 *     the same random partition into k equal groups from a shared seed, and (appendix,
 *     proof of the lemma) that two workers are separated with probability
 *     n(k-1)/(k(n-1)), i.e. the partition is uniform.  The hash below that realises it
 *     is a convention of this build; its bits are not pinned by the paper.
 *   - Update (Sec. 3.2 "Gradient Correction", the SESGD update equation; Algorithm 1):
 *     local step into x-hat, then the mean of x-hat over the worker's group.  The factor
 *     k/n of the equation is 1/group_size.
 *   - Momentum (Sec. 4.1 hyper-parameters: "0.9"): v <- mu*v + g, x-hat = x - lr*v,
 *     one buffer per worker, never averaged (Algorithm 1 all-reduces x-hat only).
 *   - Baseline (Sec. 3.2, the DSGD equation): mean gradient over all n workers, the same
 *     update on every worker.
 *   - Summation order (paper is silent; a convention of this build, the same wherever rows
 *     are reduced): the members in ascending worker id are cut into consecutive blocks of 8
 *     (the last one may be shorter), each block is summed left to right, then the block sums
 *     are added left to right.  Up to 8 members that is the plain left-to-right sum.  A
 *     left-to-right sum of 64 values of the size of x would put group_size = n = 64 further
 *     than 1e-6 from the DSGD equation it must reduce to (Sec. 3.2).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_DIVISIBILITY (-2)
#define ORACLE_MAX_N 4096

/* 32-bit finaliser: xor-shift / odd-multiply rounds.  Multipliers are the first 32
 * fractional bits of sqrt(2) and sqrt(3); the additive constant is floor(2^32/phi). */
static uint32_t mix32(uint32_t z)
{
    z ^= z >> 16;
    z *= 0x6A09E667u;
    z ^= z >> 15;
    z *= 0xBB67AE85u;
    z ^= z >> 16;
    return z;
}

/* Sort key of worker i at iteration iter: absorb the six words
 * (seed low, seed high, iter low, iter high, n, i) one after the other. */
uint32_t oracle_key(uint64_t seed, int64_t iter, int n, int i)
{
    const uint32_t golden = 0x9E3779B9u;
    uint64_t t = (uint64_t)iter;
    uint32_t w[6];
    uint32_t h = golden;
    int q;
    w[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    w[1] = (uint32_t)(seed >> 32);
    w[2] = (uint32_t)(t & 0xFFFFFFFFu);
    w[3] = (uint32_t)(t >> 32);
    w[4] = (uint32_t)n;
    w[5] = (uint32_t)i;
    for (q = 0; q < 6; ++q)
        h = mix32((h ^ w[q]) + golden);
    return h;
}

/*
 * Regrouping for one iteration (Sec. 3.1; Algorithm 1).
 *   rank[i]     = number of workers whose (key, id) pair is lexicographically smaller
 *   group_of[i] = rank[i] / m
 *   members[g*m + r] = r-th smallest worker id of group g
 * keys, rank, members may be NULL.  Returns 0, or a negative error.
 */
int oracle_plan(uint64_t seed, int n, int m, int64_t iter,
                uint32_t *keys, int32_t *rank, int32_t *group_of, int32_t *members)
{
    uint32_t key_buf[ORACLE_MAX_N];
    int i, j;
    if (n < 1 || n > ORACLE_MAX_N || m < 1 || m > n || iter < 0 || group_of == NULL)
        return ORACLE_ERR_ARG;
    if (n % m != 0)
        return ORACLE_ERR_DIVISIBILITY;
    for (i = 0; i < n; ++i)
        key_buf[i] = oracle_key(seed, iter, n, i);
    for (i = 0; i < n; ++i) {
        int below = 0;
        for (j = 0; j < n; ++j) {
            if (key_buf[j] < key_buf[i] || (key_buf[j] == key_buf[i] && j < i))
                ++below;
        }
        if (keys) keys[i] = key_buf[i];
        if (rank) rank[i] = below;
        group_of[i] = below / m;
    }
    if (members) {
        int k = n / m, g;
        for (g = 0; g < k; ++g) {
            int r = 0;
            for (i = 0; i < n; ++i)          /* ascending worker id */
                if (group_of[i] == g)
                    members[g * m + r++] = i;
        }
    }
    return ORACLE_OK;
}

/* The fixed summation order: blocks of ORACLE_BLOCK consecutive values left to right, then
 * the block sums left to right.  val[0..m-1] are in ascending worker id. */
#define ORACLE_BLOCK 8
static float sum_in_order(const float *val, int m)
{
    float total = 0.0f;
    int b, r;
    for (b = 0; b < m; b += ORACLE_BLOCK) {
        float part = val[b];
        for (r = b + 1; r < m && r < b + ORACLE_BLOCK; ++r)
            part = part + val[r];
        total = (b == 0) ? part : total + part;
    }
    return total;
}

/* bf16 -> fp32 is exact: the 16 bits are the high half of the fp32 pattern. */
static float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static float load_grad(const void *grads, int grads_are_bf16, int64_t idx)
{
    if (grads_are_bf16)
        return bf16_to_f32(((const uint16_t *)grads)[idx]);
    return ((const float *)grads)[idx];
}

/*
 * One SESGD iteration on columns [col_begin, col_end) of n replica rows of length
 * `pitch` (Sec. 3.2, the SESGD update equation; Algorithm 1 body).
 *
 *   for every group G of this iteration's plan, every column e:
 *     for members j of G in ascending id:
 *        v'      = momentum ? fmaf(mu, momentum[j][e], g[j][e]) : g[j][e]
 *        xhat[j] = fmaf(-lr, v', params[j][e])
 *     s    = the xhat[j] summed in the fixed order (blocks of 8, then the block sums)
 *     mean = s * (1.0f / (float)m)
 *     params[j][e] = mean for every member j;  momentum[j][e] = v'
 *
 * momentum may be NULL (plain SGD; mu is then ignored).
 */
int oracle_step(float *params, const void *grads, int grads_are_bf16, float *momentum,
                int64_t pitch, int64_t col_begin, int64_t col_end,
                int n, int m, uint64_t seed, int64_t iter, float lr, float mu)
{
    int32_t group_of[ORACLE_MAX_N];
    int32_t members[ORACLE_MAX_N];
    float xhat[ORACLE_MAX_N];
    int rc, g, r, k;
    int64_t e;
    float inv_m;
    if (params == NULL || grads == NULL || pitch < 0 || col_begin < 0 ||
        col_end < col_begin || col_end > pitch)
        return ORACLE_ERR_ARG;
    rc = oracle_plan(seed, n, m, iter, NULL, NULL, group_of, members);
    if (rc != ORACLE_OK)
        return rc;
    k = n / m;
    inv_m = 1.0f / (float)m;
    for (g = 0; g < k; ++g) {
        const int32_t *mem = members + (size_t)g * m;
        for (e = col_begin; e < col_end; ++e) {
            float mean;
            for (r = 0; r < m; ++r) {
                int64_t idx = (int64_t)mem[r] * pitch + e;
                float gg = load_grad(grads, grads_are_bf16, idx);
                float vn;
                if (momentum) {
                    vn = fmaf(mu, momentum[idx], gg);
                    momentum[idx] = vn;
                } else {
                    vn = gg;
                }
                xhat[r] = fmaf(-lr, vn, params[idx]);
            }
            mean = sum_in_order(xhat, m) * inv_m;
            for (r = 0; r < m; ++r)
                params[(int64_t)mem[r] * pitch + e] = mean;
        }
    }
    return ORACLE_OK;
}

/*
 * One Ring-SGD (fully synchronous DSGD) iteration (Sec. 3.2, the DSGD equation):
 *   gbar = (g[0][e], g[1][e], ..., g[n-1][e] summed in the fixed order) * (1.0f / (float)n)
 *   v'   = momentum ? fmaf(mu, momentum[i][e], gbar) : gbar
 *   params[i][e] = fmaf(-lr, v', params[i][e])          for every worker i
 */
int oracle_ring_step(float *params, const void *grads, int grads_are_bf16, float *momentum,
                     int64_t pitch, int64_t col_begin, int64_t col_end,
                     int n, float lr, float mu)
{
    float gcol[ORACLE_MAX_N];
    int i;
    int64_t e;
    float inv_n;
    if (params == NULL || grads == NULL || n < 1 || n > ORACLE_MAX_N || pitch < 0 || col_begin < 0 ||
        col_end < col_begin || col_end > pitch)
        return ORACLE_ERR_ARG;
    inv_n = 1.0f / (float)n;
    for (e = col_begin; e < col_end; ++e) {
        float gbar;
        for (i = 0; i < n; ++i)
            gcol[i] = load_grad(grads, grads_are_bf16, (int64_t)i * pitch + e);
        gbar = sum_in_order(gcol, n) * inv_n;
        for (i = 0; i < n; ++i) {
            int64_t idx = (int64_t)i * pitch + e;
            float vn;
            if (momentum) {
                vn = fmaf(mu, momentum[idx], gbar);
                momentum[idx] = vn;
            } else {
                vn = gbar;
            }
            params[idx] = fmaf(-lr, vn, params[idx]);
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Extensions beyond the basic step.  Same conventions as above.
 * ------------------------------------------------------------------------------------ */

#define ORACLE_FLAG_GRAD_AVG 1u

/*
 * General step on columns [col_begin, col_end).
 *
 * weight_decay (Sec. 4.1 hyper-parameters list 5e-4 / 1e-4; the paper gives no formula, the
 * convention of the SGD optimizer it names is used): the decayed gradient of worker j is
 *     d_j = (wd != 0) ? fmaf(wd, x_j, gsrc) : gsrc
 * and it replaces the gradient in the momentum update.
 *
 * flags == 0: the SESGD update (Sec. 3.2 "Gradient Correction"), gsrc = g_j; identical to
 *   oracle_step when wd == 0.
 * flags & ORACLE_FLAG_GRAD_AVG: the variant the paper rejects (Sec. 3.2: the shuffle applied
 *   directly to the DSGD equation).  The *gradients* are averaged inside the group,
 *     gbar_G = (g_{j0}, g_{j1}, ... summed in the fixed order) * (1.0f/(float)m)   members ascending
 *   and every member updates on its own: gsrc = gbar_G,
 *     v_j = momentum ? fmaf(mu, v_j, d_j) : d_j ;  x_j = fmaf(-lr, v_j, x_j).
 *   Parameters are never averaged, so replicas drift apart (the paper's divergence equation).
 *   With m == n this is exactly oracle_ring_step.
 */
int oracle_step_ex(float *params, const void *grads, int grads_are_bf16, float *momentum,
                   int64_t pitch, int64_t col_begin, int64_t col_end,
                   int n, int m, uint64_t seed, int64_t iter,
                   float lr, float mu, float wd, unsigned flags)
{
    int32_t group_of[ORACLE_MAX_N];
    int32_t members[ORACLE_MAX_N];
    float val[ORACLE_MAX_N];
    int rc, g, r, k;
    int64_t e;
    float inv_m;
    if (params == NULL || grads == NULL || pitch < 0 || col_begin < 0 ||
        col_end < col_begin || col_end > pitch || (flags & ~ORACLE_FLAG_GRAD_AVG))
        return ORACLE_ERR_ARG;
    rc = oracle_plan(seed, n, m, iter, NULL, NULL, group_of, members);
    if (rc != ORACLE_OK)
        return rc;
    k = n / m;
    inv_m = 1.0f / (float)m;
    for (g = 0; g < k; ++g) {
        const int32_t *mem = members + (size_t)g * m;
        for (e = col_begin; e < col_end; ++e) {
            if (flags & ORACLE_FLAG_GRAD_AVG) {
                float gbar;
                for (r = 0; r < m; ++r)
                    val[r] = load_grad(grads, grads_are_bf16, (int64_t)mem[r] * pitch + e);
                gbar = sum_in_order(val, m) * inv_m;
                for (r = 0; r < m; ++r) {
                    int64_t idx = (int64_t)mem[r] * pitch + e;
                    float d = (wd != 0.0f) ? fmaf(wd, params[idx], gbar) : gbar;
                    float vn;
                    if (momentum) {
                        vn = fmaf(mu, momentum[idx], d);
                        momentum[idx] = vn;
                    } else {
                        vn = d;
                    }
                    params[idx] = fmaf(-lr, vn, params[idx]);
                }
            } else {
                float mean;
                for (r = 0; r < m; ++r) {
                    int64_t idx = (int64_t)mem[r] * pitch + e;
                    float gg = load_grad(grads, grads_are_bf16, idx);
                    float d = (wd != 0.0f) ? fmaf(wd, params[idx], gg) : gg;
                    float vn;
                    if (momentum) {
                        vn = fmaf(mu, momentum[idx], d);
                        momentum[idx] = vn;
                    } else {
                        vn = d;
                    }
                    val[r] = fmaf(-lr, vn, params[idx]);
                }
                mean = sum_in_order(val, m) * inv_m;
                for (r = 0; r < m; ++r)
                    params[(int64_t)mem[r] * pitch + e] = mean;
            }
        }
    }
    return ORACLE_OK;
}

/*
 * Final global average (Algorithm 1, last line: x-bar <- Ring-AllReduce(x_i; Global)):
 *   xbar[e] = (x_0[e], x_1[e], ..., x_{n-1}[e] summed in the fixed order) * (1.0f/(float)n),
 *   written to every row.
 */
int oracle_global_average(float *params, int64_t pitch, int64_t col_begin, int64_t col_end, int n)
{
    float xcol[ORACLE_MAX_N];
    int i;
    int64_t e;
    float inv_n;
    if (params == NULL || n < 1 || n > ORACLE_MAX_N || pitch < 0 || col_begin < 0 ||
        col_end < col_begin || col_end > pitch)
        return ORACLE_ERR_ARG;
    inv_n = 1.0f / (float)n;
    for (e = col_begin; e < col_end; ++e) {
        float mean;
        for (i = 0; i < n; ++i)
            xcol[i] = params[(int64_t)i * pitch + e];
        mean = sum_in_order(xcol, n) * inv_n;
        for (i = 0; i < n; ++i)
            params[(int64_t)i * pitch + e] = mean;
    }
    return ORACLE_OK;
}

/*
 * Replica-consistency diagnostics in double precision (the quantity behind the paper's
 * divergence equation of Sec. 3.2 and the "consistency of parameters" figure of Sec. 4.2):
 *   out[0] = sum_e sum_i (x_i[e] - xbar[e])^2   with xbar[e] = (sum_i x_i[e]) / n   (Sec. 3.3)
 *   out[1] = sum_e sum_i x_i[e]                  (the all-worker parameter sum)
 * Columns and rows are visited in ascending order.
 */
int oracle_consensus(const float *params, int64_t pitch, int64_t col_begin, int64_t col_end,
                     int n, double *out)
{
    int i;
    int64_t e;
    double dist = 0.0, total = 0.0;
    if (params == NULL || out == NULL || n < 1 || pitch < 0 || col_begin < 0 ||
        col_end < col_begin || col_end > pitch)
        return ORACLE_ERR_ARG;
    for (e = col_begin; e < col_end; ++e) {
        double s = 0.0, mean, d = 0.0;
        for (i = 0; i < n; ++i)
            s += (double)params[(int64_t)i * pitch + e];
        mean = s / (double)n;
        for (i = 0; i < n; ++i) {
            double t = (double)params[(int64_t)i * pitch + e] - mean;
            d += t * t;
        }
        dist += d;
        total += s;
    }
    out[0] = dist;
    out[1] = total;
    return ORACLE_OK;
}

/*
 * Communication-time model of the paper for one layer of G bytes on a network of bandwidth
 * nu (bytes/s) and latency t_tau (s):
 *   ring over w workers (Sec. 2.2, the all-reduce cost equation): 2 (w-1) (G/(w nu) + t_tau)
 * Ring-SGD uses w = n; SESGD with k groups uses w = n/k (Sec. 3.1; with k = sqrt(n) this is
 * the approximate form 2G/nu + 2 sqrt(n) t_tau of the paper).
 * handshakes: 2 (w-1) per layer (Sec. 2.3 counts 50 * 2 * 15 = 1500 for 50 layers, n = 16).
 */
double oracle_ring_time(double layer_bytes, int workers, double nu, double t_tau)
{
    if (workers < 1 || nu <= 0.0) return -1.0;
    return 2.0 * (double)(workers - 1) * (layer_bytes / ((double)workers * nu) + t_tau);
}

long oracle_handshakes(int layers, int workers)
{
    return (long)layers * 2L * (long)(workers - 1);
}

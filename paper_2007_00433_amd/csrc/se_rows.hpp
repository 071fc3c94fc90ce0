// Row batches shared by the step kernels: B member rows of a group loaded back to back (all
// loads of a batch are in flight together), then the arithmetic, then the stores; and the
// loops that walk a group's members in the library's summation order.
#pragma once

#include "se_device.hpp"

namespace se {

// ---- kSesgd: B members at once -------------------------------------------------------------
template <int VEC, bool BF16, bool HAS_V, bool HAS_WD, int NT, int B, bool FIRST>
__device__ __forceinline__ void sesgd_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                            uint32_t goff, uint64_t gpitch_bytes, Pack<VEC> &s)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) row[b] = next_row(todo);
    Pack<VEC> X[B], G[B], V[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        X[b] = load_f32<VEC, NT>((const char *)p.x + row[b] * p.pitch_bytes + off);
        G[b] = load_grad<VEC, BF16, NT>((const char *)p.g + row[b] * gpitch_bytes + goff);
        if constexpr (HAS_V)
            V[b] = load_f32<VEC, NT>((const char *)p.v + row[b] * p.pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        Pack<VEC> vn;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const float d = HAS_WD ? __builtin_fmaf(p.wd, X[b].a[c], G[b].a[c]) : G[b].a[c];
            vn.a[c] = HAS_V ? __builtin_fmaf(p.mu, V[b].a[c], d) : d;
            const float xhat = __builtin_fmaf(p.neg_lr, vn.a[c], X[b].a[c]);
            s.a[c] = (FIRST && b == 0) ? xhat : s.a[c] + xhat;
        }
        if constexpr (HAS_V)
            store_f32<VEC, NT>((char *)p.v + row[b] * p.pitch_bytes, off, vn);
    }
}

// ---- kGradAvg / kAvgOnly, pass 1: sum one array over B members ---------------------------------
template <int VEC, bool BF16, int NT, bool PARAMS, int B, bool FIRST>
__device__ __forceinline__ void sum_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                          uint64_t pitch_bytes, Pack<VEC> &s)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) row[b] = next_row(todo);
    Pack<VEC> A[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        if constexpr (PARAMS) A[b] = load_f32<VEC, NT>((const char *)p.x + row[b] * pitch_bytes + off);
        else A[b] = load_grad<VEC, BF16, NT>((const char *)p.g + row[b] * pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int c = 0; c < VEC; ++c)
            s.a[c] = (FIRST && b == 0) ? A[b].a[c] : s.a[c] + A[b].a[c];
}

// ---- kGradAvg, pass 2: every member updates with the group's mean gradient ---------------------
template <int VEC, bool HAS_V, bool HAS_WD, int NT, int B, bool FIRST>
__device__ __forceinline__ void update_batch(const StepArgs &p, uint64_t &todo, uint32_t off,
                                             const Pack<VEC> &gbar)
{
    uint64_t row[B];
#pragma unroll
    for (int b = 0; b < B; ++b) row[b] = next_row(todo);
    Pack<VEC> X[B], V[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        X[b] = load_f32<VEC, NT>((const char *)p.x + row[b] * p.pitch_bytes + off);
        if constexpr (HAS_V)
            V[b] = load_f32<VEC, NT>((const char *)p.v + row[b] * p.pitch_bytes + off);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        Pack<VEC> vn, xn;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const float d = HAS_WD ? __builtin_fmaf(p.wd, X[b].a[c], gbar.a[c]) : gbar.a[c];
            vn.a[c] = HAS_V ? __builtin_fmaf(p.mu, V[b].a[c], d) : d;
            xn.a[c] = __builtin_fmaf(p.neg_lr, vn.a[c], X[b].a[c]);
        }
        if constexpr (HAS_V)
            store_f32<VEC, NT>((char *)p.v + row[b] * p.pitch_bytes, off, vn);
        store_f32<VEC, NT>((char *)p.x + row[b] * p.pitch_bytes, off, xn);
    }
}

// Applies CALL(B, FIRST) to all m members in batches of BMAX, then 4, 2, 1 (wave-uniform control
// flow throughout); FIRST is true for the first batch.  For passes that do not add anything up.
#define SE_FOR_MEMBER_BATCHES(BMAX, m, CALL)                                               \
    do {                                                                                   \
        int rem_ = (m);                                                                    \
        bool first_ = true;                                                                \
        if (rem_ >= BMAX) {                                                                \
            CALL(BMAX, true); rem_ -= BMAX; first_ = false;                                \
            while (rem_ >= BMAX) { CALL(BMAX, false); rem_ -= BMAX; }                      \
        }                                                                                  \
        if constexpr (BMAX > 4) { if (rem_ >= 4) {                                         \
            if (first_) { CALL(4, true); } else { CALL(4, false); } rem_ -= 4; first_ = false; } } \
        if constexpr (BMAX > 2) { if (rem_ >= 2) {                                         \
            if (first_) { CALL(2, true); } else { CALL(2, false); } rem_ -= 2; first_ = false; } } \
        if constexpr (BMAX > 1) { if (rem_ >= 1) {                                         \
            if (first_) { CALL(1, true); } else { CALL(1, false); } } }                    \
    } while (0)

// The library's summation order: the m members (ascending worker id) are cut into consecutive
// blocks of kSumBlock = 8, each block is added up left to right, then the block sums are added
// up left to right.  CALL(B, FIRST, acc) must add B members to acc, left to right, starting acc
// afresh when FIRST.  A block is walked in batches of at most BMAX rows: 8, then 4, 2, 1.  The total lands in `total`.
#define SE_SUM_MEMBER_BLOCKS(BMAX, m, VEC_, total, CALL)                                   \
    do {                                                                                   \
        static_assert(BMAX == 8 || BMAX == 4 || BMAX == 2 || BMAX == 1, "batch size");     \
        int rem_ = (m);                                                                    \
        bool first_block_ = true;                                                          \
        while (rem_ > 0) {                                                                 \
            Pack<VEC_> part_;                                                              \
            int blk_ = rem_ < kSumBlock ? rem_ : kSumBlock;                                \
            rem_ -= blk_;                                                                  \
            bool first_ = true;                                                            \
            if constexpr (BMAX >= 8) { if (blk_ == 8) {                                    \
                CALL(8, true, part_); blk_ = 0; first_ = false; } }                        \
            if constexpr (BMAX >= 4) { while (blk_ >= 4) {                                 \
                if (first_) { CALL(4, true, part_); } else { CALL(4, false, part_); }      \
                blk_ -= 4; first_ = false; } }                                             \
            if constexpr (BMAX >= 2) { while (blk_ >= 2) {                                 \
                if (first_) { CALL(2, true, part_); } else { CALL(2, false, part_); }      \
                blk_ -= 2; first_ = false; } }                                             \
            while (blk_ >= 1) {                                                            \
                if (first_) { CALL(1, true, part_); } else { CALL(1, false, part_); }      \
                blk_ -= 1; first_ = false; }                                               \
            _Pragma("unroll")                                                              \
            for (int q_ = 0; q_ < VEC_; ++q_)                                              \
                total.a[q_] = first_block_ ? part_.a[q_] : total.a[q_] + part_.a[q_];      \
            first_block_ = false;                                                          \
        }                                                                                  \
    } while (0)

}  // namespace se

// Device-side building blocks: the regrouping generator evaluated by one wavefront, and
// 128/64/32-bit row accessors addressed as (uniform row base) + (per-lane byte offset).
#pragma once

#include "se_common.hpp"

namespace se {

// ---------------------------------------------------------------- regrouping (Sec. 3.1)
// Every worker must derive the same random partition from the shared seed without
// exchanging messages (Sec. 3.1; Algorithm 1).  Here every wavefront derives it: lane i
// plays worker i, hashes (seed, iter, n, i) to a 32-bit key, and ranks itself among the n
// keys (ties by id).  Consecutive blocks of m ranks form the groups.

__device__ __forceinline__ uint32_t mix32(uint32_t z)
{
    z ^= z >> 16;
    z *= 0x6A09E667u;      // frac(sqrt 2) * 2^32
    z ^= z >> 15;
    z *= 0xBB67AE85u;      // frac(sqrt 3) * 2^32
    z ^= z >> 16;
    return z;
}

__device__ __forceinline__ uint32_t absorb(uint32_t h, uint32_t w)
{
    return mix32((h ^ w) + 0x9E3779B9u);   // 2^32 / golden ratio
}

__device__ __forceinline__ uint32_t worker_key(uint64_t seed, int64_t iter, int n, int i)
{
    uint32_t h = 0x9E3779B9u;
    h = absorb(h, (uint32_t)seed);
    h = absorb(h, (uint32_t)(seed >> 32));
    h = absorb(h, (uint32_t)(uint64_t)iter);
    h = absorb(h, (uint32_t)((uint64_t)iter >> 32));
    h = absorb(h, (uint32_t)n);           // everything above is wave-uniform
    return absorb(h, (uint32_t)i);
}

// Rank of this lane's worker among workers 0..n-1, n <= 64: the number of workers whose
// (key, id) pair is lexicographically smaller, counted with one 64-bit compare per worker.
// Lanes >= n take the largest key, so they never count as smaller (the loop runs over n
// rounded up to 4) and their own result is garbage.
__device__ __forceinline__ uint32_t wave_rank(uint64_t seed, int64_t iter, int n, int lane)
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const uint32_t key = lane < n ? worker_key(seed, iter, n, lane) : 0xFFFFFFFFu;
    const u32x2 mine2 = {(uint32_t)lane, key};                     // low word: id, high word: key
    const uint64_t mine = __builtin_bit_cast(uint64_t, mine2);
    uint32_t rank = 0;
    for (int j = 0; j < n; j += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const u32x2 other2 = {(uint32_t)(j + u),
                                  (uint32_t)__builtin_amdgcn_readlane((int)key, j + u)};
            rank += __builtin_bit_cast(uint64_t, other2) < mine ? 1u : 0u;
        }
    }
    return rank;
}

// Group index of this lane's worker; lanes that are not workers get an impossible group.
__device__ __forceinline__ uint32_t wave_group_of(uint64_t seed, int64_t iter, int n, int m,
                                                   int lane)
{
    const uint32_t rank = wave_rank(seed, iter, n, lane);
    return lane < n ? rank / (uint32_t)m : 0xFFFFFFFFu;
}

// Members of group g as a lane mask (bit i = worker i), wave-uniform: the workers whose rank
// falls in [g*m, (g+1)*m).  Exactly m bits are set.
__device__ __forceinline__ uint64_t wave_members(uint64_t seed, int64_t iter, int n, int m,
                                                 uint32_t g, int lane)
{
    // Two partitions need no ranking: one group of everybody, and singleton groups, where the
    // result does not depend on which worker is called group g (each is processed once).
    if (m == n) return n == 64 ? ~0ull : (1ull << n) - 1ull;
    if (m == 1) return 1ull << g;
    const uint32_t rank = wave_rank(seed, iter, n, lane);
    return __ballot(lane < n && rank - g * (uint32_t)m < (uint32_t)m);
}

// Next member of a group: lowest set bit of the (wave-uniform) member mask, which is cleared.
__device__ __forceinline__ uint64_t next_row(uint64_t &todo)
{
    const uint64_t r = (uint64_t)__builtin_ctzll(todo);
    todo &= todo - 1;
    return r;
}

// ---------------------------------------------------------------- row accessors
template <int N> struct Pack { float a[N]; };

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
// The 4-column accessors promise the compiler 4-byte alignment only: a multi-dword global or
// buffer access is defined for every dword-aligned address, so rows whose pitch is not a
// multiple of 4 elements can still move 128 bits per lane (the instructions are the same).
typedef float f32x4d __attribute__((ext_vector_type(4), aligned(4)));
typedef unsigned short u16x4d __attribute__((ext_vector_type(4), aligned(4)));

template <typename T, int NT> __device__ __forceinline__ T ld(const void *p)
{
    if constexpr (NT != kPlain) return __builtin_nontemporal_load((const T *)p);
    else return *(const T *)p;
}
template <typename T, int NT> __device__ __forceinline__ void st(void *p, T v)
{
    if constexpr (NT != kPlain) __builtin_nontemporal_store(v, (T *)p);
    else *(T *)p = v;
}

// Written-through streaming store of 16, 8 or 4 bytes at (wave-uniform row) + (per-lane byte
// offset): a raw buffer store, the form whose cache-policy operand reaches the sc1 bit.  The
// descriptor covers 4 GiB from `row` (rows are shorter), dword 3 is the plain raw-buffer
// setting of the gfx9 family.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kRawBufferFlags = 0x00020000;
constexpr int kAuxStreamThrough = (1 << 1) | (1 << 4);      // nt | sc1

template <typename T> __device__ __forceinline__ void st_through(void *row, uint32_t off, T v)
{
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(row, 0, -1, kRawBufferFlags);
    static_assert(sizeof(T) == 16 || sizeof(T) == 8 || sizeof(T) == 4, "store width");
    if constexpr (sizeof(T) == 16)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rsrc, (int)off, 0, kAuxStreamThrough);
    else if constexpr (sizeof(T) == 8)
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), rsrc, (int)off, 0, kAuxStreamThrough);
    else
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), rsrc, (int)off, 0, kAuxStreamThrough);
}

// fp32 vector of N columns at byte address p
template <int N, int NT> __device__ __forceinline__ Pack<N> load_f32(const char *p)
{
    Pack<N> r;
    if constexpr (N == 4) { f32x4d t = ld<f32x4d, NT>(p); r.a[0] = t.x; r.a[1] = t.y; r.a[2] = t.z; r.a[3] = t.w; }
    else if constexpr (N == 2) { f32x2 t = ld<f32x2, NT>(p); r.a[0] = t.x; r.a[1] = t.y; }
    else { r.a[0] = ld<float, NT>(p); }
    return r;
}
// fp32 vector of N columns to (wave-uniform row address) + (per-lane byte offset)
template <int N, int NT> __device__ __forceinline__ void store_f32(char *row, uint32_t off, const Pack<N> &r)
{
    if constexpr (N == 4) {
        const f32x4d t = {r.a[0], r.a[1], r.a[2], r.a[3]};
        if constexpr (NT == kStreamThrough) st_through(row, off, t); else st<f32x4d, NT>(row + off, t);
    } else if constexpr (N == 2) {
        const f32x2 t = {r.a[0], r.a[1]};
        if constexpr (NT == kStreamThrough) st_through(row, off, t); else st<f32x2, NT>(row + off, t);
    } else {
        if constexpr (NT == kStreamThrough) st_through(row, off, r.a[0]); else st<float, NT>(row + off, r.a[0]);
    }
}
// bf16 vector of N columns at byte address p, widened to fp32 (exact: bits << 16)
template <int N, int NT> __device__ __forceinline__ Pack<N> load_bf16(const char *p)
{
    Pack<N> r;
    if constexpr (N == 4) {
        u16x4d t = ld<u16x4d, NT>(p);
        r.a[0] = __uint_as_float((uint32_t)t.x << 16); r.a[1] = __uint_as_float((uint32_t)t.y << 16);
        r.a[2] = __uint_as_float((uint32_t)t.z << 16); r.a[3] = __uint_as_float((uint32_t)t.w << 16);
    } else if constexpr (N == 2) {
        u16x2 t = ld<u16x2, NT>(p);
        r.a[0] = __uint_as_float((uint32_t)t.x << 16); r.a[1] = __uint_as_float((uint32_t)t.y << 16);
    } else {
        r.a[0] = __uint_as_float((uint32_t)ld<unsigned short, NT>(p) << 16);
    }
    return r;
}
template <int N, bool BF16, int NT> __device__ __forceinline__ Pack<N> load_grad(const char *p)
{
    if constexpr (BF16) return load_bf16<N, NT>(p);
    else return load_f32<N, NT>(p);
}

}  // namespace se

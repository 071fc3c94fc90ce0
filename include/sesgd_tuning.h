/*
 * sesgd_tuning.h -- measurement and tuning entry points of libsesgd.so.  Not part of the
 * method's boundary (that is sesgd.h): nothing here changes a result, only how the launches
 * are shaped, and one helper gives the profiler's byte counters a known reference.
 */
#ifndef SESGD_TUNING_H
#define SESGD_TUNING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement helper, not part of the method: copies nbytes (a multiple of 16, below 2^37)
 * between two non-overlapping, 16-byte aligned DEVICE buffers with a plain streaming kernel
 * on `stream`.  Reads nbytes and writes nbytes: the reference reading for the profiler's HBM
 * byte counters and a practical bandwidth ceiling next to se_step's figure. */
int se_calib_copy(void *dst, const void *src, int64_t nbytes, void *stream);

/* Measurement helper: one direction only, between the same kind of buffers as se_calib_copy.
 * direction 1 reads nbytes from src and writes nothing; direction 2 writes nbytes of a constant
 * pattern to dst (its contents are lost) and reads nothing.  Tells what the memory system gives
 * to reads and to writes apart from what it gives to their mix. */
int se_calib_oneway(void *dst, const void *src, int64_t nbytes, int direction, void *stream);

/* Launch-shape knobs for measurement sweeps; results never depend on them (process-wide).
 *   "max_blocks_per_cu"   one-launch forms: cap on resident workgroups per compute unit, enforced
 *                         by requesting 160 KiB / cap of (unused) LDS per workgroup; 0 = no cap;
 *                         -1 (default) = chosen per launch so that about 48 / 32 / 24-36 KiB of
 *                         loads are in flight per compute unit for groups of 1 / 2 / more rows:
 *                         16, 11, 9 workgroups for group sizes 1, 2, 4 with momentum and fp32
 *                         gradients, more for shorter rows (bf16 gradients, no momentum buffer),
 *                         4 for groups of 8 walked two rows at a time, 2 beyond 8 rows (6 for
 *                         gradient averaging); the global average 12, 8, 4 for up to 2, 4, more
 *                         workers; 8 for the LDS-staged form; none for calls below
 *                         "cache_resident_mib"
 *   "batch_rows"          single-wavefront SESGD update: member rows whose loads are issued back
 *                         to back (1, 2, 4, 8); 0 (default) = 1 for groups up to 4, 2 up to 8, 8
 *                         beyond; below "cache_resident_mib" all rows of a small group at once
 *                         and 2 at a time beyond 8;
 *                         also the rows per batch of the split form's first launch (default 1)
 *                         and of the update pass of one-launch gradient averaging (default 1,
 *                         2 for 5-8 workers with fp32 gradients)
 *   "unaligned_wide"      1 (default): rows that do not line up on 16 bytes (a pitch that is no
 *                         multiple of 4 elements, bases at different offsets) still move 128 bits
 *                         per lane, as every row starts on a 4-byte boundary; 0: such rows take
 *                         the 64- or 32-bit body
 *   "nontemporal"         cache policy of the row accesses: 0 plain; 1 streaming (non-temporal)
 *                         loads and stores; 2 (default) streaming, and stores written through
 *                         the L2 to memory at once (measured 2-4 % faster than 1)
 *   "cooperative"         1: LDS-staged form: every wavefront of a workgroup owns one block of 8
 *                         rows of the group and stages its block sum in LDS; 0 (default): never
 *                         (it measured 0.5-7 % slower than the single-wavefront form)
 *   "coop_tiles"          LDS-staged form: consecutive 64-lane tiles one workgroup walks through;
 *                         0 = chosen by group size: 4 above 32 rows, else 1 (default 0)
 *   "cache_resident_mib"  when a full-range call would move fewer MiB than this (default 512;
 *                         the Infinity Cache holds 256 MiB) launches use plain accesses and no
 *                         residency cap, which is faster when nothing streams from HBM;
 *                         0 = always stream
 *   "split"               two-launch form for reductions over more than 8 rows (see sesgd.h,
 *                         "Device memory of the library's own"): 1 whenever the 128-bit path
 *                         applies, 0 never, -1 (default) when a launch moves 2 GiB or more
 *                         (3 GiB for the plain parameter average)
 *   "split_scratch_mib"   size of that form's buffer per (device, stream), default 128
 *   "split_sub_tiles"     tiles of 64 lane-columns per sub-chunk of its second launch; 0 (default)
 *                         = 4096 when gradients are averaged, 2048 otherwise
 *   "split_cap_reduce", "split_cap_finish"   resident workgroups per compute unit of its first
 *                         and second launch; 0 = no cap; -1 (default) = 12 and 24 when gradients
 *                         are averaged, else 7 (10 with bf16 gradients) and 16; without a
 *                         momentum buffer 10 and 32, else twice as many and 8; the plain
 *                         parameter average 6, and 48 (64 beyond 32 workers) divided by the rows
 *                         per wavefront of the second launch
 *   "split_finish_rows"   rows per wavefront of its second launch: 1, 2 or 4 when gradients are
 *                         averaged (default 1); a multiple of 8 for the SESGD update (default 8);
 *                         any number for the plain parameter average (default an eighth of the
 *                         workers, 2 to 8)
 * Returns SE_ERR_ARG for an unknown name or a value out of range. */
int se_set_tuning(const char *name, int value);
int se_get_tuning(const char *name);

#ifdef __cplusplus
}
#endif
#endif /* SESGD_TUNING_H */

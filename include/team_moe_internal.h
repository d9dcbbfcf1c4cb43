/*
 * team_moe_internal.h - tuning and testing hooks of libteam_moe.so.  NOT part of the product interface (team_moe.h): the
 * tests use them to reach code paths that ordinary inputs do not (hash collisions of the repeated-row search, a wait
 * inside the expert FFN kernel that gives up), the benchmark to compare kernel variants.  Process-wide, not thread-safe
 * against calls in flight.
 *
 * Keys (initial value: the environment variable in brackets, read once when the library is first used):
 *   "ffn_grid"         [TEAM_MOE_FFN_GRID]         > 0: workgroups of the expert FFN launch, if below the resident maximum
 *   "ffn_tiled_rows"   [TEAM_MOE_FFN_TILED_ROWS]   rows per expert (average) from which calls of more than 32 tokens take the
 *                                                  streaming body of the FFN kernel (default 18; 0: never)
 *   "ffn_wide_rows"    [TEAM_MOE_FFN_WIDE_ROWS]    rows per expert above which that body takes two token tiles per wavefront (56)
 *   "ffn_shares"       [TEAM_MOE_FFN_SHARES]       0: contiguous shares only; 1 (default): workgroups dealt out to experts where a
 *                                                  share would cross an expert boundary; 2: in the gate/up phase only
 *   "logits_kernel"    [TEAM_MOE_LOGITS_KERNEL]    0: by token count; 1: per-token kernel; 2: matrix-core kernel
 *   "row_hash_bits"    [TEAM_MOE_ROW_HASH_BITS]    bits of the row hashes that the repeated-row search compares (64)
 *   "ffn_spin_limit"   [TEAM_MOE_FFN_SPIN_LIMIT]   polls after which a wait inside the expert FFN kernel gives up (65536)
 *   "ffn_cooperative"  [TEAM_MOE_FFN_COOPERATIVE]  1: launch the expert FFN kernel through hipLaunchCooperativeKernel (a measurement)
 *   "ffn_skip_publish" (none)                      1: gate/up items do not announce their results, so every wait for them
 *                                                  gives up after ffn_spin_limit polls: the failure path (NaN rows, the
 *                                                  workspace's failure mark) can then be tested while every kernel still
 *                                                  runs to its normal end
 * Both calls return a team_status (unknown key or NULL pointer: TEAM_ERR_INVALID_ARG).
 */
#ifndef TEAM_MOE_INTERNAL_H
#define TEAM_MOE_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int team_moe_internal_set(const char* key, int value);
int team_moe_internal_get(const char* key, int* value);

/*
 * A plain read-only stream over `bytes` of device memory at `src` (16-byte aligned, a multiple of 16): `workgroups` workgroups of
 * 256 threads read 64 KB pieces with non-temporal 16-byte loads, as the expert FFN reads its weights, and discard the data.
 * `sink`: `workgroups` 32-bit words of device memory (practically never written).  Enqueued on `stream`; returns a team_status.
 * The benchmark times it on buffers of the sizes the expert FFN streams: the practical ceiling of such a stream on the device.
 */
int team_moe_internal_stream_read(const void* src, size_t bytes, uint32_t* sink, int32_t workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TEAM_MOE_INTERNAL_H */

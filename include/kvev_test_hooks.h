/*
 * kvev test hooks: entry points that exist for the tests of the library, not for
 * its users.  They change process-wide settings (atomically; a call that is
 * already being planned may see the old or the new value) and are declared here,
 * apart from kvev.h, so that nothing in the public interface depends on them.
 */
#ifndef KVEV_TEST_HOOKS_H
#define KVEV_TEST_HOOKS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* For tests of the gate's failure path.  Small launches of kvev_lstm_gate run a
 * group of sequences on two or four workgroups that wait for each other's data
 * (see kvev.h).  This sets, for later calls in this process, the number of polls
 * one such wait may take (default 1 << 22) and the member (0 or 1; -1 = none,
 * the default) that withholds what it would publish, so that its partners' wait
 * expires: every kernel still ends normally, the affected launch's util, gate
 * and c come back NaN and the status word of its workspace is set.
 * Errors: INVALID_ARG for spin_limit < 1 or a member outside -1..1. */
int kvev_debug_pair_wait(int spin_limit, int mute_member);

/* For parity tests of the single-kernel form of the gate (bf16, d_g = 256), which the
 * library takes for launches of at least `min_groups` groups of 16 sequences
 * (default 257: more than one group per compute unit).  Lowering it lets a test
 * run that form on a shape the CPU oracle finishes in seconds; 0 restores the
 * default.  Errors: INVALID_ARG for a negative value. */
int kvev_debug_lstm_fused_min_groups(int min_groups);

/* For parity tests of large calls of the gate at d_g = 512, which the library cuts into launches of at most one
 * workgroup per compute unit (four workgroups per group of 32 sequences).  This lowers the number of groups per
 * launch for later calls in this process (and the exchange scratch that kvev_workspace_bytes reports with it), so
 * that a shape the CPU oracle finishes in seconds takes several launches; 0 restores the default (compute units / 4).
 * Errors: INVALID_ARG for a negative value. */
int kvev_debug_lstm_quad_groups(int groups);

/* The single-query attention kernels read their rows with the non-temporal hint
 * when a launch reads more than `bytes` (default 256 MiB, what the memory-side
 * cache holds; 0 restores the default).  Lowering it to 1 lets a parity test run
 * the streaming form of the loads on a shape the CPU oracle finishes in seconds;
 * the hint changes how the caches treat the rows, never the result.  Errors:
 * none (always KVEV_OK). */
int kvev_debug_attn_stream_bytes(size_t bytes);

/* Calibration of the memory system for the benchmark's roofline notes (bench.py
 * --calibrate-stream): a plain streaming kernel, one workgroup per tile, reads
 * src_bytes of device memory in tiles of tile_bytes (a multiple of 4096 that
 * divides src_bytes) and writes write_bytes_per_tile (a multiple of 16, 0 =
 * none) per tile to dst (device memory of at least tiles * write_bytes_per_tile
 * bytes, 16 at least).  The memory pattern of chunk pooling without its
 * arithmetic.  hints: bit 0 = the loads, bit 1 = the stores carry the
 * non-temporal hint (what the library's own streaming kernels use); bit 2 =
 * persistent workgroups hold their outputs back and write them in chip-wide
 * bursts, once per 82 us slot of the real-time counter (what chunk pooling does
 * at scale; write_bytes_per_tile at most 48 KiB then); 0 = plain accesses.  Enqueued on `stream`; errors: INVALID_ARG. */
int kvev_debug_stream_probe(const void *src, size_t src_bytes, int tile_bytes, void *dst, size_t dst_bytes,
                            int write_bytes_per_tile, int hints, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KVEV_TEST_HOOKS_H */

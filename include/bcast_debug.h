/*
 * bcast_debug.h -- test hooks, diagnostics and experiment knobs of the broadcast
 * library.  Same shared library and same conventions as bcast.h (plain C, HOST
 * pointers unless stated, BCAST_OK or a negative bcast_status_t); nothing here
 * is needed to broadcast.  Kernels always run to completion under every setting
 * declared here.
 */
#ifndef BCAST_DEBUG_H
#define BCAST_DEBUG_H

#include "bcast.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Wait limit and a forced stall, so that the bounded wait of the hand-off
 * (Sec. IV-B's forward step) can be tested from the host.  spin_limit_ticks:
 * wait limit in 100 MHz ticks (0 = default, about 10 s).  mute_hop: chain
 * position (1..P-2) that stores its chunks but never publishes them, so that
 * its right neighbour runs into the wait limit; 0 = off. */
int bcast_plan_set_debug(bcast_plan_t *plan, uint64_t spin_limit_ticks, int mute_hop);

/* Make the plan behave as if it had already run `epoch` times (never fewer than
 * it has).  Runs are told apart by a 32-bit count in the flag words; bcast_run
 * drains the device and clears the flags before the count would wrap, and this
 * lets a test reach that point without 2^32 runs.  BCAST_ERR_ARG if epoch is
 * below the plan's count or above 2^32 - 2. */
int bcast_plan_debug_set_epoch(bcast_plan_t *plan, uint64_t epoch);

/* Chain kernel modes (bit mask).  BCAST_MODE_COUNT: count the hand-offs whose
 * producer and consumer waves ran on the same XCD (one L2) and on different
 * XCDs; read back (after a device synchronise) by bcast_plan_handoff_counts.
 * The counts accumulate over runs.  Diagnostic: it slows the kernel down.
 * BCAST_MODE_FIXED_SPANS / BCAST_MODE_ROTATE_SPANS (not both): where nranks-1 is
 * no multiple of the stage count, the first stages keep the extra hop for every
 * chunk (every chunk has chunk 0's spans of bcast_chain_stage_span), or the
 * extra hop is passed round as that function describes.  With neither bit the
 * library rotates where a stage plays fewer than four hops. */
#define BCAST_MODE_COUNT 2u
#define BCAST_MODE_FIXED_SPANS 16u
#define BCAST_MODE_ROTATE_SPANS 32u
int bcast_plan_set_mode(bcast_plan_t *plan, unsigned mode);
int bcast_plan_handoff_counts(bcast_plan_t *plan, uint64_t *same_xcd, uint64_t *cross_xcd);

/* Pipeline trace.  After bcast_plan_enable_trace(plan, entries), every chain
 * run records, for the first `entries` (stage, chunk) pairs in stage-major
 * order (index = stage * nchunks + chunk), the 100 MHz device clock at which
 * lane 0's wavefront of the stage began copying the chunk (after its wait) and
 * at which all its stores for the chunk had completed.  bcast_plan_read_trace
 * synchronises the device and copies `entries` pairs [begin, end] into `out`
 * (2 * entries words).  entries == 0 turns the trace off.  Each run overwrites
 * the previous one's record. */
int bcast_plan_enable_trace(bcast_plan_t *plan, size_t entries);
int bcast_plan_read_trace(bcast_plan_t *plan, uint64_t *out, size_t entries);

/* Cache policy of the chain kernel's four kinds of payload access, for
 * measurements.  Each value is -1 (the library's choice) or a combination of
 * BCAST_CACHE_AGENT (sc1: agent scope -- loads are not served from a possibly
 * stale L1/L2 line, stores are written through) and BCAST_CACHE_STREAM (nt: not
 * expected to be reused); 0 is an ordinary cached access.
 *   ld_root  loads of the root's buffer (nobody writes it during a run);
 *   ld_edge  loads of what another stage's wavefronts stored: must be agent scope;
 *   ld_back  a wavefront's read-back of its own stores inside a stage;
 *   st_mid   stores the wavefront itself reads back, and the last position's.
 * Write-back stores (st_mid without AGENT) must not be read back at agent scope.
 * Every admitted combination gives the same bytes; only the speed differs.
 * The two sets the library chooses by itself are built into the kernel; any
 * other set is read from the arguments at every hop, which alone costs a few
 * per cent (measured 6 % at 8 ranks x 64 MiB). */
#define BCAST_CACHE_STREAM 2
#define BCAST_CACHE_AGENT 16
int bcast_plan_set_cache_policy(bcast_plan_t *plan, int ld_root, int ld_edge, int ld_back, int st_mid);

/* Trip size of the chain reduction for measurements: 4096 (contributions loaded
 * 4 positions at a time) or 1024 (16 at a time), 0 = the library's choice. */
int bcast_plan_set_reduce_trip(bcast_plan_t *plan, int trip_bytes);

/* Measurement kernels: what the device's memory gives the two access patterns
 * every algorithm here is made of, with no dependencies between accesses.
 * bufs: HOST array of nbufs (1..BCAST_MAX_RANKS) DEVICE pointers, 16-byte
 * aligned; bytes: a multiple of 4096.
 * bcast_debug_store_pattern overwrites bytes [0, bytes) of every buffer, tile
 * by tile over all buffers (the fan-out without its read): the floor of any
 * broadcast to nbufs ranks on one die.
 * bcast_debug_load_pattern reads every buffer once (streaming loads, xor-folded
 * in registers) and, if write_result != 0, writes the fold to out (DEVICE,
 * bytes bytes, 16-byte aligned; required either way): the floor of a reduction
 * of nbufs contributions.  Errors: ERR_ARG, ERR_HIP. */
int bcast_debug_store_pattern(void *const *bufs, int nbufs, size_t bytes, bcast_stream_t stream);
int bcast_debug_load_pattern(void *const *bufs, int nbufs, size_t bytes, void *out, int write_result, bcast_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* BCAST_DEBUG_H */

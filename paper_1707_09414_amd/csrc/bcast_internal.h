// Shared declarations between the host side (plan, validation, tuning) and
// the gfx950 kernels of the broadcast library.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "bcast.h"
#include "bcast_debug.h"

namespace bcast {

typedef unsigned long long u64;

// Workgroups are 256 threads = 4 wavefronts of 64 (the chain kernel can also be
// launched with 1 or 2); every wavefront is an independent copy engine (no
// workgroup barriers anywhere in the library).
constexpr int kBlockThreads = 256;
constexpr int kWaveSize = 64;
constexpr int kWavesPerBlock = kBlockThreads / kWaveSize;

// The chain with one wavefront per rank: a workgroup holds at most this many
// waves, one per consecutive chain position.
constexpr int kRankWavesMax = 16;
constexpr int kRankBlockThreadsMax = kRankWavesMax * kWaveSize;
// Trips a rank may be ahead of its right neighbour's reading: what it stored
// should be read out of the compute unit's cache before later trips push it out
// (measured on MI355X: without a limit 19-21 ms at 64 ranks x 1 GiB, with 1, 2
// or 4 trips 15.0 ms).
constexpr unsigned kRankLead = 2;  // also the number of trip slots a wave has in LDS (kModeLdsHandoff)

// One ready flag per (hop, lane), each alone in a 128-byte line so that a
// producer's store and other lanes' polls never share a line.
constexpr int kFlagStrideWords = 16;

// A wavefront moves kUnroll 16-byte vectors per lane per trip: 4 KiB in flight.
constexpr int kUnroll = 4;
constexpr u64 kTileBytes = (u64)kWaveSize * 16 * kUnroll;
// The chain kernel's trip: `unroll` vector instructions per lane, unroll KiB
// per wave at 16 bytes per lane.  The trips of a CU's resident waves must fit
// its 32 KiB vector L1 to be read back from it (see chain_kernel); measured on
// MI355X, 8 waves per CU with 3 KiB trips (24 KiB) is best for many ranks and
// 4 KiB trips for few; the kernel is built for 2, 3, 4 and 6 KiB (the chain with
// a wavefront per rank also for 1 and 8), the tuner sweeps 3 and 4, and these two
// are the rules without a table.
constexpr int kTripUnrollDefault = 4;
constexpr int kTripUnrollSmall = 3;

// Cache-policy bits of the raw-buffer accesses (gfx940-class encoding): sc1
// marks an access as agent-scope (a load is not served from a line that may be
// stale in this CU's L1 or this XCD's L2, a store is written through), nt marks
// it as streaming (not expected to be reused).
constexpr int kAuxAgent = 16;
constexpr int kAuxCached = 0;
constexpr int kAuxStream = 2;

// The reduction kernel's trips: 16-byte vectors per lane, trip and position
// (4 KiB per wave) for streaming messages, one (1 KiB) for small ones.
constexpr int kRedUnroll = 4;
constexpr int kRedUnrollSmall = 1;
constexpr u64 kRedSmallMaxBytes = 2u << 20;  // measured crossover on MI355X: 2-4 MiB
constexpr int kRedResultStore = kAuxAgent;  // the result is written through: measured 3-6 % faster than write-back stores among the streaming reads

// Wait limit default: 10 s of the 100 MHz constant clock.
constexpr u64 kDefaultSpinTicks = 1000000000ull;

// Arguments of the persistent chain kernel (Sec. IV-B).  buf[] is indexed by
// chain position: buf[0] is the root's buffer, buf[k] receives from buf[k-1].
struct ChainArgs {
    char *buf[BCAST_MAX_RANKS];
    u64 *flags;        // device: [(nranks-1) * lanes] flags, kFlagStrideWords apart
    u64 *abort_word;   // device: set to the run's epoch when a wave gives up
    u64 *status;       // pinned host, device-visible: [0] = 1 on timeout, [1] = hop<<32|chunk
    u64 *trace;        // device: [stage][chunk][begin, end] clock values of lane 0's wave (kModeTrace)
    u64 trace_entries; // (stage, chunk) pairs the trace buffer holds
    u64 *counters;     // device: [0] hand-offs within an XCD, [1] across XCDs (kModeCount)
    u64 base;          // epoch << 32; chunk c of this run is ready when flag >= base + ((c + 1) << 4)
    u64 *epoch_word;   // device, or null: if set, the epoch is read from here instead (see advance_epoch_kernel) and base is unused
    u64 bytes;         // M
    u64 chunk_bytes;   // C (multiple of 16)
    u64 spin_ticks;    // wait limit in 100 MHz ticks
    unsigned nchunks;
    unsigned lanes;    // wavefronts per stage
    unsigned stages;   // groups of consecutive chain positions, each served by its own waves
    unsigned hops_per_stage; // the most hops a stage plays for one chunk (informational)
    unsigned unroll;   // vector instructions per lane and trip (KiB per wave at 16-byte vectors): one the kernel is built for
    unsigned nranks;
    unsigned mute_hop; // debug: this position never publishes (0 = off)
    unsigned mode;     // kMode* bits
    // chain kernel: cache-policy bits (kAux*) of its four kinds of access
    unsigned char ld_root;  // loads of the root's buffer, which nobody writes during the run
    unsigned char ld_edge;  // loads of what another stage's waves stored: agent scope
    unsigned char ld_back;  // a wave's read-back of its own stores inside a stage
    unsigned char st_mid;   // stores the wave itself reads back, and the last position's
    // pipelined k-nomial tree only (tree_kernel): the position each position
    // receives from, and the positions that have children (bit = position)
    unsigned char parent[BCAST_MAX_RANKS];
    u64 forward_mask;
    // chain reduction only (reduce_kernel): buf[] holds the contributions by
    // chain position (read only); recv is the root's result buffer; stage g < last
    // hands its running sum to stage g + 1 through scratch + g * scratch_stride
    char *recv;
    char *scratch;
    u64 scratch_stride;
};

// Number of chain hops that lie before stage g for chunk c, so that stage g plays
// hops stage_begin(g) + 1 .. stage_begin(g + 1) of that chunk.  Every stage plays
// hops_min = hops / stages hops and hops_extra = hops % stages of the stages one
// more; which ones rotates with the chunk: stage j has the extra hop for chunk c
// iff (j + c) mod stages < hops_extra.  Over any `stages` consecutive chunks
// every stage plays exactly `hops` hops.
__host__ __device__ inline unsigned stage_begin(unsigned g, unsigned c, unsigned stages, unsigned hops_min, unsigned hops_extra)
{
    // extras among stages 0..g-1 = the residues (c mod stages) .. (c mod stages) + g - 1
    // that are below hops_extra; below(x) counts them in [0, x)
    const unsigned start = c % stages;
    const unsigned x1 = start + g, x0 = start;
    const unsigned below1 = (x1 / stages) * hops_extra + (x1 % stages < hops_extra ? x1 % stages : hops_extra);
    const unsigned below0 = (x0 / stages) * hops_extra + (x0 % stages < hops_extra ? x0 % stages : hops_extra);
    return g * hops_min + below1 - below0;
}

// ChainArgs::mode
// Count hand-offs whose two waves ran on the same XCD / on different XCDs.
// Diagnostic only: every wave ends with two atomics on one cache line, which
// costs tens of microseconds at full occupancy.
constexpr unsigned kModeCount = 2;
// Lane 0's wave of every stage records when it begins and ends each chunk.
constexpr unsigned kModeTrace = 8;
// The stages that play one hop more do not rotate from chunk to chunk: the
// first hops % stages stages always have it.  The host sets it per run unless
// rotation pays (see rotate_spans in bcast.cpp); kModeRotateSpans is the
// caller's request to rotate regardless and never reaches the kernel.
constexpr unsigned kModeFixedSpans = 16;
constexpr unsigned kModeRotateSpans = 32;
// Wave-per-rank chain: inside a workgroup a trip travels from rank to rank
// through LDS (two slots per rank) instead of being read back out of the left
// neighbour's buffer through the compute unit's cache.
constexpr unsigned kModeLdsHandoff = 64;
// Largest message whose in-stage stores are write-back by default (measured
// crossover on MI355X: 2-4 MiB).
constexpr u64 kStageWriteBackMaxBytes = 2u << 20;

// Arguments of the plain copy kernels: up to 32 simultaneous (src -> dst)
// whole-message copies (one binomial round has at most 32 at P = 64; the
// direct algorithm uses one per launch), or one source and nranks-1
// destinations for the fan-out.
struct CopyArgs {
    char *buf[BCAST_MAX_RANKS]; // by chain position
    unsigned char src_pos[BCAST_MAX_RANKS / 2];
    unsigned char dst_pos[BCAST_MAX_RANKS / 2];
    unsigned npairs;
    unsigned nranks;
    u64 lo;   // first byte offset to move
    u64 hi;   // one past the last byte offset to move
};

// Arguments of the ranged copy kernel: up to 64 simultaneous copies, each of its
// own byte range [lo, hi) (same offsets on both sides): one round of the
// binomial scatter or one step of the ring allgather (Sec. III-A, Eq. 4).
struct RangedCopyArgs {
    char *buf[BCAST_MAX_RANKS]; // by chain position
    u64 lo[BCAST_MAX_RANKS];
    u64 hi[BCAST_MAX_RANKS];
    unsigned char src_pos[BCAST_MAX_RANKS];
    unsigned char dst_pos[BCAST_MAX_RANKS];
    unsigned npairs;
};

// The statically allocated scratch array (kernels.hip): flag lines, then staging.
constexpr int kStaticFlagWaves = 8192;                                  // ready flags it holds
constexpr u64 kStaticFlagLines = (u64)kStaticFlagWaves + 2;             // + abort word + run counter
constexpr u64 kStaticFlagBytes = kStaticFlagLines * kFlagStrideWords * sizeof(u64);
constexpr u64 kStaticStagingBytes = 32ull << 20;                        // running sums between stages
constexpr u64 kStaticScratchBytes = kStaticFlagBytes + kStaticStagingBytes;
constexpr int kStaticMaxDevices = 64;
// Device address of the current device's copy of the array (looked up once per
// device; `device` must be the current device on that first call).
hipError_t static_scratch_address(int device, char **ptr);
hipError_t launch_advance_epoch(u64 *epoch_word, u64 *flags, u64 clear_words, u64 limit, hipStream_t stream);

// Launchers implemented in kernels.hip.  vec_bytes is 16, 8, 4 or 1: every
// buffer address in the call is congruent modulo vec_bytes.
hipError_t launch_chain(const ChainArgs &a, int vec_bytes, int grid_blocks, int block_threads, hipStream_t stream);
bool valid_chain_block(int block_threads);  // 64, 128 or 256
bool valid_chain_unroll(int unroll);        // vector instructions per lane and trip the chain kernel is built for
// device: the current device; lds_limit: the LDS a workgroup may use there (both only looked at under kModeLdsHandoff)
hipError_t launch_rank_chain(const ChainArgs &a, int vec_bytes, int grid_blocks, int block_threads, int device, int lds_limit,
                             hipStream_t stream);
hipError_t rank_chain_max_blocks_per_cu(int block_threads, int *blocks);
size_t rank_chain_lds_bytes(int waves, int unroll, int vec_bytes);  // dynamic LDS of a workgroup under kModeLdsHandoff
constexpr u64 kRankLdsMinBytes = 2u << 20;  // without a request: trips through LDS for messages above this size
constexpr size_t kRankStaticLdsBytes = 2 * kRankWavesMax * sizeof(unsigned);  // the kernel's own trip counters
hipError_t launch_tree(const ChainArgs &a, int vec_bytes, int grid_blocks, hipStream_t stream);
hipError_t launch_reduce(const ChainArgs &a, int grid_blocks, hipStream_t stream);
hipError_t reduce_max_blocks_per_cu(int *blocks);
hipError_t tree_max_blocks_per_cu(int *blocks);
hipError_t launch_pair_copy(const CopyArgs &a, int vec_bytes, int grid_x, hipStream_t stream);
hipError_t launch_fanout(const CopyArgs &a, int vec_bytes, int grid_x, hipStream_t stream);
hipError_t launch_store_pattern(const CopyArgs &a, int grid_x, hipStream_t stream);
hipError_t launch_load_pattern(const CopyArgs &a, char *out, bool write_result, int grid_x, hipStream_t stream);
hipError_t launch_ranged_copy(const RangedCopyArgs &a, int vec_bytes, int grid_x, hipStream_t stream);
hipError_t chain_max_blocks_per_cu(int block_threads, int *blocks);

}  // namespace bcast

// Host side of the broadcast library: plans, argument checks, the mapping of
// each algorithm onto kernel launches, and the C ABI declared in bcast.h.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "bcast_internal.h"
#include "tune_table.h"

using namespace bcast;

struct bcast_plan {
    int nranks = 0;
    size_t bytes = 0;
    size_t chunk_bytes = 0;  // as requested; 0 = choose per run
    int algo = BCAST_ALGO_AUTO;
    int device = 0;
    int cu_count = 0;
    // wavefronts of the chain kernel the device holds at once, per workgroup
    // size (index: 0 = 64, 1 = 128, 2 = 256 threads)
    int max_waves[3] = {0, 0, 0};
    int max_flags = 0;                    // flags allocated: the largest of the above
    int max_waves_reduce = 0;             // the same limit for the reduction kernel (256-thread workgroups)
    int max_waves_tree = 0;               // ... and for the pipelined tree kernel
    char *d_scratch = nullptr;            // reduction: running sums handed from stage to stage
    size_t scratch_bytes = 0;             // (bcast_plan_reserve_reduce; the run path never allocates)
    char *static_scratch = nullptr;       // this device's copy of the library's static scratch array
    u64 *d_flags = nullptr;  // max_waves flags, kFlagStrideWords apart, plus the abort word
    u64 *d_abort = nullptr;
    u64 *d_counters = nullptr; // two words after the abort word
    u64 *d_epoch = nullptr;    // the run counter in device memory, one line after the counters (replayable plans)
    bool replayable = false;   // runs take their epoch from d_epoch (bcast_plan_set_replayable)
    u64 *d_trace = nullptr;    // optional (bcast_plan_enable_trace)
    size_t trace_entries = 0;
    unsigned mode = 0;
    u64 *h_status = nullptr; // pinned host: [0] timeout seen, [1] hop<<32|chunk
    u64 *d_status = nullptr; // the same two words as the device sees them
    u64 epoch = 0;
    int lanes_request = 0;
    int stages_request = 0;
    int radix_request = 0;
    int trip_request = 0;  // bytes at 16-byte vectors: 0 = choose, else a size the run's chain kernel is built for
    int block_request = 0; // chain workgroup size: 0 = choose, else 64, 128 or 256
    u64 spin_ticks = kDefaultSpinTicks;
    int mute_hop = 0;
    int policy_request[4] = {-1, -1, -1, -1};  // ld_root, ld_edge, ld_back, st_mid; -1 = choose
    int reduce_trip_request = 0;               // reduction: 0 = choose, 4096 or 1024
    int stage_store = BCAST_STORE_AUTO;        // chain: in-stage stores written through or write-back
    int chain_waves = BCAST_CHAIN_AUTO;        // chain: a wavefront per stage (chain_kernel) or per rank (rank_chain_kernel)
    int rank_blocks_per_cu[kRankWavesMax + 1] = {0};  // workgroups of w waves a CU holds (0 = not asked yet)
    int rank_handoff = BCAST_HANDOFF_AUTO;     // wave-per-rank chain: trips between ranks through LDS or the CU's cache
    int lds_per_block = 0;                     // LDS a workgroup may use / a compute unit has, bytes
    int lds_per_cu = 0;
};

static thread_local int g_last_hip_error = 0;

static int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    (void)hipGetLastError();  // leave no sticky error behind for the caller's next HIP call
    return e == hipErrorOutOfMemory ? BCAST_ERR_NOMEM : BCAST_ERR_HIP;
}

#define HIP_TRY(expr)                               \
    do {                                            \
        hipError_t e_ = (expr);                     \
        if (e_ != hipSuccess) return hip_fail(e_);  \
    } while (0)

static u64 ceil_div(u64 a, u64 b) { return (a + b - 1) / b; }
static u64 round_up(u64 a, u64 b) { return ceil_div(a, b) * b; }


// Stages for `hops` chain hops when the caller asks for `request` (0 = one per
// hop): that many, and each plays floor or ceil(hops / stages) consecutive hops
// (where stages are short the kernel passes the extra hop round from chunk to
// chunk, see rotate_spans).
static void stage_shape(int hops, int request, int *stages, int *hops_per_stage)
{
    *stages = request > 0 ? std::min(request, hops) : hops;
    *hops_per_stage = (hops + *stages - 1) / *stages;
}

// Bytes of one trip of the copy loop at 16-byte vectors: the least worth a lane.
static u64 trip_bytes_of(int unroll) { return (u64)unroll * kWaveSize * 16; }
static bool valid_trip(u64 t) { return t != 0 && t % (kWaveSize * 16) == 0 && valid_chain_unroll((int)(t / (kWaveSize * 16))); }
// ... and of the chain kernel with one wavefront per rank
static bool valid_rank_trip(u64 t) { return t == 1024 || t == 2048 || t == 3072 || t == 4096 || t == 6144 || t == 8192; }

// Chunk size when the caller gives none and no tuning entry applies.  On one
// die every hop shares the same HBM, so Eq. 5's fill term (n - 2 idle links)
// costs little.  What matters is how many waves run: a lane gets one trip per
// chunk, and about 2048 waves in total (8 per CU) keep what a wave re-reads
// inside its stage in the CU's L1 while hiding the store latency (see
// chain_kernel).  So: chunk = lanes * trip with lanes = 2048 / stages, but never
// more lanes than the device holds.
constexpr u64 kWavesTarget = 2048;

static u64 default_chunk(int nranks, int max_waves, int stages_request, u64 trip)
{
    int stages = 1, hps = 1;
    stage_shape(std::max(1, nranks - 1), stages_request, &stages, &hps);
    u64 lanes = std::max<u64>(1, std::min<u64>(kWavesTarget, (u64)max_waves) / (u64)stages);
    u64 p = 1;
    while (p * 2 <= lanes) p *= 2;
    return p * trip;
}

// Runs of one plan are told apart by a 32-bit epoch in the flag words.
constexpr u64 kEpochLimit = 0xFFFFFFFEull;

static int block_index(int block_threads) { return block_threads == 64 ? 0 : block_threads == 128 ? 1 : 2; }

extern "C" int bcast_chain_geometry(int nranks, size_t bytes, size_t chunk_bytes, int max_waves,
                                    const bcast_chain_request_t *req, bcast_plan_info_t *info)
{
    const bcast_chain_request_t none = {0, 0, 0, 0};
    if (!req) req = &none;
    const int lanes_request = req->lanes, stages_request = req->stages;
    if (!info || nranks < 1 || nranks > BCAST_MAX_RANKS || max_waves < 1 || lanes_request < 0 || stages_request < 0)
        return BCAST_ERR_ARG;
    const u64 trip = req->trip_bytes ? (u64)req->trip_bytes : trip_bytes_of(kTripUnrollDefault);
    if (!valid_trip(trip)) return BCAST_ERR_ARG;
    const int block = req->block_threads ? req->block_threads : kBlockThreads;
    if (!valid_chain_block(block)) return BCAST_ERR_ARG;
    if (chunk_bytes == 0 || chunk_bytes % 16 != 0) return BCAST_ERR_ARG;
    memset(info, 0, sizeof *info);
    info->algo = BCAST_ALGO_CHAIN;
    info->block_threads = block;
    info->vec_bytes = 16;
    if (nranks < 2 || bytes == 0) {
        info->chunk_bytes = chunk_bytes;
        return BCAST_OK;
    }
    // C >= M is the unpipelined chain: one chunk that is the whole message
    u64 C = std::min<u64>(chunk_bytes, round_up(bytes, 16));
    u64 nchunks = ceil_div(bytes, C);
    if (nchunks >= (1ull << 27)) return BCAST_ERR_ARG;  // the flag word keeps the count in 28 bits
    int hops = nranks - 1;
    int stages = 0, hps = 0;
    stage_shape(hops, stages_request, &stages, &hps);
    if (max_waves < stages) return BCAST_ERR_ARG;  // every stage needs a resident wavefront
    // Lanes per hop: a power of two.  Measured on MI355X, 2^k lanes per hop run
    // 15-20 % faster than nearby counts: with 4-wave workgroups dealt round-robin
    // over 8 XCDs and then over each XCD's CUs, every hop's workgroups then
    // spread evenly over the XCDs and CUs, and a lane's waves of all hops share
    // an XCD (from 32 lanes up).
    auto shape = [](u64 l) -> u64 {
        u64 p = 1;
        while (p * 2 <= l) p *= 2;
        return p;
    };
    u64 lanes_max = shape((u64)(max_waves / stages));
    // a lane should own at least one trip of a chunk unless the chunk is smaller
    u64 useful = std::max<u64>(1, ceil_div(C, trip));
    u64 lanes = lanes_request > 0 ? std::min<u64>((u64)lanes_request, (u64)(max_waves / stages))
                                  : shape(std::min(useful, lanes_max));
    lanes = std::max<u64>(1, lanes);
    // a lane takes every lanes-th trip of a chunk
    info->trip_bytes = (int)trip;
    info->slice_bytes = ceil_div(C, lanes * trip) * trip;
    info->chunk_bytes = C;
    info->nchunks = nchunks;
    info->lanes = (int)lanes;
    info->stages = stages;
    info->hops_per_stage = hps;
    info->grid_blocks = (int)ceil_div((u64)stages * lanes, (u64)(block / kWaveSize));
    info->launches = 1;
    info->algorithmic_bytes = 2ull * hops * bytes;
    return BCAST_OK;
}

// Whether the longer stages rotate from chunk to chunk.  Measured on MI355X
// (same buffers, same process): rotation gains 3-20 % where a stage plays fewer
// than four hops (P = 8 in two stages: 4|3 hops, 8.27 vs 8.03 TB/s; in three:
// 6.5 vs 5.4), where the idle time of the shorter stages is large; with long
// stages (P >= 16 in two stages) it loses 5 % at 3 KiB trips -- there the short
// idle time of one stage relieves the CUs' L1, which those trips fill to the brim.
static bool rotate_spans(unsigned mode, int table_choice, int hops, int stages)
{
    if (mode & kModeRotateSpans) return true;
    if (mode & kModeFixedSpans) return false;
    if (hops % stages == 0) return false;
    if (table_choice == BCAST_SPANS_ROTATE) return true;
    if (table_choice == BCAST_SPANS_FIXED) return false;
    return hops / stages < 4;
}

extern "C" int bcast_chain_stage_span(int nranks, int stages, int stage, uint64_t chunk, int *first_hop, int *last_hop)
{
    if (nranks < 2 || nranks > BCAST_MAX_RANKS || stages < 1 || stages > nranks - 1 || stage < 0 || stage >= stages ||
        !first_hop || !last_hop)
        return BCAST_ERR_ARG;
    const unsigned hops = (unsigned)(nranks - 1), S = (unsigned)stages;
    const unsigned c = (unsigned)(chunk % S);  // the pattern repeats every `stages` chunks
    *first_hop = (int)stage_begin((unsigned)stage, c, S, hops / S, hops % S) + 1;
    *last_hop = (int)stage_begin((unsigned)stage + 1, c, S, hops / S, hops % S);
    return BCAST_OK;
}

extern "C" int bcast_plan_create(bcast_plan_t **out, int nranks, size_t bytes, size_t chunk_bytes, int algo)
{
    if (!out) return BCAST_ERR_ARG;
    *out = nullptr;
    if (nranks < 1 || nranks > BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    if (algo < BCAST_ALGO_AUTO || algo > BCAST_ALGO_KNOMIAL_PIPELINED) return BCAST_ERR_ARG;
    if (chunk_bytes % 16 != 0) return BCAST_ERR_ARG;

    bcast_plan *p = new (std::nothrow) bcast_plan;
    if (!p) return BCAST_ERR_NOMEM;
    p->nranks = nranks;
    p->bytes = bytes;
    p->chunk_bytes = chunk_bytes;
    p->algo = algo;

    int rc = BCAST_OK;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&p->device);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, p->device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&p->lds_per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, p->device);
    if (e == hipSuccess) {
        // what a compute unit has for all its resident workgroups; never less than one workgroup's share
        if (hipDeviceGetAttribute(&p->lds_per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, p->device) != hipSuccess) {
            (void)hipGetLastError();
            p->lds_per_cu = 0;
        }
        p->lds_per_cu = std::max(p->lds_per_cu, p->lds_per_block);
    }
    if (e == hipSuccess) {
        p->cu_count = prop.multiProcessorCount;
        // the chain grid never exceeds what the device holds at once, so every
        // wave a waiter depends on is resident (stage-major numbering alone
        // already makes waits point at earlier-dispatched workgroups); at most
        // 32 waves per CU are counted on
        for (int b = 0; b < 3 && e == hipSuccess; ++b) {
            const int threads = kWaveSize << b, waves = 1 << b;
            int per_cu = 0;
            e = chain_max_blocks_per_cu(threads, &per_cu);
            per_cu = std::max(1, std::min(per_cu * waves, 32) / waves);
            p->max_waves[b] = std::max(nranks, p->cu_count * per_cu * waves);
            p->max_flags = std::max(p->max_flags, p->max_waves[b]);
        }
    }
    if (e == hipSuccess) {
        int per_cu = 0;
        e = reduce_max_blocks_per_cu(&per_cu);
        per_cu = std::max(1, std::min(per_cu, 8));
        p->max_waves_reduce = std::min(p->max_flags, std::max(nranks, p->cu_count * per_cu * kWavesPerBlock));
    }
    if (e == hipSuccess) {
        // the tree kernel's own residency limit (its waves wait for their parents' waves)
        int per_cu = 0;
        e = tree_max_blocks_per_cu(&per_cu);
        per_cu = std::max(1, std::min(per_cu, 8));
        p->max_waves_tree = std::min(p->max_flags, std::max(nranks, p->cu_count * per_cu * kWavesPerBlock));
    }
    if (e == hipSuccess) {
        size_t flag_bytes = ((size_t)p->max_flags + 3) * kFlagStrideWords * sizeof(u64);
        e = hipMalloc((void **)&p->d_flags, flag_bytes);
        if (e == hipSuccess) e = hipMemset(p->d_flags, 0, flag_bytes);
        if (e == hipSuccess) {
            p->d_abort = p->d_flags + (size_t)p->max_flags * kFlagStrideWords;
            p->d_counters = p->d_abort + kFlagStrideWords;
            p->d_epoch = p->d_counters + kFlagStrideWords;
        }
    }
    // set-up for bcast_reduce_sum_f32_static: the address of this device's copy of
    // the static scratch array, looked up while the device is current
    if (e == hipSuccess) e = static_scratch_address(p->device, &p->static_scratch);
    if (e == hipSuccess) e = hipHostMalloc((void **)&p->h_status, 2 * sizeof(u64), hipHostMallocMapped);
    if (e == hipSuccess) {
        p->h_status[0] = p->h_status[1] = 0;
        e = hipHostGetDevicePointer((void **)&p->d_status, p->h_status, 0);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        rc = hip_fail(e);
        if (p->d_flags) (void)hipFree(p->d_flags);
        if (p->h_status) (void)hipHostFree(p->h_status);
        delete p;
        return rc;
    }
    *out = p;
    return BCAST_OK;
}

extern "C" int bcast_plan_destroy(bcast_plan_t *p)
{
    if (!p) return BCAST_ERR_ARG;
    int rc = BCAST_OK;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) rc = hip_fail(e);
    if (p->d_flags && (e = hipFree(p->d_flags)) != hipSuccess) rc = hip_fail(e);
    if (p->d_trace && (e = hipFree(p->d_trace)) != hipSuccess) rc = hip_fail(e);
    if (p->d_scratch && (e = hipFree(p->d_scratch)) != hipSuccess) rc = hip_fail(e);
    if (p->h_status && (e = hipHostFree(p->h_status)) != hipSuccess) rc = hip_fail(e);
    delete p;
    return rc;
}

extern "C" int bcast_plan_set_lanes(bcast_plan_t *p, int lanes)
{
    if (!p || lanes < 0) return BCAST_ERR_ARG;
    p->lanes_request = lanes;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_stages(bcast_plan_t *p, int stages)
{
    if (!p || stages < 0) return BCAST_ERR_ARG;
    p->stages_request = stages;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_trip(bcast_plan_t *p, int trip_bytes)
{
    // the two chain kernels are built for different sets of sizes; which one a run
    // uses is known when the run is described, and checked again there
    if (!p || (trip_bytes != 0 && !valid_trip((u64)trip_bytes) && !valid_rank_trip((u64)trip_bytes))) return BCAST_ERR_ARG;
    p->trip_request = trip_bytes;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_block_threads(bcast_plan_t *p, int block_threads)
{
    if (!p || (block_threads != 0 && !valid_chain_block(block_threads))) return BCAST_ERR_ARG;
    p->block_request = block_threads;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_radix(bcast_plan_t *p, int radix)
{
    if (!p || radix < 0 || radix == 1 || radix > BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    p->radix_request = radix;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_debug(bcast_plan_t *p, uint64_t spin_limit_ticks, int mute_hop)
{
    if (!p || mute_hop < 0 || mute_hop >= BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    p->spin_ticks = spin_limit_ticks ? spin_limit_ticks : kDefaultSpinTicks;
    p->mute_hop = mute_hop;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_cache_policy(bcast_plan_t *p, int ld_root, int ld_edge, int ld_back, int st_mid)
{
    if (!p) return BCAST_ERR_ARG;
    const int v[4] = {ld_root, ld_edge, ld_back, st_mid};
    for (int x : v)
        if (x != -1 && (x & ~(kAuxAgent | kAuxStream))) return BCAST_ERR_ARG;
    // what another stage stored must be loaded at agent scope, and a wave's own
    // write-back stores are not read back at agent scope
    if (ld_edge != -1 && !(ld_edge & kAuxAgent)) return BCAST_ERR_ARG;
    if (st_mid != -1 && !(st_mid & kAuxAgent) && ld_back != -1 && (ld_back & kAuxAgent)) return BCAST_ERR_ARG;
    if (st_mid == -1 && ld_back != -1 && (ld_back & kAuxAgent)) return BCAST_ERR_ARG;  // the default store may be write-back
    for (int i = 0; i < 4; ++i) p->policy_request[i] = v[i];
    return BCAST_OK;
}

extern "C" int bcast_plan_set_reduce_trip(bcast_plan_t *p, int trip_bytes)
{
    if (!p || (trip_bytes != 0 && trip_bytes != 4096 && trip_bytes != 1024)) return BCAST_ERR_ARG;
    p->reduce_trip_request = trip_bytes;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_stage_store(bcast_plan_t *p, int mode)
{
    if (!p || mode < BCAST_STORE_AUTO || mode > BCAST_STORE_BACK) return BCAST_ERR_ARG;
    p->stage_store = mode;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_rank_handoff(bcast_plan_t *p, int mode)
{
    if (!p || mode < BCAST_HANDOFF_AUTO || mode > BCAST_HANDOFF_LDS) return BCAST_ERR_ARG;
    p->rank_handoff = mode;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_chain_waves(bcast_plan_t *p, int mode)
{
    if (!p || mode < BCAST_CHAIN_AUTO || mode > BCAST_CHAIN_WAVE_PER_RANK) return BCAST_ERR_ARG;
    p->chain_waves = mode;
    return BCAST_OK;
}

// The plan's run count: the host's, or (replayable plans) the word in device
// memory, which only the device advances; reading it waits for the device.
static int current_epoch(bcast_plan *p, u64 *epoch)
{
    *epoch = p->epoch;
    if (!p->replayable) return BCAST_OK;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(epoch, p->d_epoch, sizeof(u64), hipMemcpyDeviceToHost));
    return BCAST_OK;
}

extern "C" int bcast_plan_set_replayable(bcast_plan_t *p, int on)
{
    if (!p || (on != 0 && on != 1)) return BCAST_ERR_ARG;
    if ((on != 0) == p->replayable) return BCAST_OK;
    // the count moves to where the next runs will look for it; runs in flight finish first
    u64 epoch = 0;
    int rc = current_epoch(p, &epoch);
    if (rc != BCAST_OK) return rc;
    HIP_TRY(hipDeviceSynchronize());
    if (on) HIP_TRY(hipMemcpy(p->d_epoch, &epoch, sizeof(u64), hipMemcpyHostToDevice));
    p->epoch = epoch;
    p->replayable = on != 0;
    return BCAST_OK;
}

extern "C" int bcast_plan_debug_set_epoch(bcast_plan_t *p, uint64_t epoch)
{
    if (!p || epoch > kEpochLimit) return BCAST_ERR_ARG;
    // flags left by earlier runs must stay below every later run's base
    u64 now = 0;
    int rc = current_epoch(p, &now);
    if (rc != BCAST_OK) return rc;
    if (epoch < now) return BCAST_ERR_ARG;
    if (p->replayable) HIP_TRY(hipMemcpy(p->d_epoch, &epoch, sizeof(u64), hipMemcpyHostToDevice));
    p->epoch = epoch;
    return BCAST_OK;
}

extern "C" int bcast_plan_set_mode(bcast_plan_t *p, unsigned mode)
{
    if (!p || (mode & ~(kModeCount | kModeFixedSpans | kModeRotateSpans))) return BCAST_ERR_ARG;
    if ((mode & kModeFixedSpans) && (mode & kModeRotateSpans)) return BCAST_ERR_ARG;
    p->mode = mode;
    return BCAST_OK;
}

extern "C" int bcast_plan_enable_trace(bcast_plan_t *p, size_t entries)
{
    if (!p || entries > ((size_t)1 << 24)) return BCAST_ERR_ARG;
    HIP_TRY(hipDeviceSynchronize());
    if (p->d_trace) {
        HIP_TRY(hipFree(p->d_trace));
        p->d_trace = nullptr;
        p->trace_entries = 0;
    }
    if (entries == 0) return BCAST_OK;
    HIP_TRY(hipMalloc((void **)&p->d_trace, entries * 2 * sizeof(u64)));
    HIP_TRY(hipMemset(p->d_trace, 0, entries * 2 * sizeof(u64)));
    p->trace_entries = entries;
    return BCAST_OK;
}

extern "C" int bcast_plan_read_trace(bcast_plan_t *p, uint64_t *out, size_t entries)
{
    if (!p || !out || !p->d_trace || entries > p->trace_entries) return BCAST_ERR_ARG;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(out, p->d_trace, entries * 2 * sizeof(u64), hipMemcpyDeviceToHost));
    return BCAST_OK;
}

extern "C" int bcast_plan_handoff_counts(bcast_plan_t *p, uint64_t *same_xcd, uint64_t *cross_xcd)
{
    if (!p || !same_xcd || !cross_xcd) return BCAST_ERR_ARG;
    u64 host[2] = {0, 0};
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host, p->d_counters, sizeof host, hipMemcpyDeviceToHost));
    *same_xcd = host[0];
    *cross_xcd = host[1];
    return BCAST_OK;
}

extern "C" int bcast_plan_status(bcast_plan_t *p, uint64_t *detail)
{
    if (!p) return BCAST_ERR_ARG;
    volatile u64 *st = p->h_status;
    if (st[0] == 0) return BCAST_OK;
    if (detail) *detail = st[1];
    return BCAST_ERR_TIMEOUT;
}

extern "C" int bcast_plan_clear_status(bcast_plan_t *p)
{
    if (!p) return BCAST_ERR_ARG;
    volatile u64 *st = p->h_status;
    st[1] = 0;
    st[0] = 0;
    return BCAST_OK;
}

// Widest access every buffer supports together: all addresses must agree
// modulo the vector size so that one head/body/tail split serves both sides
// of every copy.
static int common_vec_bytes(void *const *bufs, int n)
{
    if (!bufs) return 16;
    uintptr_t diff = 0;
    for (int i = 1; i < n; ++i) diff |= (uintptr_t)bufs[i] ^ (uintptr_t)bufs[0];
    if ((diff & 15) == 0) return 16;
    if ((diff & 7) == 0) return 8;
    if ((diff & 3) == 0) return 4;
    return 1;
}

struct Resolved {
    int algo;
    u64 chunk;
    int stages;  // 0 = built-in rule
    int radix;   // k-nomial only
    int trip;    // chain: bytes per trip
    bool rank_waves;  // chain: a wavefront per rank
    int stage_store;  // chain: BCAST_STORE_THROUGH or _BACK
    int lanes;        // chain with a wavefront per stage: wavefronts per stage, 0 = derive from the chunk
    int spans;        // chain with a wavefront per stage: BCAST_SPANS_*
};

// Without a measurement: two stages (hops 1..h | h+1..P-1).  On one die the
// fewer, larger stages run faster (a wave re-reads what it just stored from the
// Infinity Cache, and DRAM sees few streams), and two is the fewest that still
// hands every chunk over through a flag.
static int default_stages(int nranks) { return std::min(std::max(1, nranks - 1), 2); }

// Co-residency limit of the chain kernel at the plan's workgroup size.
static int waves_for(const bcast_plan *p, size_t)
{
    return p->max_waves[block_index(p->block_request ? p->block_request : kBlockThreads)];
}

// Wavefronts per position of the pipelined tree: every position but the root has
// its own, all resident at once; a power of two like the chain's lanes.
static u64 tree_lanes_max(const bcast_plan *p)
{
    const u64 per_pos = (u64)p->max_waves_tree / (u64)std::max(1, p->nranks - 1);
    u64 l = 1;
    while (l * 2 <= per_pos) l *= 2;
    return l;
}

static int resolve(const bcast_plan *p, size_t bytes, Resolved *r)
{
    r->algo = p->algo;
    r->chunk = p->chunk_bytes;
    r->stages = p->stages_request;
    r->trip = p->trip_request;
    r->rank_waves = p->chain_waves == BCAST_CHAIN_WAVE_PER_RANK;
    r->stage_store = p->stage_store;
    r->lanes = p->lanes_request;
    r->spans = BCAST_SPANS_AUTO;
    bcast_tune_entry_t e;
    const bool tuned = bcast_tune_get(p->nranks, bytes, &e) == BCAST_OK;
    // a table entry's chunk, stages and trip belong to the wave mode it was
    // measured in: they apply if the plan leaves the mode open or asks for that one
    auto mode_fits = [&](int entry_rank_waves) {
        return p->chain_waves == BCAST_CHAIN_AUTO || (p->chain_waves == BCAST_CHAIN_WAVE_PER_RANK) == (entry_rank_waves != 0);
    };
    if (p->algo == BCAST_ALGO_AUTO) {
        if (!tuned) return BCAST_ERR_UNTUNED;
        r->algo = e.algo;
        if (r->chunk == 0 && (e.algo != BCAST_ALGO_CHAIN || mode_fits(e.rank_waves))) {
            r->chunk = e.chunk_bytes;
            if (r->stages == 0) r->stages = e.stages;
            if (e.algo == BCAST_ALGO_CHAIN) {
                if (r->trip == 0) r->trip = e.trip_bytes;
                r->rank_waves = e.rank_waves != 0;
                if (r->stage_store == BCAST_STORE_AUTO) r->stage_store = e.stage_store;
                if (r->lanes == 0) r->lanes = e.lanes;
                r->spans = e.spans;
            }
        }
    } else if (p->algo == BCAST_ALGO_CHAIN && r->chunk == 0 && tuned && e.chain_chunk_bytes != 0 && mode_fits(e.chain_rank_waves)) {
        r->chunk = e.chain_chunk_bytes;
        if (r->stages == 0) r->stages = e.chain_stages;
        if (r->trip == 0) r->trip = e.chain_trip_bytes;
        r->rank_waves = e.chain_rank_waves != 0;
        if (r->stage_store == BCAST_STORE_AUTO) r->stage_store = e.chain_stage_store;
        if (r->lanes == 0) r->lanes = e.chain_lanes;
        r->spans = e.chain_spans;
    }
    // no request and no table entry: write-back for small messages, whose time is
    // the sum of their hops' round trips, write-through for those that stream
    if (r->stage_store == BCAST_STORE_AUTO) r->stage_store = bytes <= kStageWriteBackMaxBytes ? BCAST_STORE_BACK : BCAST_STORE_THROUGH;
    r->radix = p->radix_request;
    if (r->algo == BCAST_ALGO_KNOMIAL || r->algo == BCAST_ALGO_KNOMIAL_PIPELINED) {
        // an AUTO plan takes the radix the table recorded (in the stages column)
        if (r->radix == 0 && p->algo == BCAST_ALGO_AUTO && tuned && e.algo == r->algo) r->radix = e.stages;
        if (r->radix < 2) r->radix = 4;
        r->radix = std::min(r->radix, std::max(2, p->nranks));
        r->stages = 0;
    }
    if (r->algo == BCAST_ALGO_KNOMIAL_PIPELINED) {
        // default chunk: one 4 KiB trip for each of a position's wavefronts
        if (r->chunk == 0) r->chunk = tree_lanes_max(p) * trip_bytes_of(kTripUnrollDefault);
        r->chunk = round_up(r->chunk, 16);
    }
    if (r->algo == BCAST_ALGO_CHAIN && r->rank_waves) {
        r->chunk = round_up(r->chunk, 16);  // 0 = one trip per lane and chunk (rank_chain_geometry)
        return BCAST_OK;
    }
    if (r->algo == BCAST_ALGO_CHAIN) {
        if (r->stages == 0) r->stages = default_stages(p->nranks);
        // without a table: 3 KiB trips where they were measured to win (8 ranks
        // and more, messages of 8 MiB and more), provided the chunk follows suit
        if (!valid_trip((u64)r->trip))
            r->trip = (int)trip_bytes_of(r->chunk == 0 && p->nranks >= 8 && bytes >= ((size_t)8 << 20) ? kTripUnrollSmall
                                                                                                      : kTripUnrollDefault);
        if (r->chunk == 0) r->chunk = default_chunk(p->nranks, waves_for(p, bytes), r->stages, (u64)r->trip);
        r->chunk = round_up(r->chunk, 16);
    }
    return BCAST_OK;
}

// Grid for the plain copy kernels: enough 4-wave workgroups to cover the
// bytes once, capped at a few workgroups per CU (waves stride beyond that).
static int copy_grid(const bcast_plan *p, u64 bytes, int concurrent_copies)
{
    u64 need = std::max<u64>(1, ceil_div(bytes, kTileBytes * kWavesPerBlock));
    u64 cap = std::max<u64>(1, (u64)p->cu_count * 8 / std::max(1, concurrent_copies));
    return (int)std::min(need, cap);
}

// Scatter + ring allgather (Sec. III-A, Eq. 4) as a list of launches, each a set
// of (src position, dst position, byte range) copies.  Pieces: position q owns
// bytes [q * piece, (q+1) * piece) clipped to the message, piece = ceil(M / P).
// Binomial scatter: strides from the top power of two down; a position that is
// a multiple of 2*stride hands the upper half of the pieces it holds to position
// + stride.  Ring: in step t position q passes piece (q - t) mod P to q + 1,
// with wrap-around; the copy that would land in the root (which already owns
// everything and is input only) is left out.
struct SagLaunch {
    RangedCopyArgs args;
    u64 max_range;
};

template <typename F>
static void walk_scatter_allgather(int P, u64 M, F &&emit)
{
    const u64 piece = ceil_div(M, (u64)P);
    auto piece_lo = [&](u64 q) { return std::min(q * piece, M); };
    int top = 1;
    while (top < P) top *= 2;
    for (int stride = top / 2; stride >= 1; stride /= 2) {
        SagLaunch l;
        memset(&l, 0, sizeof l);
        for (int q = 0; q + stride < P; q += 2 * stride) {
            const int last = std::min(q + 2 * stride, P);
            const unsigned n = l.args.npairs++;
            l.args.src_pos[n] = (unsigned char)q;
            l.args.dst_pos[n] = (unsigned char)(q + stride);
            l.args.lo[n] = piece_lo((u64)(q + stride));
            l.args.hi[n] = piece_lo((u64)last);
            l.max_range = std::max(l.max_range, l.args.hi[n] - l.args.lo[n]);
        }
        emit(l);
    }
    for (int t = 0; t < P - 1; ++t) {
        SagLaunch l;
        memset(&l, 0, sizeof l);
        for (int q = 0; q < P; ++q) {
            const int dst = (q + 1) % P;
            if (dst == 0) continue;
            const int pc = ((q - t) % P + P) % P;
            const unsigned n = l.args.npairs++;
            l.args.src_pos[n] = (unsigned char)q;
            l.args.dst_pos[n] = (unsigned char)dst;
            l.args.lo[n] = piece_lo((u64)pc);
            l.args.hi[n] = piece_lo((u64)pc + 1);
            l.max_range = std::max(l.max_range, l.args.hi[n] - l.args.lo[n]);
        }
        emit(l);
    }
}

// Launch shape of the chain with one wavefront per rank: a stage is a workgroup
// of (hops of the stage) waves, `lanes` workgroups per stage, all resident at
// once.  Rules without a measurement (from the sweeps on MI355X): stages so that
// a workgroup holds at most 8 ranks; 8 KiB trips; lanes so that the waves of a
// compute unit have about 64 KiB of trips in flight (a power of two, like the
// staged chain's lanes); one trip per lane and chunk.  From 16 MiB and 10 ranks up,
// where the hand-offs go through LDS: 16 ranks per workgroup, 4 KiB trips, 8 trips
// per lane and chunk (see `deep` below).
constexpr int kRankWavesPreferred = 8;
constexpr u64 kRankTripDefault = 8192;
constexpr u64 kRankBytesPerCu = 64u << 10;
constexpr u64 kRankDeepMinBytes = 16u << 20;
constexpr u64 kRankDeepTripBytes = 4096;
constexpr u64 kRankDeepTripsPerChunk = 8;

static int rank_chain_geometry(bcast_plan *p, size_t bytes, u64 chunk, int stages_request, int trip_request, int lanes_request,
                               bcast_plan_info_t *info)
{
    const int P = p->nranks;
    memset(info, 0, sizeof *info);
    info->algo = BCAST_ALGO_CHAIN;
    info->vec_bytes = 16;
    info->rank_waves = 1;
    info->chunk_bytes = chunk;
    if (P < 2 || bytes == 0) return BCAST_OK;
    const int hops = P - 1;
    // Long chains of a message that streams, with stages and trips left open and LDS at hand for the hand-offs:
    // 16 ranks per workgroup at 4 KiB trips (half the stages, so half the reads of the message from memory) and
    // several trips per lane and chunk -- measured at 64 ranks x 1 GiB 10.3-10.4 ms against 10.7-10.9 with 8 ranks
    // per workgroup and 8 KiB trips, at 32 ranks x 512 MiB 2.60 against 2.69 ms.
    const bool deep = stages_request == 0 && trip_request == 0 && hops > kRankWavesPreferred && bytes >= kRankDeepMinBytes &&
                      p->rank_handoff != BCAST_HANDOFF_CACHE &&
                      rank_chain_lds_bytes(kRankWavesMax, (int)(kRankDeepTripBytes / (kWaveSize * 16)), 16) + kRankStaticLdsBytes <=
                          (u64)p->lds_per_block;
    // as many stages as asked for, but no stage longer than a workgroup can hold waves
    const int per_workgroup = deep ? kRankWavesMax : kRankWavesPreferred;
    int stages = stages_request > 0 ? std::min(stages_request, hops) : (hops + per_workgroup - 1) / per_workgroup;
    stages = std::max(stages, (hops + kRankWavesMax - 1) / kRankWavesMax);
    const int waves = (hops + stages - 1) / stages;  // of the longest stage = of every workgroup
    if (p->rank_blocks_per_cu[waves] == 0) {
        int n = 0;
        HIP_TRY(rank_chain_max_blocks_per_cu(waves * kWaveSize, &n));
        p->rank_blocks_per_cu[waves] = std::max(1, std::min(n, 32 / waves));
    }
    const u64 trip = trip_request ? (u64)trip_request : (deep ? kRankDeepTripBytes : kRankTripDefault);
    if (!valid_rank_trip(trip)) return BCAST_ERR_ARG;
    // trips between the ranks of a workgroup through LDS (two slots per wave, beside the kernel's own
    // counters) where that fits, else through the compute unit's cache
    const u64 lds = rank_chain_lds_bytes(waves, (int)(trip / (kWaveSize * 16)), 16) + kRankStaticLdsBytes;
    const bool lds_fits = lds <= (u64)p->lds_per_block;
    if (p->rank_handoff == BCAST_HANDOFF_LDS && !lds_fits) return BCAST_ERR_ARG;
    // left to the library: LDS for messages that stream (measured crossover 1-4 MiB: below it a hop is an LDS
    // round trip more with nothing to overlap it with, 42 vs 38 us for 4 KiB over 64 ranks)
    const bool via_lds = waves > 1 && lds_fits &&
                         (p->rank_handoff == BCAST_HANDOFF_LDS || (p->rank_handoff == BCAST_HANDOFF_AUTO && bytes > kRankLdsMinBytes));
    info->rank_handoff = via_lds ? BCAST_HANDOFF_LDS : BCAST_HANDOFF_CACHE;
    u64 blocks_per_cu = (u64)p->rank_blocks_per_cu[waves];
    if (via_lds) blocks_per_cu = std::max<u64>(1, std::min<u64>(blocks_per_cu, (u64)p->lds_per_cu / lds));
    // every workgroup resident at once, and a flag for every (stage, lane)
    const u64 lanes_most = std::min<u64>(blocks_per_cu * p->cu_count, (u64)p->max_flags) / stages;
    if (lanes_most < 1) return BCAST_ERR_ARG;
    auto pow2_floor = [](u64 x) {
        u64 l = 1;
        while (l * 2 <= x) l *= 2;
        return l;
    };
    const u64 lanes_rule = pow2_floor(std::max<u64>(1, kRankBytesPerCu * p->cu_count / (trip * waves * stages)));
    u64 lanes;
    if (lanes_request > 0) {  // the plan's, else the table's
        lanes = std::min<u64>((u64)lanes_request, lanes_most);
    } else if (chunk == 0) {
        lanes = std::min(lanes_rule, pow2_floor(std::min<u64>(lanes_most, std::max<u64>(1, ceil_div(bytes, trip)))));
    } else {
        // a given chunk: a lane should own at least one trip of it
        lanes = pow2_floor(std::min<u64>(std::min(lanes_rule, lanes_most), std::max<u64>(1, ceil_div(std::min<u64>(chunk, bytes), trip))));
    }
    if (chunk == 0) chunk = lanes * trip * (deep && stages >= 2 ? kRankDeepTripsPerChunk : 1);
    const u64 C = std::min<u64>(chunk, round_up(bytes, 16));
    const u64 nchunks = ceil_div(bytes, C);
    if (C == 0 || C % 16 != 0 || nchunks >= (1ull << 27)) return BCAST_ERR_ARG;
    info->chunk_bytes = C;
    info->nchunks = nchunks;
    info->stages = stages;
    info->hops_per_stage = waves;
    info->lanes = (int)lanes;
    info->trip_bytes = (int)trip;
    info->slice_bytes = ceil_div(C, lanes * trip) * trip;
    info->grid_blocks = (int)((u64)stages * lanes);
    info->block_threads = waves * kWaveSize;
    info->launches = 1;
    info->algorithmic_bytes = 2ull * hops * bytes;
    return BCAST_OK;
}

static int describe(bcast_plan *p, void *const *rank_bufs, size_t bytes, bcast_plan_info_t *info)
{
    Resolved r;
    int rc = resolve(p, bytes, &r);
    if (rc != BCAST_OK) return rc;
    const int P = p->nranks;
    const int vec = common_vec_bytes(rank_bufs, P);
    if (r.algo == BCAST_ALGO_CHAIN && r.rank_waves) {
        rc = rank_chain_geometry(p, bytes, r.chunk, r.stages, r.trip, r.lanes, info);
        if (rc != BCAST_OK) return rc;
        info->vec_bytes = vec;
        info->stage_store = r.stage_store;
        return BCAST_OK;
    }
    if (r.algo == BCAST_ALGO_CHAIN) {
        const bcast_chain_request_t req = {r.lanes, r.stages, r.trip, p->block_request};
        rc = bcast_chain_geometry(P, bytes, (size_t)r.chunk, waves_for(p, bytes), &req, info);
        if (rc != BCAST_OK) return rc;
        info->vec_bytes = vec;
        info->rotating_spans = info->stages > 0 && rotate_spans(p->mode, r.spans, P - 1, info->stages) ? 1 : 0;
        info->stage_store = r.stage_store;
        return BCAST_OK;
    }
    memset(info, 0, sizeof *info);
    info->algo = r.algo;
    info->chunk_bytes = bytes;
    info->nchunks = bytes ? 1 : 0;
    info->block_threads = kBlockThreads;
    info->vec_bytes = vec;
    if (P < 2 || bytes == 0) return BCAST_OK;
    switch (r.algo) {
    case BCAST_ALGO_DIRECT:
        info->launches = P - 1;
        info->grid_blocks = copy_grid(p, bytes, 1);
        info->algorithmic_bytes = 2ull * (P - 1) * bytes;
        break;
    case BCAST_ALGO_BINOMIAL: {
        int rounds = 0;
        for (int reach = 1; reach < P; reach *= 2) ++rounds;
        info->launches = rounds;
        info->grid_blocks = copy_grid(p, bytes, 1);
        info->algorithmic_bytes = 2ull * (P - 1) * bytes;
        break;
    }
    case BCAST_ALGO_KNOMIAL: {
        int rounds = 0;
        for (long reach = 1; reach < P; reach *= r.radix) ++rounds;
        info->launches = rounds;
        info->stages = r.radix;  // reported here: the tree's radix
        info->grid_blocks = copy_grid(p, bytes, 1);
        info->algorithmic_bytes = 2ull * (P - 1) * bytes;
        break;
    }
    case BCAST_ALGO_KNOMIAL_PIPELINED: {
        const u64 trip = trip_bytes_of(kTripUnrollDefault);
        const u64 C = std::min<u64>(r.chunk, round_up(bytes, 16));
        const u64 nchunks = ceil_div(bytes, C);
        if (nchunks >= (1ull << 27)) return BCAST_ERR_ARG;  // the flag word keeps the count in 28 bits
        u64 lanes = std::max<u64>(1, std::min(tree_lanes_max(p), ceil_div(C, trip)));
        if (p->lanes_request > 0) lanes = std::min<u64>((u64)p->lanes_request, (u64)p->max_waves_tree / (u64)(P - 1));
        else {
            u64 l = 1;
            while (l * 2 <= lanes) l *= 2;
            lanes = l;
        }
        if (lanes < 1) return BCAST_ERR_ARG;
        info->chunk_bytes = C;
        info->nchunks = nchunks;
        info->lanes = (int)lanes;
        info->trip_bytes = (int)trip;
        info->slice_bytes = ceil_div(C, lanes * trip) * trip;
        info->stages = r.radix;  // reported here: the tree's radix
        info->hops_per_stage = 1;
        info->launches = 1;
        info->grid_blocks = (int)ceil_div((u64)(P - 1) * lanes, kWavesPerBlock);
        info->algorithmic_bytes = 2ull * (P - 1) * bytes;
        break;
    }
    case BCAST_ALGO_FANOUT:
        info->launches = 1;
        info->grid_blocks = copy_grid(p, bytes, 1);
        info->algorithmic_bytes = (u64)P * bytes;
        break;
    case BCAST_ALGO_SCATTER_ALLGATHER: {
        u64 moved = 0;
        int launches = 0;
        walk_scatter_allgather(P, bytes, [&](const SagLaunch &l) {
            ++launches;
            for (unsigned i = 0; i < l.args.npairs; ++i) moved += l.args.hi[i] - l.args.lo[i];
        });
        info->launches = launches;
        info->chunk_bytes = ceil_div(bytes, (u64)P);  // the piece size
        info->nchunks = (u64)P;
        info->grid_blocks = copy_grid(p, info->chunk_bytes, P - 1);
        info->algorithmic_bytes = 2 * moved;
        break;
    }
    default:
        return BCAST_ERR_ARG;
    }
    return BCAST_OK;
}

extern "C" int bcast_plan_info(bcast_plan_t *p, void *const *rank_bufs, size_t bytes, bcast_plan_info_t *info)
{
    if (!p || !info || bytes > p->bytes) return BCAST_ERR_ARG;
    return describe(p, rank_bufs, bytes, info);
}

// Where a run's ready flags live and which run counter tells its runs apart:
// the plan's own flags with the host's count or (replayable plans) the plan's
// word in device memory, or the static scratch array's flags with that array's
// word -- always in device memory there, because every plan on the device shares
// the array and its callers may replay captured launches.
struct FlagHome {
    u64 *flags;
    u64 *abort_word;
    u64 *epoch;       // host counter of runs that used these flags, or null
    u64 *epoch_word;  // ... or the counter in device memory, advanced by a kernel ahead of every run
    u64 clear_words;  // 64-bit words from `flags` on to clear before the counter wraps
};

// What the chain, the pipelined tree and the reduction share: buffers by
// position, ready flags, status words and wait limit, the chunking, and a fresh
// epoch.  uses_flags: whether any wave of the launch waits for or raises a flag
// (a single stage does neither and needs no epoch).
static int begin_flag_run(bcast_plan *p, ChainArgs *a, char *const *by_pos, size_t bytes, const bcast_plan_info_t &info,
                          const FlagHome &home, bool uses_flags, hipStream_t stream)
{
    memset(a, 0, sizeof *a);
    memcpy(a->buf, by_pos, sizeof(char *) * p->nranks);
    a->flags = home.flags;
    a->abort_word = home.abort_word;
    a->status = p->d_status;
    a->bytes = bytes;
    a->chunk_bytes = info.chunk_bytes;
    a->spin_ticks = p->spin_ticks;
    a->nchunks = (unsigned)info.nchunks;
    a->lanes = (unsigned)info.lanes;
    a->nranks = (unsigned)p->nranks;
    a->mute_hop = (unsigned)p->mute_hop;
    if (a->nchunks == 0 || a->lanes == 0 || a->chunk_bytes == 0) return BCAST_ERR_ARG;
    if ((u64)a->nchunks * a->chunk_bytes < a->bytes) return BCAST_ERR_ARG;
    // The flag word keeps the epoch in its upper 32 bits: before that would
    // wrap (after 2^32 - 2 runs on these flags), the flags and the abort word
    // are cleared and the count starts from one again.
    if (home.epoch_word) {
        // counted on the device: one small kernel ahead of the run adds one (and
        // clears at the wrap); nothing here waits, allocates or differs from
        // replay to replay
        a->epoch_word = home.epoch_word;
        if (uses_flags) HIP_TRY(launch_advance_epoch(home.epoch_word, home.flags, home.clear_words, kEpochLimit, stream));
        return BCAST_OK;
    }
    if (*home.epoch >= kEpochLimit) {
        HIP_TRY(hipDeviceSynchronize());
        HIP_TRY(hipMemset(home.flags, 0, home.clear_words * sizeof(u64)));
        HIP_TRY(hipDeviceSynchronize());
        *home.epoch = 0;
    }
    a->base = (++*home.epoch) << 32;
    return BCAST_OK;
}

static FlagHome plan_flags(bcast_plan *p)
{
    const u64 clear_words = ((u64)p->max_flags + 2) * kFlagStrideWords;  // flags, abort word, counters
    if (p->replayable) return FlagHome{p->d_flags, p->d_abort, nullptr, p->d_epoch, clear_words};
    return FlagHome{p->d_flags, p->d_abort, &p->epoch, nullptr, clear_words};
}

extern "C" int bcast_run(bcast_plan_t *p, void *const *rank_bufs, int root, size_t bytes, bcast_stream_t stream)
{
    if (!p || !rank_bufs) return BCAST_ERR_ARG;
    const int P = p->nranks;
    if (root < 0 || root >= P || bytes > p->bytes) return BCAST_ERR_ARG;
    for (int i = 0; i < P; ++i)
        if (!rank_bufs[i]) return BCAST_ERR_ARG;
    // buffers must not overlap over the message (duplicates included): sorted by
    // address, every buffer must end before the next one begins
    {
        uintptr_t at[BCAST_MAX_RANKS];
        for (int i = 0; i < P; ++i) at[i] = (uintptr_t)rank_bufs[i];
        std::sort(at, at + P);
        for (int i = 0; i + 1 < P; ++i)
            if (at[i + 1] == at[i] || at[i + 1] - at[i] < bytes) return BCAST_ERR_ARG;
    }
    if (P < 2 || bytes == 0) return BCAST_OK;

    bcast_plan_info_t info;
    int rc = describe(p, rank_bufs, bytes, &info);
    if (rc != BCAST_OK) return rc;

    // chain position k is rank (root + k) mod P: no wrap-around back to the root
    char *by_pos[BCAST_MAX_RANKS];
    for (int k = 0; k < P; ++k) by_pos[k] = (char *)rank_bufs[(root + k) % P];

    if (info.algo == BCAST_ALGO_CHAIN) {
        ChainArgs a;
        rc = begin_flag_run(p, &a, by_pos, bytes, info, plan_flags(p), info.stages > 1, stream);
        if (rc != BCAST_OK) return rc;
        a.counters = p->d_counters;
        a.trace = p->d_trace;
        a.trace_entries = p->trace_entries;
        a.mode = p->mode & ~(kModeFixedSpans | kModeRotateSpans);
        if (!info.rotating_spans) a.mode |= kModeFixedSpans;
        // cache policies: everything another wave reads or wrote at agent scope;
        // the wave's own read-back cached; its in-stage stores write-through, or
        // write-back for small messages
        const int chosen[4] = {kAuxAgent, kAuxAgent, kAuxCached, info.stage_store == BCAST_STORE_BACK ? kAuxCached : kAuxAgent};
        unsigned char pol[4];
        for (int i = 0; i < 4; ++i) pol[i] = (unsigned char)(p->policy_request[i] >= 0 ? p->policy_request[i] : chosen[i]);
        a.ld_root = pol[0];
        a.ld_edge = pol[1];
        a.ld_back = pol[2];
        a.st_mid = pol[3];
        if (p->d_trace) a.mode |= kModeTrace;
        a.stages = (unsigned)info.stages;
        a.hops_per_stage = (unsigned)info.hops_per_stage;
        a.unroll = (unsigned)(info.trip_bytes / (kWaveSize * 16));
        if (info.rank_waves) {
            a.mode |= kModeFixedSpans;
            if (info.rank_handoff == BCAST_HANDOFF_LDS) a.mode |= kModeLdsHandoff;
            if ((u64)a.stages * a.lanes > (u64)p->max_flags) return BCAST_ERR_ARG;
            HIP_TRY(launch_rank_chain(a, info.vec_bytes, info.grid_blocks, info.block_threads, p->device, p->lds_per_block, stream));
            return BCAST_OK;
        }
        // the launch must match what the kernel indexes: stages*lanes waves, each with its own flag,
        // and no more stages than hops
        if ((u64)a.stages * a.lanes > (u64)waves_for(p, bytes)) return BCAST_ERR_ARG;
        if ((u64)info.grid_blocks * (u64)(info.block_threads / kWaveSize) < (u64)a.stages * a.lanes) return BCAST_ERR_ARG;
        if (a.stages == 0 || a.stages > (unsigned)(P - 1)) return BCAST_ERR_ARG;
        if (a.nchunks == 0 || a.lanes == 0 || a.chunk_bytes == 0) return BCAST_ERR_ARG;
        if ((u64)a.nchunks * a.chunk_bytes < a.bytes) return BCAST_ERR_ARG;
        HIP_TRY(launch_chain(a, info.vec_bytes, info.grid_blocks, info.block_threads, stream));
        return BCAST_OK;
    }

    CopyArgs c;
    memset(&c, 0, sizeof c);
    memcpy(c.buf, by_pos, sizeof(char *) * P);
    c.nranks = (unsigned)P;
    c.lo = 0;
    c.hi = bytes;
    if (info.algo == BCAST_ALGO_DIRECT) {
        // a serialized loop of point-to-point sends from the root (Eq. 1)
        for (int k = 1; k < P; ++k) {
            c.npairs = 1;
            c.src_pos[0] = 0;
            c.dst_pos[0] = (unsigned char)k;
            HIP_TRY(launch_pair_copy(c, info.vec_bytes, info.grid_blocks, stream));
        }
        return BCAST_OK;
    }
    if (info.algo == BCAST_ALGO_BINOMIAL) {
        // round j: every position q < 2^j sends to q + 2^j (Eq. 3, k = 2);
        // stream order between launches is the round barrier
        for (int reach = 1; reach < P; reach *= 2) {
            unsigned n = 0;
            for (int q = 0; q < reach && q + reach < P; ++q) {
                c.src_pos[n] = (unsigned char)q;
                c.dst_pos[n] = (unsigned char)(q + reach);
                ++n;
            }
            c.npairs = n;
            HIP_TRY(launch_pair_copy(c, info.vec_bytes, copy_grid(p, bytes, (int)n), stream));
        }
        return BCAST_OK;
    }
    if (info.algo == BCAST_ALGO_FANOUT) {
        HIP_TRY(launch_fanout(c, info.vec_bytes, info.grid_blocks, stream));
        return BCAST_OK;
    }
    if (info.algo == BCAST_ALGO_KNOMIAL_PIPELINED) {
        ChainArgs a;
        rc = begin_flag_run(p, &a, by_pos, bytes, info, plan_flags(p), true, stream);
        if (rc != BCAST_OK) return rc;
        const int k = info.stages;
        if (k < 2) return BCAST_ERR_ARG;
        if ((u64)(P - 1) * a.lanes > (u64)p->max_waves_tree) return BCAST_ERR_ARG;
        // the k-nomial tree of Eq. 3: position q = holder + i k^j (holder < k^j,
        // 1 <= i < k) receives from holder, i.e. from q without its leading
        // base-k digit
        for (long reach = 1; reach < P; reach *= k)
            for (long holder = 0; holder < reach; ++holder)
                for (long i = 1; i < k; ++i) {
                    const long child = holder + i * reach;
                    if (child >= P) continue;
                    a.parent[child] = (unsigned char)holder;
                    a.forward_mask |= 1ull << holder;
                }
        HIP_TRY(launch_tree(a, info.vec_bytes, info.grid_blocks, stream));
        return BCAST_OK;
    }
    if (info.algo == BCAST_ALGO_KNOMIAL) {
        // round j: every holder q < k^j sends to q + i k^j, i = 1..k-1 (Eq. 3); all
        // copies of a round go out in one launch, stream order is the round barrier
        const int k = info.stages;
        if (k < 2) return BCAST_ERR_ARG;
        for (long reach = 1; reach < P; reach *= k) {
            RangedCopyArgs ra;
            memset(&ra, 0, sizeof ra);
            memcpy(ra.buf, by_pos, sizeof(char *) * P);
            for (long q = 0; q < reach; ++q)
                for (long i = 1; i < k; ++i) {
                    const long child = q + i * reach;
                    if (child >= P) continue;
                    const unsigned n = ra.npairs++;
                    ra.src_pos[n] = (unsigned char)q;
                    ra.dst_pos[n] = (unsigned char)child;
                    ra.lo[n] = 0;
                    ra.hi[n] = bytes;
                }
            HIP_TRY(launch_ranged_copy(ra, info.vec_bytes, copy_grid(p, bytes, (int)ra.npairs), stream));
        }
        return BCAST_OK;
    }
    if (info.algo == BCAST_ALGO_SCATTER_ALLGATHER) {
        hipError_t err = hipSuccess;
        walk_scatter_allgather(P, bytes, [&](SagLaunch &l) {
            if (err != hipSuccess || l.max_range == 0) return;  // a round of empty pieces moves nothing
            memcpy(l.args.buf, by_pos, sizeof(char *) * P);
            err = launch_ranged_copy(l.args, info.vec_bytes, copy_grid(p, l.max_range, (int)l.args.npairs), stream);
        });
        HIP_TRY(err);
        return BCAST_OK;
    }
    return BCAST_ERR_ARG;
}

// Launch shape of a reduction of `bytes` bytes: the chain's geometry (stages of
// consecutive hops, lanes, chunks) with 4 KiB trips and fixed spans, inside what
// the staging memory (`staging_bytes`, for the running sums that cross a stage
// boundary: one region of round_up(bytes, 256) per boundary) and the flags
// (`max_waves`) allow.  A stage count the caller asked for is an error if the
// staging memory cannot carry it (BCAST_ERR_CAPACITY); the library's own choice
// shrinks to what fits (one stage needs none).
static int reduce_shape(const bcast_plan *p, size_t bytes, size_t staging_bytes, int max_waves, bcast_plan_info_t *info)
{
    const int hops = std::max(1, p->nranks - 1);
    // what the plan leaves open comes from the reduction's tuning table, if it has an entry
    bcast_reduce_entry_t e;
    const bool tuned = p->nranks >= 2 && bytes > 0 && bcast_tune_reduce_get(p->nranks, bytes, &e) == BCAST_OK;
    const bool open_shape = p->chunk_bytes == 0 && p->stages_request == 0;
    int stages = p->stages_request > 0 ? std::min(p->stages_request, hops)
                                       : (tuned && open_shape ? std::min(e.stages, hops) : default_stages(p->nranks));
    if (p->nranks >= 2 && bytes > 0) {
        const u64 region = round_up(bytes, 256);
        const u64 fit = 1 + staging_bytes / region;  // stages the staging memory carries
        if ((u64)stages > fit) {
            if (p->stages_request > 0) return BCAST_ERR_CAPACITY;
            stages = (int)fit;
        }
    }
    const bool use_entry = tuned && open_shape && stages == std::min(e.stages, hops);
    // trips: 4 KiB and 4 positions loaded at a time for messages that stream, 1 KiB
    // and 16 positions for small ones (more lanes share the work, fewer dependent
    // memory round trips per stage)
    u64 trip = p->reduce_trip_request ? (u64)p->reduce_trip_request
                                      : (use_entry ? (u64)e.trip_bytes
                                                   : trip_bytes_of(bytes <= kRedSmallMaxBytes ? kRedUnrollSmall : kRedUnroll));
    size_t chunk = p->chunk_bytes;
    if (chunk == 0) chunk = use_entry ? (size_t)e.chunk_bytes : (size_t)default_chunk(p->nranks, max_waves, stages, trip_bytes_of(kRedUnroll));
    const bcast_chain_request_t req = {p->lanes_request, stages, (int)trip_bytes_of(kRedUnroll), 0};
    int rc = bcast_chain_geometry(p->nranks, bytes, chunk, max_waves, &req, info);
    if (rc != BCAST_OK) return rc;
    if (p->nranks >= 2 && bytes > 0 && trip != trip_bytes_of(kRedUnroll)) {
        const u64 most = (u64)(max_waves / info->stages);
        u64 lanes = p->lanes_request > 0 ? std::min<u64>((u64)p->lanes_request, most)
                                         : std::min<u64>(ceil_div(info->chunk_bytes, trip), most);
        if (p->lanes_request == 0) {
            u64 l = 1;
            while (l * 2 <= lanes) l *= 2;
            lanes = l;
        }
        lanes = std::max<u64>(1, lanes);
        info->lanes = (int)lanes;
        info->trip_bytes = (int)trip;
        info->slice_bytes = ceil_div(info->chunk_bytes, lanes * trip) * trip;
        info->grid_blocks = (int)ceil_div((u64)info->stages * lanes, kWavesPerBlock);
    }
    // every input byte is read once and every result byte written once
    info->algorithmic_bytes = ((u64)p->nranks + 1) * bytes;
    return BCAST_OK;
}

extern "C" int bcast_reduce_info(bcast_plan_t *p, size_t count, bcast_plan_info_t *info)
{
    if (!p || !info || count > p->bytes / sizeof(float)) return BCAST_ERR_ARG;
    return reduce_shape(p, count * sizeof(float), p->scratch_bytes, p->max_waves_reduce, info);
}

extern "C" int bcast_plan_reserve_reduce(bcast_plan_t *p, size_t count, int stages)
{
    if (!p || stages < 0 || count > p->bytes / sizeof(float)) return BCAST_ERR_ARG;
    if (stages == 0) {
        bcast_reduce_entry_t e;
        stages = p->nranks >= 2 && count > 0 && bcast_tune_reduce_get(p->nranks, count * sizeof(float), &e) == BCAST_OK
                     ? e.stages
                     : default_stages(p->nranks);
    }
    stages = std::min(stages, std::max(1, p->nranks - 1));
    const size_t need = (size_t)(stages - 1) * round_up(count * sizeof(float), 256);
    if (need <= p->scratch_bytes) return BCAST_OK;
    // earlier runs may still read the old staging memory
    HIP_TRY(hipDeviceSynchronize());
    if (p->d_scratch) {
        HIP_TRY(hipFree(p->d_scratch));
        p->d_scratch = nullptr;
        p->scratch_bytes = 0;
    }
    HIP_TRY(hipMalloc((void **)&p->d_scratch, need));
    p->scratch_bytes = need;
    return BCAST_OK;
}

// Argument checks shared by the two reduction entry points.
static int reduce_check(const bcast_plan *p, const void *const *send_bufs, const void *recv_buf, int root, size_t count)
{
    if (!p || !send_bufs || !recv_buf) return BCAST_ERR_ARG;
    const int P = p->nranks;
    if (root < 0 || root >= P || count > p->bytes / sizeof(float)) return BCAST_ERR_ARG;
    const size_t bytes = count * sizeof(float);
    // whole 16-byte vectors are moved: every buffer must start on a 16-byte boundary
    if ((uintptr_t)recv_buf & 15u) return BCAST_ERR_ARG;
    for (int i = 0; i < P; ++i)
        if (!send_bufs[i] || ((uintptr_t)send_bufs[i] & 15u)) return BCAST_ERR_ARG;
    // contributions must not overlap each other; the result may be the root's own
    // contribution (in place) but must not touch any other buffer
    uintptr_t at[BCAST_MAX_RANKS + 1];
    int n = 0;
    for (int i = 0; i < P; ++i) at[n++] = (uintptr_t)send_bufs[i];
    if (recv_buf != send_bufs[root]) at[n++] = (uintptr_t)recv_buf;
    std::sort(at, at + n);
    for (int i = 0; i + 1 < n; ++i)
        if (at[i + 1] == at[i] || at[i + 1] - at[i] < bytes) return BCAST_ERR_ARG;
    return BCAST_OK;
}

// Enqueue the reduction kernel with the given flags and staging memory.  Calls
// nothing that allocates or waits for the device (a host-counted plan's
// once-in-2^32-runs clearing aside, see begin_flag_run).
static int reduce_enqueue(bcast_plan *p, const void *const *send_bufs, void *recv_buf, int root, size_t bytes,
                          const bcast_plan_info_t &info, const FlagHome &home, char *staging, size_t staging_bytes, int max_waves,
                          hipStream_t stream)
{
    const int P = p->nranks;
    const size_t region = round_up(bytes, 256);
    if ((size_t)(info.stages - 1) * region > staging_bytes) return BCAST_ERR_CAPACITY;
    char *by_pos[BCAST_MAX_RANKS];
    for (int k = 0; k < P; ++k) by_pos[k] = (char *)const_cast<void *>(send_bufs[(root + k) % P]);
    ChainArgs a;
    int rc = begin_flag_run(p, &a, by_pos, bytes, info, home, info.stages > 1, stream);
    if (rc != BCAST_OK) return rc;
    a.stages = (unsigned)info.stages;
    a.hops_per_stage = (unsigned)info.hops_per_stage;
    a.unroll = (unsigned)(info.trip_bytes / (kWaveSize * 16));
    a.recv = (char *)recv_buf;
    a.st_mid = (unsigned char)(p->policy_request[3] >= 0 ? p->policy_request[3] : kRedResultStore);
    a.scratch = staging;
    a.scratch_stride = region;
    if ((u64)a.stages * a.lanes > (u64)max_waves) return BCAST_ERR_ARG;
    HIP_TRY(launch_reduce(a, info.grid_blocks, stream));
    return BCAST_OK;
}

extern "C" int bcast_reduce_sum_f32(bcast_plan_t *p, const void *const *send_bufs, void *recv_buf, int root, size_t count,
                                    bcast_stream_t stream)
{
    int rc = reduce_check(p, send_bufs, recv_buf, root, count);
    if (rc != BCAST_OK) return rc;
    const size_t bytes = count * sizeof(float);
    if (bytes == 0) return BCAST_OK;
    if (p->nranks == 1) {
        if (recv_buf != send_bufs[0]) HIP_TRY(hipMemcpyAsync(recv_buf, send_bufs[0], bytes, hipMemcpyDeviceToDevice, stream));
        return BCAST_OK;
    }
    bcast_plan_info_t info;
    rc = reduce_shape(p, bytes, p->scratch_bytes, p->max_waves_reduce, &info);
    if (rc != BCAST_OK) return rc;
    return reduce_enqueue(p, send_bufs, recv_buf, root, bytes, info, plan_flags(p), p->d_scratch, p->scratch_bytes,
                          p->max_waves_reduce, stream);
}

extern "C" int bcast_reduce_sum_f32_static(bcast_plan_t *p, const void *const *send_bufs, void *recv_buf, int root, size_t count,
                                           bcast_stream_t stream)
{
    int rc = reduce_check(p, send_bufs, recv_buf, root, count);
    if (rc != BCAST_OK) return rc;
    const size_t bytes = count * sizeof(float);
    if (bytes == 0) return BCAST_OK;
    if (p->nranks == 1) {
        if (recv_buf != send_bufs[0]) HIP_TRY(hipMemcpyAsync(recv_buf, send_bufs[0], bytes, hipMemcpyDeviceToDevice, stream));
        return BCAST_OK;
    }
    // the static array of the device the plan was made on (its address was looked
    // up at plan creation): flags first, staging after them
    int device = -1;
    HIP_TRY(hipGetDevice(&device));
    if (device != p->device || !p->static_scratch || device < 0 || device >= kStaticMaxDevices) return BCAST_ERR_ARG;
    const int max_waves = std::min(p->max_waves_reduce, kStaticFlagWaves);
    bcast_plan_info_t info;
    rc = reduce_shape(p, bytes, (size_t)kStaticStagingBytes, max_waves, &info);
    if (rc != BCAST_OK) return rc;
    // flags, then the abort word, then the array's run counter
    u64 *flags = reinterpret_cast<u64 *>(p->static_scratch);
    u64 *abort_word = flags + (u64)kStaticFlagWaves * kFlagStrideWords;
    const FlagHome home{flags, abort_word, nullptr, abort_word + kFlagStrideWords, ((u64)kStaticFlagWaves + 1) * kFlagStrideWords};
    return reduce_enqueue(p, send_bufs, recv_buf, root, bytes, info, home, p->static_scratch + kStaticFlagBytes,
                          (size_t)kStaticStagingBytes, max_waves, stream);
}

extern "C" int bcast_allreduce_sum_f32(bcast_plan_t *p, const void *const *send_bufs, void *const *recv_bufs, int root,
                                       size_t count, bcast_stream_t stream)
{
    if (!p || !send_bufs || !recv_bufs) return BCAST_ERR_ARG;
    const int P = p->nranks;
    if (root < 0 || root >= P || count > p->bytes / sizeof(float)) return BCAST_ERR_ARG;
    const size_t bytes = count * sizeof(float);
    // every rank's result is either its own contribution (in place) or memory that
    // touches no contribution and no other result
    {
        uintptr_t at[2 * BCAST_MAX_RANKS];
        int n = 0;
        for (int i = 0; i < P; ++i) {
            if (!send_bufs[i] || !recv_bufs[i]) return BCAST_ERR_ARG;
            at[n++] = (uintptr_t)send_bufs[i];
            if (recv_bufs[i] != send_bufs[i]) at[n++] = (uintptr_t)recv_bufs[i];
        }
        std::sort(at, at + n);
        for (int i = 0; i + 1 < n; ++i)
            if (at[i + 1] == at[i] || at[i + 1] - at[i] < bytes) return BCAST_ERR_ARG;
    }
    // the chain reduction to the root, then the root's result down the broadcast
    // chain: stream order makes the second wait for the first
    int rc = bcast_reduce_sum_f32(p, send_bufs, recv_bufs[root], root, count, stream);
    if (rc != BCAST_OK) return rc;
    return bcast_run(p, recv_bufs, root, bytes, stream);
}

// Measurement calls (bcast_debug.h): the two dependency-free access patterns.
static int pattern_args(void *const *bufs, int nbufs, size_t bytes, CopyArgs *c)
{
    if (!bufs || nbufs < 1 || nbufs > BCAST_MAX_RANKS || bytes == 0 || bytes % kTileBytes != 0) return BCAST_ERR_ARG;
    memset(c, 0, sizeof *c);
    for (int i = 0; i < nbufs; ++i) {
        if (!bufs[i] || ((uintptr_t)bufs[i] & 15u)) return BCAST_ERR_ARG;
        c->buf[i] = (char *)bufs[i];
    }
    c->nranks = (unsigned)nbufs;
    c->hi = bytes;
    return BCAST_OK;
}

static int pattern_grid(size_t bytes)
{
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 2048;
    const u64 need = std::max<u64>(1, ceil_div(bytes, kTileBytes * kWavesPerBlock));
    return (int)std::min<u64>(need, (u64)prop.multiProcessorCount * 8);
}

extern "C" int bcast_debug_store_pattern(void *const *bufs, int nbufs, size_t bytes, bcast_stream_t stream)
{
    CopyArgs c;
    int rc = pattern_args(bufs, nbufs, bytes, &c);
    if (rc != BCAST_OK) return rc;
    HIP_TRY(launch_store_pattern(c, pattern_grid(bytes), stream));
    return BCAST_OK;
}

extern "C" int bcast_debug_load_pattern(void *const *bufs, int nbufs, size_t bytes, void *out, int write_result, bcast_stream_t stream)
{
    CopyArgs c;
    int rc = pattern_args(bufs, nbufs, bytes, &c);
    if (rc != BCAST_OK) return rc;
    if (!out || ((uintptr_t)out & 15u)) return BCAST_ERR_ARG;
    HIP_TRY(launch_load_pattern(c, (char *)out, write_result != 0, pattern_grid(bytes), stream));
    return BCAST_OK;
}

extern "C" const char *bcast_strerror(int status)
{
    switch (status) {
    case BCAST_OK: return "ok";
    case BCAST_ERR_ARG: return "invalid argument";
    case BCAST_ERR_NOMEM: return "out of memory";
    case BCAST_ERR_HIP: return "HIP runtime call failed";
    case BCAST_ERR_TIMEOUT: return "chain wave gave up waiting for its left neighbour";
    case BCAST_ERR_UNTUNED: return "no tuning table entry for this number of ranks";
    case BCAST_ERR_CAPACITY: return "staging memory too small for this size and stage count (reserve more, or beyond the static array's limit)";
    default: return "unknown status";
    }
}

extern "C" int bcast_last_hip_error(void) { return g_last_hip_error; }

extern "C" const char *bcast_version(void) { return "bcast-gfx950 0.2"; }

/*
 * bcast.h -- C ABI of the single-GPU broadcast library for MI355X (gfx950).
 *
 * The library implements the rooted broadcast of the paper's Sec. I / III-A
 * (MPI_Bcast: every rank owns one buffer, the root's is the input, afterwards
 * every buffer holds the root's bytes) for P "virtual ranks" that are P
 * distinct device buffers in one GPU's HBM.  The flagship algorithm is the
 * pipelined chain of Sec. IV-B (Eq. 5); the direct algorithm (Eq. 1), the
 * binomial and k-nomial trees (Eq. 3; per level, and pipelined in one launch),
 * scatter + ring allgather (Eq. 4), a one-die fan-out and a tuning table that
 * picks algorithm and chunk size per (message bytes, ranks) (Sec. III-B, IV-B)
 * sit beside it, and so does the chain run backwards as a rooted fp32 sum
 * (MPI_Reduce, the collective Sec. VII names next), alone or followed by the
 * broadcast (MPI_Allreduce).
 *
 * Conventions for every call
 *   - Plain C linkage, no C++ or torch types.  Every pointer argument says
 *     whether it is a HOST or a DEVICE pointer.
 *   - Return value: BCAST_OK (0) or a negative bcast_status_t.  Nothing
 *     aborts or throws.  After BCAST_ERR_HIP, bcast_last_hip_error() gives the
 *     hipError_t value of the failing runtime call on this thread.
 *   - The caller owns all rank buffers and the rank_bufs array; the library
 *     owns what a plan allocates (ready flags, status word, the reduction's
 *     scratch buffer) until bcast_plan_destroy.
 *   - Streams are passed as HIP's own handle type.  To keep this header free
 *     of HIP includes it is spelled bcast_stream_t, which is the same type as
 *     hipStream_t (struct ihipStream_t *); NULL is the default stream.
 */
#ifndef BCAST_H
#define BCAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BCAST_MAX_RANKS 64

typedef struct ihipStream_t *bcast_stream_t; /* == hipStream_t */
typedef struct bcast_plan bcast_plan_t;      /* opaque, library-owned */

typedef enum {
    BCAST_ALGO_AUTO = 0,     /* look (bytes, nranks) up in the tuning table (Sec. IV-B, last paragraph) */
    BCAST_ALGO_CHAIN = 1,    /* pipelined chain, Sec. IV-B Eq. 5; one chunk = plain chain, Eq. 2 */
    BCAST_ALGO_DIRECT = 2,   /* root copies to each other rank in turn, Sec. III-A Eq. 1 */
    BCAST_ALGO_BINOMIAL = 3, /* binomial tree, Sec. III-A Eq. 3 with k = 2 */
    BCAST_ALGO_FANOUT = 4,   /* one-die shortcut: read root once, store to all ranks (no paper equivalent) */
    BCAST_ALGO_SCATTER_ALLGATHER = 5, /* binomial scatter + ring allgather, Sec. III-A Eq. 4 */
    BCAST_ALGO_KNOMIAL = 6,  /* k-nomial tree, Sec. III-A Eq. 3, radix from bcast_plan_set_radix (default 4) */
    BCAST_ALGO_KNOMIAL_PIPELINED = 7 /* the same tree in ONE launch, chunked and flag-driven like the chain
                                        (Sec. IV-B's pipelining applied to Eq. 3's tree): every position copies
                                        chunk c out of its parent's buffer as soon as the parent holds it */
} bcast_algo_t;

typedef enum {
    BCAST_OK = 0,
    BCAST_ERR_ARG = -1,     /* invalid argument; nothing was enqueued */
    BCAST_ERR_NOMEM = -2,   /* host or device allocation failed */
    BCAST_ERR_HIP = -3,     /* a HIP runtime call failed; see bcast_last_hip_error() */
    BCAST_ERR_TIMEOUT = -4, /* a chain wave gave up waiting for its left neighbour */
    BCAST_ERR_UNTUNED = -5, /* BCAST_ALGO_AUTO but the table has no entry for this nranks */
    BCAST_ERR_CAPACITY = -6 /* the staging memory at hand (reserved for the plan, or the library's static
                               array) cannot carry this size at this stage count; nothing was enqueued */
} bcast_status_t;

/* What a plan will launch for a given message size (host-side bookkeeping). */
typedef struct {
    int algo;              /* resolved bcast_algo_t (never AUTO) */
    uint64_t chunk_bytes;  /* chunk size C in use (== bytes when unchunked) */
    uint64_t nchunks;      /* ceil(bytes / C) */
    int stages;            /* chain: groups of consecutive hops; each stage has its own wavefronts and flags */
    int hops_per_stage;    /* chain: hops a stage's wavefront plays one after the other (1 = a stage per rank);
                              where nranks-1 is no multiple of stages this is the larger of the two counts */
    int lanes;             /* chain: wavefronts per stage, each streaming its own share of every chunk */
    int rotating_spans;    /* chain: 1 if the stages that play one hop more change from chunk to chunk */
    int trip_bytes;        /* chain: bytes a wavefront moves per trip at 16-byte accesses (a multiple of 1024) */
    uint64_t slice_bytes;  /* chain: bytes of every chunk owned by one lane, in trips dealt round-robin over the lanes */
    int grid_blocks;       /* workgroups of the (first) launch */
    int block_threads;     /* threads per workgroup */
    int vec_bytes;         /* widest access usable for these pointers: 16, 8, 4 or 1 */
    int launches;          /* kernel launches per bcast_run */
    uint64_t algorithmic_bytes; /* HBM bytes the schedule must move: reads + writes */
    int rank_waves;        /* chain: 1 if every rank has wavefronts of its own (a stage is a workgroup of
                              hops_per_stage wavefronts), 0 if one wavefront plays its stage's ranks in turn */
    int stage_store;       /* chain: how stores inside a stage are issued, BCAST_STORE_THROUGH or BCAST_STORE_BACK */
    int rank_handoff;      /* chain with a wavefront per rank: how a trip travels between the ranks of a workgroup,
                              BCAST_HANDOFF_CACHE or BCAST_HANDOFF_LDS (0 otherwise) */
} bcast_plan_info_t;

/*
 * bcast_plan_create -- reserve what a broadcast among `nranks` buffers of up
 * to `bytes` bytes needs (Sec. IV-B: the chunked chain and its chunk size).
 *   out         HOST pointer; receives the plan on success, NULL otherwise.
 *   nranks      number of ranks P, 1..BCAST_MAX_RANKS (the paper's n).
 *   bytes       largest message M this plan will carry (0 allowed).
 *   chunk_bytes chunk size C for CHAIN and KNOMIAL_PIPELINED: a positive multiple
 *               of 16; values >= bytes give the unpipelined chain (Eq. 2) or
 *               tree (Eq. 3).  0 = choose: the tuning table's entry if one is
 *               loaded, else a built-in rule.  Ignored by DIRECT, BINOMIAL,
 *               KNOMIAL, FANOUT and SCATTER_ALLGATHER (whose piece size is
 *               ceil(bytes / nranks)).
 *   algo        a bcast_algo_t.  AUTO resolves per run from the tuning table and
 *               fails with BCAST_ERR_UNTUNED if no table covers nranks.
 * Allocates device memory for ready flags (zeroed once; they are never reset,
 * runs are told apart by an epoch) and a pinned host status word.
 * Errors: ERR_ARG (ranges, chunk not a multiple of 16), ERR_NOMEM, ERR_HIP.
 */
int bcast_plan_create(bcast_plan_t **out, int nranks, size_t bytes, size_t chunk_bytes, int algo);

/*
 * bcast_run -- enqueue one broadcast on `stream` (MPI_Bcast's statement of the
 * problem, Sec. I and III-A; chain order per Sec. III-A "Chain and Ring").
 *   plan       from bcast_plan_create.  One plan must not run on two streams
 *              at once (not detected); back-to-back runs on one stream are fine.
 *              Calls on one plan must come from one thread at a time; different
 *              plans are independent.
 *   rank_bufs  HOST array of plan.nranks DEVICE pointers, one per rank, on the
 *              current device, pairwise non-overlapping over `bytes`.  Read
 *              during the call only; the buffers must stay valid until the
 *              stream has passed the run.  Any byte alignment is accepted;
 *              the 128-bit path needs all pointers congruent mod 16.
 *   root       rank whose buffer is the message; it is only read.
 *   bytes      message size M, 0 <= M <= plan bytes.  Bytes at offsets >= M
 *              are never written.
 *   stream     hipStream_t to enqueue on.
 * The chain position of rank r is (r - root) mod P: the root pushes chunks to
 * rank root+1, which forwards to root+2, ... and rank root-1 only receives.
 * Returns after enqueueing; completion follows stream order.  Every run gets a
 * fresh epoch from the host as a kernel argument, so a bcast_run recorded into
 * a HIP graph must not be replayed unless the plan is replayable (see
 * bcast_plan_set_replayable).  The epoch is a 32-bit count: once in 2^32 - 2
 * runs of a plan, bcast_run waits for the device and clears the plan's flags
 * before it goes on (a replayable plan does that on the device, without waiting).
 * bytes == 0 or nranks == 1 succeed without launching.
 * Errors: ERR_ARG (NULL/duplicate/overlapping pointers, root or bytes out of
 * range), ERR_UNTUNED, ERR_HIP.  A wave that waits longer than the plan's
 * spin limit records ERR_TIMEOUT in the plan's status word (see below).
 */
int bcast_run(bcast_plan_t *plan, void *const *rank_bufs, int root, size_t bytes, bcast_stream_t stream);

/*
 * bcast_plan_status -- BCAST_OK, or BCAST_ERR_TIMEOUT if any run of this plan
 * that has finished so far hit the wait limit.  Reads a pinned host word the
 * kernels write; synchronises nothing (synchronise the stream first to cover a
 * given run).  `detail` (HOST, nullable) receives hop << 32 | chunk of the
 * first wave that gave up.  bcast_plan_clear_status resets the word.
 */
int bcast_plan_status(bcast_plan_t *plan, uint64_t *detail);
int bcast_plan_clear_status(bcast_plan_t *plan);

/*
 * bcast_plan_set_replayable -- on = 1: from now on the plan's runs (bcast_run,
 * bcast_reduce_sum_f32, bcast_allreduce_sum_f32) read their epoch from a word in
 * the plan's device memory, which a one-workgroup kernel enqueued ahead of each
 * run that uses flags advances.  Such a run enqueues kernels only -- no
 * allocation, no wait, no memset, nothing that differs from one execution to
 * the next -- so it may be recorded during stream capture and the graph
 * replayed any number of times (deep-learning steps repeat the same broadcasts
 * every iteration, Sec. I); captured and directly issued runs of the plan may
 * alternate.  What is recorded is what the call saw: buffers, root, size, the
 * launch shape and the tuning table's choice.  Costs one small launch per run.
 * on = 0 returns to the host's count.  Either change waits for the device.
 * As for any run: one plan must not run on two streams, or in two graph
 * branches, at once.  Errors: ERR_ARG, ERR_HIP.
 */
int bcast_plan_set_replayable(bcast_plan_t *plan, int on);

/* bcast_plan_info -- HOST-side description of what a run of `bytes` bytes over
 * these pointers (nullable: then 16-byte alignment is assumed) would launch. */
int bcast_plan_info(bcast_plan_t *plan, void *const *rank_bufs, size_t bytes, bcast_plan_info_t *info);

/* bcast_plan_destroy -- waits for the device, then frees the plan's memory. */
int bcast_plan_destroy(bcast_plan_t *plan);

/* Launch-shape knobs.  lanes: wavefronts per chain stage (0 = automatic).
 * stages: how many groups of consecutive hops get wavefronts of their own (0 =
 * automatic; nranks-1 = one stage per receiving rank, the literal picture of
 * Sec. IV-B; fewer = a wavefront plays several consecutive ranks in turn,
 * re-reading from each rank's buffer what it stored there, and flags are only
 * used between stages; where nranks-1 is no multiple of stages, the stages that
 * play one hop more rotate from chunk to chunk, so the stage boundaries differ
 * between chunks).  Test and diagnostic hooks are declared in bcast_debug.h. */
int bcast_plan_set_lanes(bcast_plan_t *plan, int lanes);
/* How a stage of the chain is executed (Sec. IV-B).
 * BCAST_CHAIN_WAVE_PER_RANK: every receiving rank has wavefronts of its own --
 * the literal picture of the section: receive a piece from the left neighbour,
 * store it, tell the right neighbour.  A stage is a workgroup of up to 16
 * wavefronts, one per consecutive rank, on one compute unit; neighbours inside
 * it hand a trip (the pipelining unit there, bcast_plan_set_trip) over with a
 * workgroup-scope release/acquire on a counter in LDS and the payload moves
 * through LDS or the compute unit's cache (bcast_plan_set_rank_handoff); between stages whole chunks are handed over
 * through the ready flags in memory.  stages = 0 then means: as few stages as
 * 8 ranks per workgroup allow (at least ceil((nranks-1)/16) are needed); for
 * messages from 16 MiB whose trips go through LDS, with the trip size left open
 * too: 16 ranks per workgroup at 4 KiB trips.
 * BCAST_CHAIN_WAVE_PER_STAGE: one wavefront plays all ranks of its stage in
 * turn, reading back from each rank's buffer what it stored there.
 * BCAST_CHAIN_AUTO (default): the tuning table's choice, else WAVE_PER_STAGE.
 * The bytes every rank ends up with are the same in all modes. */
#define BCAST_CHAIN_AUTO 0
#define BCAST_CHAIN_WAVE_PER_STAGE 1
#define BCAST_CHAIN_WAVE_PER_RANK 2
int bcast_plan_set_chain_waves(bcast_plan_t *plan, int mode);
/* Chain with a wavefront per rank: how a trip's payload gets from a rank to its
 * right neighbour inside a workgroup (the counters in LDS tell when in both).
 * BCAST_HANDOFF_CACHE: the neighbour reads it out of the rank's buffer, which the
 * compute unit's cache serves while the trips in flight fit it.
 * BCAST_HANDOFF_LDS: the rank stores the trip into its buffer and also into one
 * of its two trip slots in LDS, and the neighbour takes it from there: the LDS is
 * the link between the two ranks, and the buffers in memory are written and not
 * read again inside the workgroup.  Needs 2 x trip bytes of LDS per wavefront of the workgroup;
 * BCAST_ERR_ARG from bcast_run / bcast_plan_info if the device has less.
 * BCAST_HANDOFF_AUTO (default): LDS where it fits and the message is longer than
 * 2 MiB (below that the cache is the faster way), else the cache.  Trips with a
 * ragged end or a misaligned start always go through the cache.  Same bytes
 * either way; bcast_plan_info reports the one in use. */
#define BCAST_HANDOFF_AUTO 0
#define BCAST_HANDOFF_CACHE 1
#define BCAST_HANDOFF_LDS 2
int bcast_plan_set_rank_handoff(bcast_plan_t *plan, int mode);
/* How the chain issues the stores that stay inside a stage (those the storing
 * wavefront, or its workgroup, reads back itself, and the last position's;
 * what another stage reads is always written through).  BCAST_STORE_THROUGH:
 * written through to memory; BCAST_STORE_BACK: ordinary write-back stores,
 * which the cache acknowledges sooner and the end of the kernel writes back.
 * BCAST_STORE_AUTO (default): the tuning table's choice, else write-back up to
 * 2 MiB and write-through above.  Same bytes either way. */
#define BCAST_STORE_AUTO 0
#define BCAST_STORE_THROUGH 1
#define BCAST_STORE_BACK 2
int bcast_plan_set_stage_store(bcast_plan_t *plan, int mode);
int bcast_plan_set_stages(bcast_plan_t *plan, int stages);
/* Bytes a chain wavefront moves per trip (16-byte accesses): a multiple of
 * 1024 the run's kernel is built for (2048, 3072, 4096 or 6144 with a wavefront
 * per stage; 1024, 2048, 3072, 4096, 6144 or 8192 with a wavefront per rank),
 * 0 = the tuning table's choice, else 4096 (8192 with a wavefront per rank). */
int bcast_plan_set_trip(bcast_plan_t *plan, int trip_bytes);
/* Threads per workgroup of the chain kernel: 64, 128 or 256 (1, 2 or 4
 * wavefronts; they never synchronise, the workgroup is only the unit placed on
 * a compute unit), 0 = default. */
int bcast_plan_set_block_threads(bcast_plan_t *plan, int block_threads);
/* Radix k of BCAST_ALGO_KNOMIAL, 2..nranks (0 = the tuning table's, else 4):
 * in round j every position q < k^j sends to q + i k^j, i = 1..k-1. */
int bcast_plan_set_radix(bcast_plan_t *plan, int radix);
/* Launch-shape requests for the chain kernel; 0 = automatic in every field. */
typedef struct {
    int lanes;         /* wavefronts per stage */
    int stages;        /* groups of consecutive chain positions served by one set of wavefronts */
    int trip_bytes;    /* 2048, 3072, 4096 or 6144 */
    int block_threads; /* 64, 128 or 256 */
} bcast_chain_request_t;

/*
 * Chain geometry as a pure HOST function (no GPU needed): how a chain of
 * `nranks` ranks moving `bytes` bytes in chunks of `chunk_bytes` is laid over
 * at most `max_waves` co-resident wavefronts.  `request` (nullable = all
 * automatic) carries what the plan setters would.  Fills nchunks, stages, hops_per_stage, lanes, slice_bytes, grid_blocks, block_threads, chunk_bytes.
 */
int bcast_chain_geometry(int nranks, size_t bytes, size_t chunk_bytes, int max_waves,
                         const bcast_chain_request_t *request, bcast_plan_info_t *info);

/*
 * Placement of buffers in the device's memory.  Measured on MI355X, the memory
 * answers as three regions, each a third of the physical address range: writes
 * spread over two regions run 1.2 times faster than writes into one, and reads
 * mixed with writes to the same region cost far more than their bytes.  The
 * broadcast's receiving buffers are therefore best spread over two regions, a
 * reduction's contributions kept in one region and its result in another.
 * Every call here takes plain device pointers allocated by anyone; these calls
 * are for callers who want the library to allocate them well placed.
 *
 * bcast_memory_regions -- how many regions the current device's memory has
 * (3) and the size of each (a third of the device's memory).
 *
 * bcast_buffers_alloc -- allocate n device buffers, buffer i of bytes[i] > 0
 * bytes with region label region[i] (0, 1 or 2): buffers with the same label
 * are packed together (in slabs of a power-of-two size, 16 GiB at most, each
 * from one region of the device's memory), buffers with different labels are
 * placed in different regions.  Labels only tell groups apart; which physical
 * region a label gets is the library's business.
 * bytes, region: HOST arrays of n; ptrs: HOST array of n, receives the DEVICE
 * pointers (2 MiB aligned).  They point INTO the slabs: give them back with
 * bcast_buffers_free, never with hipFree; a slab is freed when the last of its
 * buffers is.  The contents are undefined (the library has written to them).
 * Memory: a group occupies the next power of two of its size (2 GiB at least).
 * *placed (HOST, nullable) receives
 *   BCAST_PLACED_NO        the buffers are allocated, but a slab could not be
 *                          got apart from those of other labels (ten allocations
 *                          tried, or memory ran out): it was taken where it fell;
 *   BCAST_PLACED_BY_ORDER  nothing to tell apart (one label only);
 *   BCAST_PLACED_MEASURED  every slab was measured to lie apart from the slabs
 *                          of other labels: writing to both at once ran at the
 *                          rate of a write set spread over regions.
 * How: the order in which the driver hands memory out depends on all that was
 * allocated and freed before, so nothing is assumed about addresses.  A
 * candidate slab is written together with the slabs already placed under other
 * labels (a few ms each); one that lies in the same region as any of them is
 * kept aside, so that the next candidate is other memory, and freed at the end.
 * The call therefore waits for the device and temporarily allocates up to a
 * few times 16 GiB more.  On failure nothing stays allocated.
 * Errors: ERR_ARG, ERR_NOMEM, ERR_HIP.
 * bcast_buffers_free -- give back buffers from bcast_buffers_alloc (any subset,
 * any order; NULL entries are skipped).  ERR_ARG for a pointer that is not one
 * of them (the others are still freed).
 */
#define BCAST_PLACED_NO 0
#define BCAST_PLACED_BY_ORDER 1
#define BCAST_PLACED_MEASURED 2
int bcast_memory_regions(int *count, size_t *region_bytes);
int bcast_buffers_alloc(int n, const size_t *bytes, const int *region, void **ptrs, int *placed);
int bcast_buffers_free(int n, void *const *ptrs);

/*
 * bcast_reduce_sum_f32 -- enqueue one rooted reduction (MPI_Reduce with MPI_SUM
 * on MPI_FLOAT) as a pipelined chain: the collective the paper names as the
 * next one to receive its chain design (Sec. VII), built here as the chain of
 * Sec. IV-B run backwards.  With x_k the contribution of chain position
 * k = (rank - root) mod P,
 *     recv[i] = x_0[i] + (x_1[i] + ( ... + (x_{P-2}[i] + x_{P-1}[i]))),
 * every addition rounded to fp32 (round to nearest even, denormals kept): the
 * result is defined bit for bit.
 *   plan       from bcast_plan_create (its algo is not used; chunk_bytes is the
 *              chunk size, 0 = the reduction table's entry, else a built-in rule;
 *              bcast_plan_set_stages / _lanes apply).
 *   send_bufs  HOST array of plan.nranks DEVICE pointers to `count` floats each,
 *              16-byte aligned, pairwise non-overlapping; only read.
 *   recv_buf   DEVICE pointer to `count` floats, 16-byte aligned: either
 *              send_bufs[root] itself (in place) or memory that overlaps no
 *              contribution.  Only these count floats are written.
 *   count      elements, count * 4 <= plan bytes.
 * The running sums that cross a stage boundary go through staging memory the
 * plan owns: one region of round_up(count * 4, 256) bytes per boundary, reserved
 * beforehand with bcast_plan_reserve_reduce.  This call itself never allocates
 * and never waits for the device.  A stage count set with bcast_plan_set_stages
 * that the reserved memory cannot carry fails with BCAST_ERR_CAPACITY; the
 * library's own choice of stages shrinks to what fits (one stage needs none, so
 * a plan without any reservation reduces in one stage).  Flags, epoch, wait
 * limit and status word are the plan's, as for bcast_run.
 * Errors: ERR_ARG (NULL, misaligned or overlapping pointers, root or count out
 * of range), ERR_CAPACITY, ERR_HIP; ERR_TIMEOUT through the status word.
 */
int bcast_reduce_sum_f32(bcast_plan_t *plan, const void *const *send_bufs, void *recv_buf, int root, size_t count,
                         bcast_stream_t stream);
/* bcast_plan_reserve_reduce -- make sure the plan owns staging memory for
 * reductions of up to `count` floats in up to `stages` stages (cut down to
 * nranks - 1; 0 = what the library would choose for `count` floats: the
 * reduction table's entry, else two).  Grows only; growing waits for the device, frees the
 * old memory and allocates (stages - 1) * round_up(count * 4, 256) bytes.
 * Errors: ERR_ARG (count * 4 beyond the plan's bytes), ERR_NOMEM, ERR_HIP. */
int bcast_plan_reserve_reduce(bcast_plan_t *plan, size_t count, int stages);
/*
 * bcast_reduce_sum_f32_static -- bcast_reduce_sum_f32 for callers that cannot
 * allocate device memory at all: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result
 * bits, same argument checks.  It allocates nothing and needs no reservation:
 * ready flags and staging memory come out of one array in the library's own
 * data segment (about 33 MiB per GPU the library runs on, held until the
 * process ends), whose address on the plan's device was looked up when the plan
 * was created.  Limits: (stages - 1) * round_up(count * 4, 256) <= 32 MiB of
 * staging (so 8 Mi floats in two stages, any size in one stage) and at most
 * 8192 wavefronts; a stage count set with bcast_plan_set_stages beyond that
 * fails with BCAST_ERR_CAPACITY and enqueues nothing, the library's own choice
 * shrinks to what fits.  The plan's device must be the current device.
 * Every call on a GPU shares that GPU's array: calls that overlap in time on
 * one GPU (two streams, two threads, two plans) race and give undefined
 * results; calls that follow one another in stream order are fine -- runs are
 * told apart by a run count in the flag words, nothing needs to be cleared
 * between them.  That count lives in the array itself and is advanced by a
 * one-workgroup kernel enqueued ahead of every run that uses flags (once in
 * 2^32 - 2 runs it clears the flags first), so a call recorded during stream
 * capture replays correctly.  Timeouts surface through the plan's status word
 * as usual.
 */
int bcast_reduce_sum_f32_static(bcast_plan_t *plan, const void *const *send_bufs, void *recv_buf, int root, size_t count,
                                bcast_stream_t stream);
/* MPI_Allreduce (sum of fp32) as the two chains one after the other on `stream`:
 * bcast_reduce_sum_f32 into recv_bufs[root], then bcast_run of that result to
 * every recv_bufs[r] with the plan's broadcast algorithm (an AUTO plan needs a
 * tuning table).  recv_bufs: HOST array of nranks DEVICE pointers, 16-byte
 * aligned; recv_bufs[r] may be send_bufs[r] (in place) and must otherwise
 * overlap nothing.  Every rank ends with the same bits, those
 * bcast_reduce_sum_f32 defines.  Errors as for the two calls. */
int bcast_allreduce_sum_f32(bcast_plan_t *plan, const void *const *send_bufs, void *const *recv_bufs, int root, size_t count,
                            bcast_stream_t stream);
/* The launch shape bcast_reduce_sum_f32 would use for `count` elements (fields as
 * for the chain; algorithmic_bytes = (nranks + 1) * count * 4: every input read
 * once, the result written once). */
int bcast_reduce_info(bcast_plan_t *plan, size_t count, bcast_plan_info_t *info);

/* Pure host arithmetic: the chain positions that `stage` (0-based, of `stages`)
 * plays for chunk number `chunk`: hops *first_hop .. *last_hop, hop h being the
 * copy from position h-1 to position h.  With nranks-1 = q stages + r, every
 * stage plays q hops and r of them one more; stage j has the extra hop for
 * chunk c iff (j + c) mod stages < r, so the longer stages rotate and over any
 * `stages` consecutive chunks all stages play the same number of hops.  This is
 * the function the kernel itself evaluates when spans rotate (plan info's
 * rotating_spans); when they do not, every chunk has the spans of chunk 0.
 * BCAST_ERR_ARG unless 2 <= nranks <= BCAST_MAX_RANKS, 1 <= stages <= nranks-1, 0 <= stage < stages. */
int bcast_chain_stage_span(int nranks, int stages, int stage, uint64_t chunk, int *first_hop, int *last_hop);

/*
 * Tuning table (Sec. III-B "Discussion" and IV-B last paragraph: algorithm and
 * chunk size are chosen per message-size range and process count from
 * measurements).  Process-wide; entries are keyed by (nranks, floor(log2 bytes)).
 *
 * bcast_tune measures, on the current device and `stream`, every candidate
 * (chain over chunk sizes 8 KiB..64 MiB, stage counts and trip sizes, with a
 * wavefront per stage and with a wavefront per rank, direct, binomial, and
 * -- only if `algo_mask` has their bits -- the fan-out, scatter + allgather,
 * the k-nomial tree at radix 4 and 8 and the one-launch pipelined k-nomial
 * tree at radix 2, 4, 8, 16 and nranks (the flat tree)) for message sizes that are
 * powers of two in [min_bytes, max_bytes], keeps the fastest per size, installs
 * the entries, and, if table_path (HOST, nullable) is given, appends them there
 * as text.  It allocates nranks scratch buffers of max_bytes itself.
 * algo_mask: bit (1 << algo) enables a candidate; 0 = chain|direct|binomial.
 */
int bcast_tune(int nranks, size_t min_bytes, size_t max_bytes, unsigned algo_mask,
               bcast_stream_t stream, const char *table_path);
/* algo_mask flag: also try the chain with a single stage (one wavefront plays
 * every rank of its share in turn; no flag hand-off is left). */
#define BCAST_TUNE_FOLDED (1u << 16)
/* algo_mask flag: leave out the chain with a wavefront per rank. */
#define BCAST_TUNE_NO_RANK_WAVES (1u << 17)

/* One table entry: the fastest candidate for the bucket and, beside it, the
 * chain's own best setting (whoever won), which a CHAIN plan with
 * chunk_bytes == 0 uses.  stages: 0 = automatic. */
typedef struct {
    int algo;                   /* winner: bcast_algo_t */
    uint64_t chunk_bytes;       /* winner's chunk size (chain and pipelined k-nomial tree) */
    int stages;                 /* winner's stage count (chain) or radix (k-nomial trees) */
    int trip_bytes;             /* winner's trip size (chain only; 0 = default) */
    double usec;                /* winner's measured time */
    uint64_t chain_chunk_bytes; /* chain: best chunk size (0 = not measured) */
    int chain_stages;           /* chain: best stage count */
    int chain_trip_bytes;       /* chain: best trip size (0 = default) */
    double chain_usec;          /* chain: time at that setting */
    int rank_waves;             /* winner is the chain with a wavefront per rank (1) or per stage (0) */
    int chain_rank_waves;       /* the same for the chain's own best setting */
    int stage_store;            /* winner (chain only): BCAST_STORE_THROUGH / _BACK, 0 = the library's rule */
    int chain_stage_store;      /* the same for the chain's own best setting */
    int lanes;                  /* winner (chain only): wavefronts (with a wavefront per rank: workgroups) per stage,
                                   0 = one per trip of a chunk, up to what the kernel's rule allows (so chunk_bytes /
                                   lanes / trip_bytes trips per lane and chunk) */
    int chain_lanes;            /* the same for the chain's own best setting */
    int spans;                  /* winner (chain with a wavefront per stage only), where nranks-1 is no multiple of
                                   stages: BCAST_SPANS_FIXED (the first stages keep the extra hop) or BCAST_SPANS_ROTATE
                                   (it is passed round from chunk to chunk, see bcast_chain_stage_span); 0 = the library's rule */
    int chain_spans;            /* the same for the chain's own best setting */
} bcast_tune_entry_t;
#define BCAST_SPANS_AUTO 0
#define BCAST_SPANS_FIXED 1
#define BCAST_SPANS_ROTATE 2

/* While a log path (HOST, NULL = off) is set, bcast_tune appends one line per
 * candidate it times: "nranks bytes algo chunk_bytes stages usec trip_bytes rank_waves stage_store lanes spans"
 * (stages holds the radix for the k-nomial trees) -- the raw
 * material for fitting the cost models of Sec. III-A / IV-B. */
int bcast_tune_set_log(const char *log_path);
int bcast_tune_load(const char *table_path);  /* HOST path; adds the file's entries */
int bcast_tune_save(const char *table_path);  /* HOST path; writes all entries */
int bcast_tune_clear(void);
int bcast_tune_put(int nranks, size_t bytes, const bcast_tune_entry_t *entry);
/* Nearest entry for nranks at or below log2(bytes), else the nearest above.  If
 * the table has no entry for nranks at all, the rank count in the table that is
 * closest to it in ratio stands in (the larger on a tie); stage counts and
 * radices beyond what nranks allows are cut down when a plan uses them.
 * BCAST_ERR_UNTUNED if the table is empty. */
int bcast_tune_get(int nranks, size_t bytes, bcast_tune_entry_t *entry);
/* Shorthands: set / look up the winner only. */
int bcast_tune_set(int nranks, size_t bytes, int algo, size_t chunk_bytes, double usec);
int bcast_tune_lookup(int nranks, size_t bytes, int *algo, size_t *chunk_bytes, double *usec);
int bcast_tune_count(void);

/*
 * The reduction's own tuning table (Sec. III-B applied to the collective
 * Sec. VII names next): per (nranks, floor(log2 bytes)) the stage count, chunk
 * size and trip size bcast_reduce_sum_f32 uses when the plan leaves them open
 * (chunk_bytes == 0 and no bcast_plan_set_stages).  Process-wide, saved to and
 * loaded from the same text file as the broadcast's entries (lines
 * "reduce nranks log2_bytes chunk_bytes stages trip_bytes usec").
 * trip_bytes: 4096 (contributions loaded 4 positions at a time) or 1024 (16 at
 * a time, for small messages).
 */
typedef struct {
    uint64_t chunk_bytes; /* multiple of 16 */
    int stages;           /* 1..nranks-1; 1 = no hand-off at all, no staging memory */
    int trip_bytes;       /* 4096 or 1024 */
    double usec;          /* measured time at that setting */
} bcast_reduce_entry_t;
/* bcast_tune_reduce -- measure, on the current device and `stream`, the chain
 * reduction of `nranks` contributions over stage counts 1, 2 and 4, both trip
 * sizes and chunk sizes lanes * trip for power-of-two lane counts (and the whole
 * message as one chunk), for message sizes that are powers of two in
 * [min_bytes, max_bytes]; keeps the fastest per size, installs the entries and,
 * if table_path (HOST, nullable) is given, appends them there.  Allocates
 * nranks + 1 buffers of max_bytes and the staging memory itself. */
int bcast_tune_reduce(int nranks, size_t min_bytes, size_t max_bytes, bcast_stream_t stream, const char *table_path);
int bcast_tune_reduce_put(int nranks, size_t bytes, const bcast_reduce_entry_t *entry);
/* Nearest entry as for bcast_tune_get; BCAST_ERR_UNTUNED if there is none. */
int bcast_tune_reduce_get(int nranks, size_t bytes, bcast_reduce_entry_t *entry);

const char *bcast_strerror(int status);
int bcast_last_hip_error(void);
const char *bcast_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BCAST_H */

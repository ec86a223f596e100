// gfx950 kernels of the broadcast library.
//
// All kernels move raw bytes between device buffers of one GPU.  The unit of
// work is a wavefront (64 lanes): it copies one contiguous span with 16-byte
// accesses per lane (1 KiB per wave instruction, kUnroll of them in flight),
// and byte accesses for a head/tail that is not 16-byte aligned.  There are no
// workgroup barriers and no LDS: the path is bound by HBM, not by arithmetic.
#include <algorithm>
#include <atomic>
#include <mutex>

#include "bcast_internal.h"

namespace bcast {

template <int V> struct VecOf;
template <> struct VecOf<16> { typedef unsigned int type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<8> { typedef unsigned int type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<4> { typedef unsigned int type; };
template <> struct VecOf<1> { typedef unsigned char type; };

// Copy bytes [lo, hi) of src to the same offsets of dst with one wavefront.
// Requires (src + lo) and (dst + lo) congruent modulo V.
template <int V>
__device__ __forceinline__ void copy_span(char *__restrict__ dst, const char *__restrict__ src,
                                          u64 lo, u64 hi, unsigned lane)
{
    typedef typename VecOf<V>::type T;
    const char *s = src + lo;
    char *d = dst + lo;
    u64 n = hi - lo;

    u64 head = (V - ((uintptr_t)s & (V - 1))) & (V - 1);  // bytes up to the next V-aligned address
    if (head > n) head = n;
    if (lane < head) d[lane] = s[lane];
    s += head;
    d += head;
    n -= head;

    const u64 nvec = n / V;
    const T *__restrict__ sv = reinterpret_cast<const T *>(s);
    T *__restrict__ dv = reinterpret_cast<T *>(d);
    u64 i = lane;
    for (; i + (kUnroll - 1) * kWaveSize < nvec; i += kUnroll * kWaveSize) {
        T r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) r[u] = sv[i + u * kWaveSize];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) dv[i + u * kWaveSize] = r[u];
    }
    for (; i < nvec; i += kWaveSize) dv[i] = sv[i];

    const u64 done = nvec * V;
    const u64 tail = n - done;  // < V
    if (lane < tail) d[done + lane] = s[done + lane];
}

// ---------------------------------------------------------------------------
// Agent-scope coherent accesses for payload that another wavefront, possibly on
// another XCD (each XCD has its own L2), reads or wrote during the same kernel.
// On gfx940-class targets the cache-policy bit sc1 marks an access as
// agent-scope: a load with sc1 is not served from a line that may be stale in
// this CU's L1 or this XCD's L2, and a store with sc1 is written through, so
// that once it has completed (vmcnt reaches 0) any sc1 load on the device sees
// it.  These are the bits the compiler itself emits for relaxed agent-scope
// atomic loads and stores; the buffer intrinsics let 16-byte payload accesses
// carry them too.  With every payload access of the chain kernel marked this
// way there is nothing stale to invalidate and nothing dirty to write back, so
// the hand-off needs no L2 write-back / invalidate (which cost microseconds
// per wave and serialise on the L2).
// ---------------------------------------------------------------------------
constexpr int kRsrcWord3 = 0x00020000;      // raw buffer, 32-bit data format

// LD / ST: cache-policy bits of the loads / stores (kAuxAgent or kAuxCached).
template <int V, int LD, int ST> struct AgentIO;
template <int LD, int ST> struct AgentIO<16, LD, ST> {
    typedef VecOf<16>::type T;
    static __device__ __forceinline__ T ld(__amdgpu_buffer_rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, LD); }
    static __device__ __forceinline__ void st(T v, __amdgpu_buffer_rsrc_t r, unsigned off) { __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, ST); }
};
template <int LD, int ST> struct AgentIO<8, LD, ST> {
    typedef VecOf<8>::type T;
    static __device__ __forceinline__ T ld(__amdgpu_buffer_rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, LD); }
    static __device__ __forceinline__ void st(T v, __amdgpu_buffer_rsrc_t r, unsigned off) { __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, ST); }
};
template <int LD, int ST> struct AgentIO<4, LD, ST> {
    typedef VecOf<4>::type T;
    static __device__ __forceinline__ T ld(__amdgpu_buffer_rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, LD); }
    static __device__ __forceinline__ void st(T v, __amdgpu_buffer_rsrc_t r, unsigned off) { __builtin_amdgcn_raw_buffer_store_b32(v, r, off, 0, ST); }
};
template <int LD, int ST> struct AgentIO<1, LD, ST> {
    typedef VecOf<1>::type T;
    static __device__ __forceinline__ T ld(__amdgpu_buffer_rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b8(r, off, 0, LD); }
    static __device__ __forceinline__ void st(T v, __amdgpu_buffer_rsrc_t r, unsigned off) { __builtin_amdgcn_raw_buffer_store_b8(v, r, off, 0, ST); }
};

// copy_span with agent-scope accesses for a span of at most a few trips (the
// chain kernel passes one trip at a time; offsets inside a buffer descriptor
// are 32-bit).  The vector body runs a wave-uniform loop of U loads then U
// stores per lane with no remainder loop: the body's descriptors
// end exactly at the last whole vector, so a lane whose offset lies beyond it
// is range-checked by the hardware (the load returns zero, the store is
// dropped).  A short span therefore costs one memory round trip, not one per
// kilobyte.
template <int V, int U, int LD = kAuxAgent, int ST = kAuxAgent>
__device__ __forceinline__ void copy_span_agent(char *dst, const char *src, u64 lo, u64 hi, unsigned lane)
{
    typedef AgentIO<V, LD, ST> IO;
    typedef AgentIO<1, LD, ST> IO1;
    typedef typename IO::T T;
    const unsigned n = (unsigned)(hi - lo);
    unsigned head = (V - (unsigned)((uintptr_t)(src + lo) & (V - 1))) & (V - 1);
    if (head > n) head = n;
    const unsigned nvec = (n - head) / V;
    const unsigned body_end = head + nvec * V;

    if (head != 0 || body_end != n) {  // ragged ends: at most V-1 bytes each
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(src + lo), 0, n, kRsrcWord3);
        const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(dst + lo, 0, n, kRsrcWord3);
        if (lane < head) IO1::st(IO1::ld(rs, lane), rd, lane);
        if (lane < n - body_end) IO1::st(IO1::ld(rs, body_end + lane), rd, body_end + lane);
    }
    if (nvec == 0) return;

    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(src + lo), 0, body_end, kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(dst + lo, 0, body_end, kRsrcWord3);
    const unsigned trip = U * kWaveSize * V;  // bytes per wave per trip
    unsigned off = head + lane * V;
    for (unsigned base = head; base < body_end; base += trip, off += trip) {
        T r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = IO::ld(rs, off + u * kWaveSize * V);
#pragma unroll
        for (int u = 0; u < U; ++u) IO::st(r[u], rd, off + u * kWaveSize * V);
    }
}

// copy_span_agent with the cache policies as run-time (wave-uniform) values: the
// host picks them per run.  ld and st are each one of kAuxCached, kAuxStream,
// kAuxAgent, kAuxAgent | kAuxStream.
template <int V, int U>
__device__ __forceinline__ void copy_span_policy(char *dst, const char *src, u64 lo, u64 hi, unsigned lane, unsigned ld, unsigned st)
{
#define BCAST_POLICY_CASE(LD, ST) \
    case ((LD) | ((ST) << 8)): copy_span_agent<V, U, (LD), (ST)>(dst, src, lo, hi, lane); break;
    switch (ld | (st << 8)) {
        BCAST_POLICY_CASE(kAuxCached, kAuxCached)
        BCAST_POLICY_CASE(kAuxCached, kAuxStream)
        BCAST_POLICY_CASE(kAuxCached, kAuxAgent)
        BCAST_POLICY_CASE(kAuxCached, kAuxAgent | kAuxStream)
        BCAST_POLICY_CASE(kAuxStream, kAuxCached)
        BCAST_POLICY_CASE(kAuxStream, kAuxStream)
        BCAST_POLICY_CASE(kAuxStream, kAuxAgent)
        BCAST_POLICY_CASE(kAuxStream, kAuxAgent | kAuxStream)
        BCAST_POLICY_CASE(kAuxAgent, kAuxCached)
        BCAST_POLICY_CASE(kAuxAgent, kAuxStream)
        BCAST_POLICY_CASE(kAuxAgent, kAuxAgent)
        BCAST_POLICY_CASE(kAuxAgent, kAuxAgent | kAuxStream)
        BCAST_POLICY_CASE(kAuxAgent | kAuxStream, kAuxCached)
        BCAST_POLICY_CASE(kAuxAgent | kAuxStream, kAuxStream)
        BCAST_POLICY_CASE(kAuxAgent | kAuxStream, kAuxAgent)
        BCAST_POLICY_CASE(kAuxAgent | kAuxStream, kAuxAgent | kAuxStream)
    default: break;  // the host admits no other value
    }
#undef BCAST_POLICY_CASE
}

// Same span, one source, many destinations: each vector is read once and
// stored to every dst (the one-die fan-out).
template <int V>
__device__ __forceinline__ void fanout_span(const CopyArgs &a, u64 lo, u64 hi, unsigned lane)
{
    typedef typename VecOf<V>::type T;
    const char *s = a.buf[0] + lo;
    u64 n = hi - lo;
    const unsigned P = a.nranks;

    u64 head = (V - ((uintptr_t)s & (V - 1))) & (V - 1);
    if (head > n) head = n;
    if (lane < head) {
        const char b = s[lane];
        for (unsigned k = 1; k < P; ++k) a.buf[k][lo + lane] = b;
    }
    const u64 body = lo + head;
    n -= head;
    const u64 nvec = n / V;
    const T *__restrict__ sv = reinterpret_cast<const T *>(a.buf[0] + body);
    u64 i = lane;
    for (; i + (kUnroll - 1) * kWaveSize < nvec; i += kUnroll * kWaveSize) {
        T r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) r[u] = sv[i + u * kWaveSize];
        for (unsigned k = 1; k < P; ++k) {
            T *__restrict__ dv = reinterpret_cast<T *>(a.buf[k] + body);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) dv[i + u * kWaveSize] = r[u];
        }
    }
    for (; i < nvec; i += kWaveSize) {
        const T r = sv[i];
        for (unsigned k = 1; k < P; ++k) reinterpret_cast<T *>(a.buf[k] + body)[i] = r;
    }
    const u64 done = body + nvec * V;
    const u64 tail = n - nvec * V;
    if (lane < tail) {
        const char b = a.buf[0][done + lane];
        for (unsigned k = 1; k < P; ++k) a.buf[k][done + lane] = b;
    }
}

// ---------------------------------------------------------------------------
// Pipelined chain (Sec. IV-B).  The P-1 hops are grouped into stages of
// consecutive hops; wavefront (stage, lane) receives lane's share of every
// chunk into the first position of its stage from the position before it,
// carries it through the stage's positions (each read out of the previous
// position's buffer), and publishes it to the next stage -- the receive /
// store / forward loop of a middle rank, with one wave playing the ranks of
// its stage in turn.  With one hop per stage every rank has waves of its own.
// Position 0 (the root) only sends: nobody writes its buffer.  The last
// position only receives: its stage publishes nothing.
//
// Hand-off protocol.  flag(stage, lane) counts the chunks of this run that the
// stage's last position has stored for `lane`, as base + (count << 4) + xcd
// with base = epoch << 32; flags only grow, so nothing is reset between runs.
// Producer: the wave waits until all of its (write-through, agent-scope)
// payload stores have completed -- one s_waitcnt for the whole wave, so it
// covers every lane's stores -- and then lane 0 stores the flag (agent scope).
// Consumer: lane 0 polls the flag with agent-scope loads; the payload loads are
// issued only after a poll has returned the awaited value, and, being
// agent-scope themselves, cannot be served from a stale cache line.
//
// Forward progress.  Wavefronts are numbered stage-major, so a wave only ever
// waits for a wave with a lower workgroup index; the host also keeps the grid
// within what the device can hold at once.  Every wait is bounded by a clock
// limit: a wave that gives up records (first hop of its stage, chunk), raises
// the abort word so that the others stop waiting too, and returns.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void report_timeout(const ChainArgs &a, u64 base, unsigned hop, unsigned chunk)
{
    const u64 epoch = base >> 32;
    const u64 old = __hip_atomic_fetch_max(a.abort_word, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old < epoch && a.status[0] == 0) {  // first wave of this run to give up
        __hip_atomic_store(&a.status[1], ((u64)hop << 32) | chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(&a.status[0], (u64)1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// One agent-scope read of a flag for the whole wave: only lane 0 issues the
// load (64 lanes reading one address still cost one request per group of
// lanes, and a device full of polling waves then eats a large share of the
// memory system's request rate), the value is broadcast through an SGPR.
__device__ __forceinline__ u64 read_flag(const u64 *flag, unsigned lane)
{
    u64 v = 0;
    if (lane == 0) v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return ((u64)hi << 32) | lo;
}

// The run's flag base, epoch << 32.  The host either passes it as an argument
// (it counts the runs itself) or names a word in device memory that a small
// kernel enqueued ahead of this one has advanced: then the launch can be
// recorded into a graph and replayed, every replay finding a new epoch.
__device__ __forceinline__ u64 run_base(const ChainArgs &a, unsigned lane)
{
    if (a.epoch_word == nullptr) return a.base;
    return read_flag(a.epoch_word, lane) << 32;
}

__device__ __forceinline__ bool wait_ready(const u64 *flag, u64 want, const ChainArgs &a, u64 base, unsigned hop,
                                           unsigned chunk, unsigned lane, u64 *seen)
{
    u64 v = read_flag(flag, lane);
    if (v < want) {
        const u64 t0 = wall_clock64();
        const u64 epoch = base >> 32;
        unsigned spins = 0;
        for (;;) {
            __builtin_amdgcn_s_sleep(2);
            v = read_flag(flag, lane);
            if (v >= want) break;
            if ((++spins & 31u) == 0) {
                if (read_flag(a.abort_word, lane) >= epoch) return false;
                if (wall_clock64() - t0 > a.spin_ticks) {
                    if (lane == 0) report_timeout(a, base, hop, chunk);
                    return false;
                }
            }
        }
    }
    // the branch on v has already waited for the poll to return; keep the
    // compiler from hoisting payload loads above it
    asm volatile("" ::: "memory");
    *seen = v;
    return true;
}

// The chain kernel's sets of cache policies (see chain_kernel).
constexpr int kPolicyThrough = 0;
constexpr int kPolicyBack = 1;
constexpr int kPolicyArgs = 2;

// One trip of whole vectors, U loads then U stores per lane, through two buffer
// descriptors that end with the trip: a lane beyond the end is range-checked by
// the hardware (its load returns zero, its store is dropped).
template <int V, int U, int LD, int ST>
__device__ __forceinline__ void move_trip(__amdgpu_buffer_rsrc_t rs, __amdgpu_buffer_rsrc_t rd, unsigned off)
{
    typedef AgentIO<V, LD, ST> IO;
    typename IO::T r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = IO::ld(rs, off + u * kWaveSize * V);
#pragma unroll
    for (int u = 0; u < U; ++u) IO::st(r[u], rd, off + u * kWaveSize * V);
}

// Wait for every store of the wave to complete.  `next` (the next position's
// descriptor) is named as an input only so that the compiler has it in registers BEFORE the
// wait: what the wave needs for its next hop is then computed while its stores
// drain, and the loads go out the moment the wait returns.
__device__ __forceinline__ void stores_done_then(__amdgpu_buffer_rsrc_t next)
{
    asm volatile("s_waitcnt vmcnt(0)" ::"s"(next) : "memory");
}

// A trip of n bytes at offset lo (whole vectors from a vector-aligned address,
// n <= one trip) carried through positions first_hop .. last_hop of a stage with
// the policies the host chooses by itself.  What the loop over the hops does
// between the completion of a hop's stores and the issue of the next hop's loads
// is time in which the wave has nothing in flight, and the hops of a stage follow
// each other every 0.5-0.8 us: so the hops are told apart outside the loop (first:
// agent-scope load; last: agent-scope store unless the chain ends here), the
// next position's address is fetched ahead of the wait, and the loop body is the
// wait, one descriptor, U loads and U stores.
template <int V, int U, int POLICY>
__device__ __forceinline__ void carry_trip(const ChainArgs &a, u64 lo, unsigned n, unsigned first_hop, unsigned last_hop,
                                           bool chain_ends, unsigned lane)
{
    constexpr int ST_MID = POLICY == kPolicyBack ? kAuxCached : kAuxAgent;
    const unsigned off = lane * V;
    __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(a.buf[first_hop - 1] + lo, 0, n, kRsrcWord3);
    __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(a.buf[first_hop] + lo, 0, n, kRsrcWord3);
    if (first_hop == last_hop) {
        if (chain_ends) move_trip<V, U, kAuxAgent, ST_MID>(rs, rd, off);
        else move_trip<V, U, kAuxAgent, kAuxAgent>(rs, rd, off);
        return;
    }
    move_trip<V, U, kAuxAgent, ST_MID>(rs, rd, off);
    for (unsigned hop = first_hop + 1; hop < last_hop; ++hop) {
        rs = rd;
        rd = __builtin_amdgcn_make_buffer_rsrc(a.buf[hop] + lo, 0, n, kRsrcWord3);
        stores_done_then(rd);
        move_trip<V, U, kAuxCached, ST_MID>(rs, rd, off);
    }
    rs = rd;
    rd = __builtin_amdgcn_make_buffer_rsrc(a.buf[last_hop] + lo, 0, n, kRsrcWord3);
    stores_done_then(rd);
    if (chain_ends) move_trip<V, U, kAuxCached, ST_MID>(rs, rd, off);
    else move_trip<V, U, kAuxCached, kAuxAgent>(rs, rd, off);
}

// Cache policy inside a stage.  A buffer that a wave stores as position h and
// reads back for position h+1 is touched by no other wave during the kernel, and
// a wave always sees its own earlier stores once s_waitcnt has passed, whatever
// cache they sit in.  So the read-back may be an ordinary cached load: the
// write-through store left the line in this CU's 32 KiB vector L1, and while the
// trips of the CU's resident waves fit there (8 waves of 3 KiB, 4-8 of 4 KiB)
// all or most of it is still there -- measured 8-10 TB/s instead of 7.3 TB/s
// when every load goes to memory.  U (3 or 4 KiB trips) is the host's choice,
// and so are four cache policies (ChainArgs::ld_root, ld_edge, ld_back, st_mid):
//   ld_root  loads of the root's buffer (never written during the run: any policy);
//   ld_edge  loads of a buffer another stage's wave stored (always agent scope);
//   ld_back  the read-back of the wave's own stores inside a stage;
//   st_mid   stores a wave reads back itself, and the chain's last position
//            (write-through at agent scope, or ordinary write-back stores whose
//            dirty lines the end of the kernel writes back like for any kernel:
//            the L2 round trip is about half the memory one, which is what a
//            small broadcast over many hops consists of).
// Buffers handed from stage to stage are always stored at agent scope.
// POLICY: the two sets of policies the host chooses by itself are built in
// (kPolicyThrough, kPolicyBack: root and edge loads at agent scope, read-back
// cached, in-stage stores write-through / write-back), any other set is read from
// the arguments at every hop (kPolicyArgs).  The selection sits in the hop loop,
// whose length is what a short broadcast consists of: measured at 8 ranks x 64
// MiB, 114 us with the policies built in against 122 us when read from the
// arguments.
template <int V, int U, int POLICY>
__global__ void __launch_bounds__(kBlockThreads) chain_kernel(const ChainArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    // workgroups of 1, 2 or 4 waves: no wave ever meets another at a barrier,
    // the workgroup is only the unit the dispatcher places on a CU
    const unsigned gw = __builtin_amdgcn_readfirstlane(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (gw >= a.stages * a.lanes) return;
    const u64 base = run_base(a, lane);
    // Stage g serves consecutive chain positions first_hop .. last_hop: its waves
    // play those ranks one after the other (one hop per stage is one stage per
    // rank).  Hand-offs between stages go through flags; inside a stage the
    // same wave stored what it reads next, so its own s_waitcnt orders the two.
    // Where the P-1 hops do not divide evenly over the stages, the stages that
    // take one hop more rotate from chunk to chunk (see stage_begin), so that
    // over the message every stage plays the same number of hops and none
    // idles while a longer one finishes.
    const unsigned g = gw / a.lanes;
    const unsigned s = gw - g * a.lanes;
    const unsigned hops = a.nranks - 1;
    const unsigned hops_min = hops / a.stages;            // every stage plays at least this many
    const unsigned hops_extra = hops - hops_min * a.stages;  // this many stages play one more
    // which XCD (L2 domain) this wave runs on: HW_REG_XCC_ID, bits 3:0
    const unsigned xcd = __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & 15u;

    const u64 *in_flag = g > 0 ? a.flags + ((u64)(g - 1) * a.lanes + s) * kFlagStrideWords : nullptr;
    u64 *const my_flag = g + 1 < a.stages ? a.flags + ((u64)g * a.lanes + s) * kFlagStrideWords : nullptr;
    unsigned near = 0, far = 0;  // hand-offs received from the same / another XCD

    // A lane's share of a chunk is every lanes-th trip (one trip = U vector
    // instructions of the wave, U KiB at 16 bytes per lane), so at any
    // moment the lanes of a stage sweep one contiguous window of the chunk: DRAM
    // sees a few wide streams per stage, not one narrow stream per wave.
    const u64 trip = (u64)U * kWaveSize * V;
    const u64 stride = trip * a.lanes;

    u64 seen = 0;  // newest value read from in_flag
    u64 chunk_lo = 0;
    for (unsigned c = 0; c < a.nchunks; ++c, chunk_lo += a.chunk_bytes) {
        u64 chunk_hi = chunk_lo + a.chunk_bytes;
        if (chunk_hi > a.bytes) chunk_hi = a.bytes;
        // this chunk's positions for this stage: the producer stage computes
        // the same boundary, so it publishes exactly the buffer read here
        const unsigned turn = (a.mode & kModeFixedSpans) ? 0u : c;
        const unsigned first_hop = stage_begin(g, turn, a.stages, hops_min, hops_extra) + 1;
        const unsigned last_hop = stage_begin(g + 1, turn, a.stages, hops_min, hops_extra);
        const bool muted = a.mute_hop >= first_hop && a.mute_hop <= last_hop;
        u64 *const out_flag = muted ? nullptr : my_flag;

        // flag value: base + (chunks stored << 4) + producer's XCD
        if (in_flag) {
            const u64 want = base + ((u64)(c + 1) << 4);
            if (seen < want && !wait_ready(in_flag, want, a, base, first_hop, c, lane, &seen)) return;
            // whichever read of the flag showed the chunk (this wait, or the look-ahead after the chunk
            // before): no payload load of this chunk may be moved above it
            asm volatile("" ::: "memory");
            const bool same_xcd = (unsigned)(seen & 15u) == xcd;
            near += same_xcd;
            far += !same_xcd;
        }
        const bool traced = (a.mode & kModeTrace) && s == 0 && (u64)g * a.nchunks + c < a.trace_entries;
        if (traced && lane == 0) a.trace[((u64)g * a.nchunks + c) * 2] = wall_clock64();
        // One trip at a time is carried through all positions of the stage
        // before the next trip starts: what the wave reads back for position
        // h+1 it stored for position h one memory round trip earlier, so with
        // few enough waves per CU it is still in that CU's vector L1.
        for (u64 lo = chunk_lo + (u64)s * trip; lo < chunk_hi; lo += stride) {
            const u64 hi = lo + trip < chunk_hi ? lo + trip : chunk_hi;
            if constexpr (POLICY != kPolicyArgs) {
                // whole vectors from an aligned address (all buffers are congruent modulo V): the short way
                if ((((uintptr_t)(a.buf[0] + lo) | (uintptr_t)(hi - lo)) & (V - 1)) == 0) {
                    carry_trip<V, U, POLICY>(a, lo, (unsigned)(hi - lo), first_hop, last_hop, g + 1 == a.stages, lane);
                    continue;
                }
            }
            for (unsigned hop = first_hop; hop <= last_hop; ++hop) {
                const char *src = a.buf[hop - 1];
                char *dst = a.buf[hop];
                // What this wave stored for position hop-1 must have completed
                // before it is read back for position hop.  (Same-address order
                // alone would make the read-back correct without this wait, but
                // measured it is 10-25 % slower with 3 KiB trips: loads issued
                // behind stores still in flight miss the L1.)
                if (hop != first_hop) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                if constexpr (POLICY == kPolicyArgs) {
                    const unsigned ld = hop != first_hop ? a.ld_back : (g == 0 ? a.ld_root : a.ld_edge);
                    const unsigned st = (hop != last_hop || g + 1 == a.stages) ? a.st_mid : (unsigned)kAuxAgent;
                    copy_span_policy<V, U>(dst, src, lo, hi, lane, ld, st);
                } else {
                    const bool ld_cached = hop != first_hop;
                    const bool st_cached = POLICY == kPolicyBack && (hop != last_hop || g + 1 == a.stages);
                    if (ld_cached && st_cached) copy_span_agent<V, U, kAuxCached, kAuxCached>(dst, src, lo, hi, lane);
                    else if (ld_cached) copy_span_agent<V, U, kAuxCached, kAuxAgent>(dst, src, lo, hi, lane);
                    else if (st_cached) copy_span_agent<V, U, kAuxAgent, kAuxCached>(dst, src, lo, hi, lane);
                    else copy_span_agent<V, U>(dst, src, lo, hi, lane);
                }
            }
        }
        // Look at the next chunk's flag while this chunk's stores drain: in
        // steady state the left neighbour is ahead and the next wait is free.
        if (in_flag && c + 1 < a.nchunks) seen = read_flag(in_flag, lane);
        if (out_flag || traced) {
            // every payload store of this wave has completed (and, being
            // write-through, is visible device-wide) before the flag is raised
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (traced && lane == 0) a.trace[((u64)g * a.nchunks + c) * 2 + 1] = wall_clock64();
        }
        if (out_flag) {
            if (lane == 0)
                __hip_atomic_store(out_flag, base + ((u64)(c + 1) << 4) + xcd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if ((a.mode & kModeCount) && lane == 0) {
        __hip_atomic_fetch_add(&a.counters[0], (u64)near, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&a.counters[1], (u64)far, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------------------
// The pipelined chain with one wavefront per rank (Sec. IV-B read literally:
// every non-root process receives a chunk from its left neighbour, stores it and
// forwards it to its right neighbour).  Stage g, lane s is a WORKGROUP; its
// wave j plays chain position first_hop(g) + j and nothing else.  The waves of
// a workgroup run on one compute unit and share its vector L1 and its LDS, so a
// hand-off between two ranks of the same workgroup stays on the CU:
//   producer (rank h):   stores of a trip complete (s_waitcnt vmcnt(0)), then a
//                        workgroup-scope release store of its trip count to LDS;
//   consumer (rank h+1): workgroup-scope acquire load of that count from LDS,
//                        then ordinary loads of the trip out of rank h's buffer,
//                        which the CU's L1 (written through by the producer a
//                        moment ago) or its XCD's L2 serves.
// At workgroup scope (and without threadgroup-split mode) the CU's L1 is the
// point of coherence for the workgroup's waves, so this is the plain
// release/acquire protocol with nothing to write back or invalidate.
// With kModeLdsHandoff the payload takes the other on-chip way, LDS as the link
// between two ranks: every wave has two trip slots there;
//   producer (rank h):   stores the trip into its buffer in memory AND into its
//                        slot (trip t into slot t mod 2), then the same release
//                        store of its trip count, which by itself waits for the
//                        LDS writes only;
//   consumer (rank h+1): the same acquire load, then the trip out of rank h's
//                        slot.
// A slot is written again once the right neighbour has read the trip before the
// last one out of it (the back-pressure count below, kRankLead = 2 = the number
// of slots).  The L1 then has nothing to keep, and the buffers in memory are
// written once and read only across workgroups.  (Nothing in the protocol needs
// a rank's stores to memory to complete before the hand-off; as compiled, the
// wave still has them complete before its last LDS write of the trip -- the
// compiler keeps one count for all vector memory operations of a wave and waits
// where the ways through this loop meet.  A build in which the stores drain
// behind the hand-offs ran no faster: 8 ranks x 64 MiB the same, 16 ranks x 528
// MB 3 % slower; the stores' completions pace the waves.)  Trips with a ragged
// end or a misaligned start go through the cache as above, decided per trip by
// producer and consumer alike.
// The pipelining unit inside a workgroup is the trip (U KiB); between workgroups
// (stage g's last rank to stage g+1's first) it is the chunk, handed over
// through the flags in memory exactly as in chain_kernel.  Every rank stores
// what its left neighbour stored, every hop is a flag hand-off, and
// every rank has wavefronts of its own: lanes workgroups per stage, each
// sweeping its share (every lanes-th trip) of every chunk.
// Forward progress: a wave waits either for the wave before it in its own
// workgroup (resident with it) or for a workgroup with a lower index; waits are
// bounded by the clock limit like everywhere else.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool wait_trip(const unsigned *count, unsigned want, const ChainArgs &a, u64 base, unsigned hop,
                                          unsigned chunk, unsigned lane)
{
    unsigned v = __builtin_amdgcn_readfirstlane(__hip_atomic_load(count, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
    if (v < want) {
        const u64 t0 = wall_clock64();
        const u64 epoch = base >> 32;
        unsigned spins = 0;
        for (;;) {
            __builtin_amdgcn_s_sleep(1);
            v = __builtin_amdgcn_readfirstlane(__hip_atomic_load(count, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
            if (v >= want) break;
            if ((++spins & 63u) == 0) {
                if (read_flag(a.abort_word, lane) >= epoch) return false;
                if (wall_clock64() - t0 > a.spin_ticks) {
                    if (lane == 0) report_timeout(a, base, hop, chunk);
                    return false;
                }
            }
        }
    }
    asm volatile("" ::: "memory");  // payload loads stay behind the acquire
    return true;
}

template <int V, int U>
__global__ void __launch_bounds__(kRankBlockThreadsMax) rank_chain_kernel(const ChainArgs a)
{
    __shared__ unsigned trips_done[kRankWavesMax];  // per wave of this workgroup: trips stored so far
    __shared__ unsigned trips_read[kRankWavesMax];  // per wave: trips whose loads have returned
    extern __shared__ __align__(16) unsigned char trip_slots[];  // kModeLdsHandoff: [wave][2] trips
    typedef typename AgentIO<V, 0, 0>::T T;
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const unsigned j = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned g = blockIdx.x / a.lanes;
    const unsigned s = blockIdx.x - g * a.lanes;
    if (threadIdx.x < kRankWavesMax) trips_done[threadIdx.x] = trips_read[threadIdx.x] = 0;
    __syncthreads();  // the only barrier: every wave of the workgroup is still here
    if (g >= a.stages) return;
    const unsigned hops = a.nranks - 1;
    const unsigned hops_min = hops / a.stages, hops_extra = hops - hops_min * a.stages;
    const unsigned first_hop = stage_begin(g, 0, a.stages, hops_min, hops_extra) + 1;
    const unsigned last_hop = stage_begin(g + 1, 0, a.stages, hops_min, hops_extra);
    const unsigned hop = first_hop + j;  // the one chain position this wave plays
    if (hop > last_hop) return;
    const u64 base = run_base(a, lane);
    const bool first = j == 0, last = hop == last_hop;
    const bool muted = a.mute_hop == hop;
    const u64 *in_flag = (first && g > 0) ? a.flags + ((u64)(g - 1) * a.lanes + s) * kFlagStrideWords : nullptr;
    u64 *const out_flag = (last && g + 1 < a.stages && !muted) ? a.flags + ((u64)g * a.lanes + s) * kFlagStrideWords : nullptr;
    const char *src = a.buf[hop - 1];
    char *dst = a.buf[hop];
    const unsigned ld = first ? (g == 0 ? a.ld_root : a.ld_edge) : a.ld_back;
    const unsigned st = (last && g + 1 < a.stages) ? (unsigned)kAuxAgent : a.st_mid;
    const bool plain_policies = (ld == kAuxAgent || ld == kAuxCached) && (st == kAuxAgent || st == kAuxCached);

    const u64 trip = (u64)U * kWaveSize * V;
    const u64 stride = trip * a.lanes;
    unsigned seq = 0;  // trips this wave has stored
    u64 seen = 0;
    u64 chunk_lo = 0;
    for (unsigned c = 0; c < a.nchunks; ++c, chunk_lo += a.chunk_bytes) {
        u64 chunk_hi = chunk_lo + a.chunk_bytes;
        if (chunk_hi > a.bytes) chunk_hi = a.bytes;
        if (in_flag) {
            const u64 want = base + ((u64)(c + 1) << 4);
            if (seen < want && !wait_ready(in_flag, want, a, base, hop, c, lane, &seen)) return;
            asm volatile("" ::: "memory");  // also behind the look-ahead read of the flag
        }
        for (u64 lo = chunk_lo + (u64)s * trip; lo < chunk_hi; lo += stride) {
            const u64 hi = lo + trip < chunk_hi ? lo + trip : chunk_hi;
            // whole vectors from an aligned address, policies without the streaming bit: the trip's two
            // descriptors are made before the waits, and the loads go out the moment the last wait returns
            const bool lean = plain_policies && (((uintptr_t)(src + lo) | (uintptr_t)(hi - lo)) & (V - 1)) == 0;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(src) + lo, 0, (unsigned)(hi - lo), kRsrcWord3);
            const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(dst + lo, 0, (unsigned)(hi - lo), kRsrcWord3);
            asm volatile("" ::"s"(rs), "s"(rd));
            if (!first && !wait_trip(&trips_done[j - 1], seq + 1, a, base, hop, c, lane)) return;
            // Back-pressure: a rank stays at most kRankLead trips ahead of its
            // right neighbour's reading, so that what it stores is read out of
            // the CU's cache before later trips push it out.
            if (!last && seq >= kRankLead && !wait_trip(&trips_read[j + 1], seq + 1 - kRankLead, a, base, hop + 1, c, lane)) return;
            static_assert(kRankLead == 2, "a wave has two trip slots: its right neighbour may be that many trips behind");
            const bool via_lds = lean && (a.mode & kModeLdsHandoff);
            if (via_lds) {
                // the trip comes out of the left neighbour's slot (the first rank of the workgroup: out of
                // memory), goes into this rank's buffer and, for the right neighbour, into this rank's slot
                const unsigned off = lane * V;
                T r[U];
                if (first) {
#pragma unroll
                    for (int u = 0; u < U; ++u) r[u] = AgentIO<V, kAuxAgent, 0>::ld(rs, off + u * kWaveSize * V);
                } else {
                    const T *in = reinterpret_cast<const T *>(trip_slots) + ((j - 1) * 2 + (seq & 1)) * (U * kWaveSize);
#pragma unroll
                    for (int u = 0; u < U; ++u) r[u] = in[u * kWaveSize + lane];
                }
                if (st == kAuxAgent) {
#pragma unroll
                    for (int u = 0; u < U; ++u) AgentIO<V, 0, kAuxAgent>::st(r[u], rd, off + u * kWaveSize * V);
                } else {
#pragma unroll
                    for (int u = 0; u < U; ++u) AgentIO<V, 0, kAuxCached>::st(r[u], rd, off + u * kWaveSize * V);
                }
                if (!last) {
                    T *out = reinterpret_cast<T *>(trip_slots) + (j * 2 + (seq & 1)) * (U * kWaveSize);
#pragma unroll
                    for (int u = 0; u < U; ++u) out[u * kWaveSize + lane] = r[u];
                }
            } else if (lean) {
                const unsigned off = lane * V;
                if (ld == kAuxAgent) {
                    if (st == kAuxAgent) move_trip<V, U, kAuxAgent, kAuxAgent>(rs, rd, off);
                    else move_trip<V, U, kAuxAgent, kAuxCached>(rs, rd, off);
                } else {
                    if (st == kAuxAgent) move_trip<V, U, kAuxCached, kAuxAgent>(rs, rd, off);
                    else move_trip<V, U, kAuxCached, kAuxCached>(rs, rd, off);
                }
            } else {
                copy_span_policy<V, U>(dst, src, lo, hi, lane, ld, st);
            }
            ++seq;
            // the stores above were issued with the loaded data, so the loads of this trip have returned
            if (!first && lane == 0)
                __hip_atomic_store(&trips_read[j], seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (!last && !muted) {
                // forward: the trip is stored (complete and written through) before the right neighbour is told;
                // a trip handed over in LDS is complete there once the release below has waited for the LDS writes
                if (!via_lds) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                if (lane == 0) __hip_atomic_store(&trips_done[j], seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        if (in_flag && c + 1 < a.nchunks) seen = read_flag(in_flag, lane);
        if (out_flag) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0)
                __hip_atomic_store(out_flag, base + ((u64)(c + 1) << 4), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ---------------------------------------------------------------------------
// Pipelined k-nomial tree in one launch: the tree of Eq. 3 with the chunking and
// the ready flags of the pipelined chain (this build's own combination of the
// two: Sec. IV-B pipelines the chain only).  Every receiving position
// has `lanes` wavefronts of its own; wavefront (position, lane) waits until its
// PARENT position has published lane's share of chunk c, copies it out of the
// parent's buffer into its own, and publishes it for its children.  A chunk
// therefore moves down all levels of the tree while later chunks follow, and a
// small message needs one launch and ceil(log_k P) flag hand-offs instead of
// one launch per level.  The protocol, the flag layout (flag(position, lane))
// and the wait limit are the chain kernel's.  Every buffer is read by other
// wavefronts (the children's), so every access is agent-scope.  Wavefronts are
// numbered position-major and a parent's position is below its children's, so
// a wave only waits for a wave with a lower workgroup index.
template <int V>
__global__ void __launch_bounds__(kBlockThreads) tree_kernel(const ChainArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const unsigned gw = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (gw >= (a.nranks - 1) * a.lanes) return;
    const u64 base = run_base(a, lane);
    const unsigned pos = gw / a.lanes + 1;  // the position this wave receives for
    const unsigned s = gw - (pos - 1) * a.lanes;
    const unsigned par = a.parent[pos];
    const u64 *in_flag = par > 0 ? a.flags + ((u64)(par - 1) * a.lanes + s) * kFlagStrideWords : nullptr;
    const bool forwards = ((a.forward_mask >> pos) & 1) != 0 && a.mute_hop != pos;
    u64 *out_flag = forwards ? a.flags + ((u64)(pos - 1) * a.lanes + s) * kFlagStrideWords : nullptr;
    const char *src = a.buf[par];
    char *dst = a.buf[pos];

    const u64 trip = (u64)kTripUnrollDefault * kWaveSize * V;
    const u64 stride = trip * a.lanes;
    u64 seen = 0;
    u64 chunk_lo = 0;
    for (unsigned c = 0; c < a.nchunks; ++c, chunk_lo += a.chunk_bytes) {
        u64 chunk_hi = chunk_lo + a.chunk_bytes;
        if (chunk_hi > a.bytes) chunk_hi = a.bytes;
        if (in_flag) {
            const u64 want = base + ((u64)(c + 1) << 4);
            if (seen < want && !wait_ready(in_flag, want, a, base, pos, c, lane, &seen)) return;
            asm volatile("" ::: "memory");  // also behind the look-ahead read of the flag
        }
        for (u64 lo = chunk_lo + (u64)s * trip; lo < chunk_hi; lo += stride) {
            const u64 hi = lo + trip < chunk_hi ? lo + trip : chunk_hi;
            copy_span_agent<V, kTripUnrollDefault>(dst, src, lo, hi, lane);
        }
        if (in_flag && c + 1 < a.nchunks) seen = read_flag(in_flag, lane);
        if (out_flag) {
            // all payload stores of this wave are complete and, being
            // write-through, visible device-wide before the flag is raised
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) __hip_atomic_store(out_flag, base + ((u64)(c + 1) << 4), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ---------------------------------------------------------------------------
// Pipelined chain reduction (fp32 sum): the collective the paper names as next
// in line for the pipelined chain (Sec. VII), built as the broadcast chain of
// Sec. IV-B run backwards.  Chain position P-1 starts the running sum of a chunk
// with its own contribution, every position below adds its own with one fp32
// addition per element and hands the sum on, position 0 (the root) stores it:
//     recv = x_0 + (x_1 + ( ... + (x_{P-2} + x_{P-1})))
// with every addition rounded to fp32, the order the CPU reference fixes, so the
// two agree bit for bit.
//
// Stages, lanes, chunks, flags and the wait limit are the chain kernel's: "hop"
// j = 1..P-1 is position P-1-j adding its contribution; stage g plays the
// consecutive hops stage_begin(g)+1 .. stage_begin(g+1).  Inside a stage the
// running sum of a trip stays in registers (it is a new value at every hop and
// nobody but the next position needs it); between stages it goes through a
// scratch buffer in memory -- written through at agent scope, flag raised, read
// at agent scope by the same lane of the next stage.  The contributions are
// read exactly once, B positions at a time so that their loads are in flight
// together; the additions then run in chain order.  Two shapes are built: trips
// of 4 KiB per position, 4 positions at a time, for messages that stream, and
// trips of 1 KiB, 16 positions at a time, for small ones, where the number of
// dependent memory round trips per stage is what a reduction takes
// (P = 64, 4 KiB: 2 instead of 8 per stage).

__device__ __forceinline__ void add_f32x4(VecOf<16>::type &acc, const VecOf<16>::type &x)
{
    // own + incoming, element by element; no contraction is possible (no multiply)
    acc.x = __float_as_uint(__uint_as_float(x.x) + __uint_as_float(acc.x));
    acc.y = __float_as_uint(__uint_as_float(x.y) + __uint_as_float(acc.y));
    acc.z = __float_as_uint(__uint_as_float(x.z) + __uint_as_float(acc.z));
    acc.w = __float_as_uint(__uint_as_float(x.w) + __uint_as_float(acc.w));
}

// One span [lo, hi) (at most one trip; a multiple of sizeof(T) bytes) through the
// hops first_hop .. last_hop: T is a 16-byte vector of four floats or one float.
// The buffer address that lane `pos` of the wave holds in (ptr_lo, ptr_hi): a
// register read instead of a dependent scalar load from the argument segment
// per position (measured: a reduction of up to 64 KiB over 64 ranks 6.9 ->
// 5.3-5.5 us).
__device__ __forceinline__ const char *position_buffer(unsigned ptr_lo, unsigned ptr_hi, unsigned pos)
{
    const u64 lo = (u64)(unsigned)__builtin_amdgcn_readlane((int)ptr_lo, (int)pos);
    const u64 hi = (u64)(unsigned)__builtin_amdgcn_readlane((int)ptr_hi, (int)pos);
    return reinterpret_cast<const char *>((hi << 32) | lo);
}

template <int V, int U, int B, int LD_IN, int ST_OUT>
__device__ __forceinline__ void reduce_span(const ChainArgs &a, unsigned ptr_lo, unsigned ptr_hi, const char *in, char *out,
                                            unsigned first_hop, unsigned last_hop, u64 lo, unsigned n, unsigned lane)
{
    typedef AgentIO<V, LD_IN, ST_OUT> EDGE;            // the running sum coming in and going out
    typedef AgentIO<V, kAuxStream, kAuxCached> OWN;    // contributions: read once, never written
    typedef typename EDGE::T T;
    const unsigned top = a.nranks - 1;
    const unsigned off = lane * V;
    T acc[U];
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(in + lo), 0, n, kRsrcWord3);
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = EDGE::ld(rin, off + u * kWaveSize * V);
    for (unsigned hop = first_hop; hop <= last_hop; hop += B) {
        T x[B][U];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            if (hop + b <= last_hop) {  // wave-uniform
                const __amdgpu_buffer_rsrc_t rx =
                    __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(position_buffer(ptr_lo, ptr_hi, top - (hop + b)) + lo), 0, n, kRsrcWord3);
#pragma unroll
                for (int u = 0; u < U; ++u) x[b][u] = OWN::ld(rx, off + u * kWaveSize * V);
            }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            if (hop + b <= last_hop) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (V == 16) add_f32x4(acc[u], x[b][u]);
                    else acc[u] = __float_as_uint(__uint_as_float(x[b][u]) + __uint_as_float(acc[u]));
                }
            }
        }
    }
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(out + lo, 0, n, kRsrcWord3);
#pragma unroll
    for (int u = 0; u < U; ++u) EDGE::st(acc[u], rout, off + u * kWaveSize * V);
}

template <int U, int B>
__global__ void __launch_bounds__(kBlockThreads) reduce_kernel(const ChainArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const unsigned gw = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (gw >= a.stages * a.lanes) return;
    const u64 base = run_base(a, lane);
    const unsigned g = gw / a.lanes;
    const unsigned s = gw - g * a.lanes;
    const unsigned hops = a.nranks - 1;
    const unsigned hops_min = hops / a.stages, hops_extra = hops - hops_min * a.stages;
    const unsigned first_hop = stage_begin(g, 0, a.stages, hops_min, hops_extra) + 1;
    const unsigned last_hop = stage_begin(g + 1, 0, a.stages, hops_min, hops_extra);
    const bool last_stage = g + 1 == a.stages;
    // the result: written through (a store that does not linger in the L2 among
    // the streaming reads) or with ordinary write-back stores; the host's choice
    const bool result_through = (a.st_mid & kAuxAgent) != 0;

    const u64 *in_flag = g > 0 ? a.flags + ((u64)(g - 1) * a.lanes + s) * kFlagStrideWords : nullptr;
    const bool muted = a.mute_hop >= first_hop && a.mute_hop <= last_hop;
    u64 *out_flag = (!last_stage && !muted) ? a.flags + ((u64)g * a.lanes + s) * kFlagStrideWords : nullptr;
    // stage 0 starts from position P-1's contribution, later stages from the previous stage's sum
    const char *in = g > 0 ? a.scratch + (u64)(g - 1) * a.scratch_stride : a.buf[hops];
    char *out = last_stage ? a.recv : a.scratch + (u64)g * a.scratch_stride;

    // lane l keeps the address of position l's contribution (the table has a
    // slot per lane; slots beyond the rank count are never read out)
    static_assert(BCAST_MAX_RANKS == kWaveSize, "one lane per chain position");
    const u64 mine = reinterpret_cast<u64>(a.buf[lane]);
    const unsigned ptr_lo = (unsigned)mine, ptr_hi = (unsigned)(mine >> 32);

    const u64 trip = (u64)U * kWaveSize * 16;
    const u64 stride = trip * a.lanes;
    u64 seen = 0;
    u64 chunk_lo = 0;
    for (unsigned c = 0; c < a.nchunks; ++c, chunk_lo += a.chunk_bytes) {
        u64 chunk_hi = chunk_lo + a.chunk_bytes;
        if (chunk_hi > a.bytes) chunk_hi = a.bytes;
        if (in_flag) {
            const u64 want = base + ((u64)(c + 1) << 4);
            if (seen < want && !wait_ready(in_flag, want, a, base, first_hop, c, lane, &seen)) return;
            asm volatile("" ::: "memory");  // also behind the look-ahead read of the flag
        }
        for (u64 lo = chunk_lo + (u64)s * trip; lo < chunk_hi; lo += stride) {
            const u64 hi = lo + trip < chunk_hi ? lo + trip : chunk_hi;
            const unsigned n = (unsigned)(hi - lo);
            const unsigned body = n & ~15u;  // whole vectors of four floats; the rest (at the message's end) float by float
            if (g > 0 && !last_stage) {
                if (body) reduce_span<16, U, B, kAuxAgent, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo, body, lane);
                if (n != body) reduce_span<4, 1, B, kAuxAgent, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo + body, n - body, lane);
            } else if (g > 0) {
                if (result_through) {
                    if (body) reduce_span<16, U, B, kAuxAgent, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo, body, lane);
                    if (n != body) reduce_span<4, 1, B, kAuxAgent, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo + body, n - body, lane);
                } else {
                    if (body) reduce_span<16, U, B, kAuxAgent, kAuxCached>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo, body, lane);
                    if (n != body) reduce_span<4, 1, B, kAuxAgent, kAuxCached>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo + body, n - body, lane);
                }
            } else if (!last_stage) {
                if (body) reduce_span<16, U, B, kAuxStream, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo, body, lane);
                if (n != body) reduce_span<4, 1, B, kAuxStream, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo + body, n - body, lane);
            } else if (result_through) {
                if (body) reduce_span<16, U, B, kAuxStream, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo, body, lane);
                if (n != body) reduce_span<4, 1, B, kAuxStream, kAuxAgent>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo + body, n - body, lane);
            } else {
                if (body) reduce_span<16, U, B, kAuxStream, kAuxCached>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo, body, lane);
                if (n != body) reduce_span<4, 1, B, kAuxStream, kAuxCached>(a, ptr_lo, ptr_hi, in, out, first_hop, last_hop, lo + body, n - body, lane);
            }
        }
        if (in_flag && c + 1 < a.nchunks) seen = read_flag(in_flag, lane);
        if (out_flag) {
            // the running sums of this chunk are written through and complete before the flag is raised
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) __hip_atomic_store(out_flag, base + ((u64)(c + 1) << 4), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ---------------------------------------------------------------------------
// Whole-message copies src -> dst for up to 32 pairs at once (blockIdx.y picks
// the pair): one round of the binomial tree (Sec. III-A, Eq. 3) or one send of
// the direct algorithm (Eq. 1).  Waves stride over 4 KiB tiles.
// ---------------------------------------------------------------------------
template <int V>
__global__ void __launch_bounds__(kBlockThreads) pair_copy_kernel(const CopyArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const unsigned pair = blockIdx.y;
    const char *src = a.buf[a.src_pos[pair]];
    char *dst = a.buf[a.dst_pos[pair]];
    const u64 nwaves = (u64)gridDim.x * kWavesPerBlock;
    u64 w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    for (u64 lo = a.lo + w * kTileBytes; lo < a.hi; lo += nwaves * kTileBytes) {
        u64 hi = lo + kTileBytes;
        if (hi > a.hi) hi = a.hi;
        copy_span<V>(dst, src, lo, hi, lane);
    }
}

// Copies with a byte range per pair (blockIdx.y picks the pair): the pieces
// moved by one round of the binomial scatter or one step of the ring allgather
// (Sec. III-A, Eq. 4).  Empty ranges are skipped.
template <int V>
__global__ void __launch_bounds__(kBlockThreads) ranged_copy_kernel(const RangedCopyArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const unsigned pair = blockIdx.y;
    const char *src = a.buf[a.src_pos[pair]];
    char *dst = a.buf[a.dst_pos[pair]];
    const u64 end = a.hi[pair];
    const u64 nwaves = (u64)gridDim.x * kWavesPerBlock;
    u64 w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    for (u64 lo = a.lo[pair] + w * kTileBytes; lo < end; lo += nwaves * kTileBytes) {
        u64 hi = lo + kTileBytes;
        if (hi > end) hi = end;
        copy_span<V>(dst, src, lo, hi, lane);
    }
}

// One-die fan-out: buf[0] is read once, every other position is written.
template <int V>
__global__ void __launch_bounds__(kBlockThreads) fanout_kernel(const CopyArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const u64 nwaves = (u64)gridDim.x * kWavesPerBlock;
    u64 w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    for (u64 lo = a.lo + w * kTileBytes; lo < a.hi; lo += nwaves * kTileBytes) {
        u64 hi = lo + kTileBytes;
        if (hi > a.hi) hi = a.hi;
        fanout_span<V>(a, lo, hi, lane);
    }
}

// ---------------------------------------------------------------------------
// Measurement kernels: what this device's memory gives the two access patterns
// every algorithm here is made of, with no dependencies at all.  store_pattern
// writes `nbufs` buffers of `bytes` bytes tile by tile (every 4 KiB tile to all
// buffers in turn, like the fan-out without its read): the floor of any
// broadcast to nbufs ranks on one die.  load_pattern reads `nbufs` buffers once
// (streaming loads, four buffers in flight per wave), folds them with xor and
// optionally writes the fold: the floor of the reduction.  bytes is a multiple
// of 4096 and every buffer 16-byte aligned (checked by the host).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlockThreads) store_pattern_kernel(const CopyArgs a)
{
    typedef VecOf<16>::type T;
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const u64 nwaves = (u64)gridDim.x * kWavesPerBlock;
    const u64 w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const T val = {(unsigned)w, lane, 0x5A5A5A5Au, 0xA5A5A5A5u};
    for (u64 lo = w * kTileBytes; lo < a.hi; lo += nwaves * kTileBytes)
        for (unsigned k = 0; k < a.nranks; ++k) {
            const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(a.buf[k] + lo, 0, (int)kTileBytes, kRsrcWord3);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) AgentIO<16, kAuxCached, kAuxCached>::st(val, r, lane * 16 + u * kWaveSize * 16);
        }
}

template <bool WRITE>
__global__ void __launch_bounds__(kBlockThreads) load_pattern_kernel(const CopyArgs a, char *out)
{
    typedef VecOf<16>::type T;
    typedef AgentIO<16, kAuxStream, kAuxAgent> IO;
    constexpr int B = 4;
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const u64 nwaves = (u64)gridDim.x * kWavesPerBlock;
    const u64 w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    for (u64 lo = w * kTileBytes; lo < a.hi; lo += nwaves * kTileBytes) {
        T acc[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc[u] = T{0, 0, 0, 0};
        for (unsigned k = 0; k < a.nranks; k += B) {
            T x[B][kUnroll];
#pragma unroll
            for (int b = 0; b < B; ++b)
                if (k + b < a.nranks) {
                    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(a.buf[k + b] + lo, 0, (int)kTileBytes, kRsrcWord3);
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) x[b][u] = IO::ld(r, lane * 16 + u * kWaveSize * 16);
                }
#pragma unroll
            for (int b = 0; b < B; ++b)
                if (k + b < a.nranks)
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) acc[u] ^= x[b][u];
        }
        // without WRITE the fold still decides a (never taken) store, so that every load is needed
        T fold = acc[0];
#pragma unroll
        for (int u = 1; u < kUnroll; ++u) fold ^= acc[u];
        if (WRITE || (fold.x ^ fold.y ^ fold.z ^ fold.w) == 0x9E3779B9u) {
            const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(out + lo, 0, (int)kTileBytes, kRsrcWord3);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) IO::st(acc[u], r, lane * 16 + u * kWaveSize * 16);
        }
    }
}

hipError_t launch_store_pattern(const CopyArgs &a, int grid_x, hipStream_t stream)
{
    if (grid_x < 1 || a.nranks < 1 || a.nranks > BCAST_MAX_RANKS || (a.hi % kTileBytes) != 0) return hipErrorInvalidValue;
    store_pattern_kernel<<<dim3(grid_x), dim3(kBlockThreads), 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_load_pattern(const CopyArgs &a, char *out, bool write_result, int grid_x, hipStream_t stream)
{
    if (grid_x < 1 || a.nranks < 1 || a.nranks > BCAST_MAX_RANKS || (a.hi % kTileBytes) != 0 || !out) return hipErrorInvalidValue;
    if (write_result) load_pattern_kernel<true><<<dim3(grid_x), dim3(kBlockThreads), 0, stream>>>(a, out);
    else load_pattern_kernel<false><<<dim3(grid_x), dim3(kBlockThreads), 0, stream>>>(a, out);
    return hipGetLastError();
}

// Launch KERNEL<V, ...> for the vector width the host found usable.
#define BCAST_LAUNCH_VB(KERNEL, vec_bytes, grid, block, stream, args, ...)                      \
    switch (vec_bytes) {                                                                        \
    case 16: KERNEL<16 __VA_OPT__(,) __VA_ARGS__><<<grid, block, 0, stream>>>(args); break;     \
    case 8: KERNEL<8 __VA_OPT__(,) __VA_ARGS__><<<grid, block, 0, stream>>>(args); break;       \
    case 4: KERNEL<4 __VA_OPT__(,) __VA_ARGS__><<<grid, block, 0, stream>>>(args); break;       \
    case 1: KERNEL<1 __VA_OPT__(,) __VA_ARGS__><<<grid, block, 0, stream>>>(args); break;       \
    default: return hipErrorInvalidValue;                                                       \
    }
#define BCAST_LAUNCH_V(KERNEL, vec_bytes, grid, stream, args, ...) \
    BCAST_LAUNCH_VB(KERNEL, vec_bytes, grid, dim3(kBlockThreads), stream, args __VA_OPT__(,) __VA_ARGS__)

static bool valid_policy(unsigned aux) { return (aux & ~(unsigned)(kAuxAgent | kAuxStream)) == 0; }

bool valid_chain_block(int block_threads) { return block_threads == 64 || block_threads == 128 || block_threads == 256; }

hipError_t launch_chain(const ChainArgs &a, int vec_bytes, int grid_blocks, int block_threads, hipStream_t stream)
{
    if (grid_blocks < 1 || !valid_chain_block(block_threads)) return hipErrorInvalidValue;
    if ((u64)grid_blocks * (unsigned)(block_threads / kWaveSize) < (u64)a.stages * a.lanes) return hipErrorInvalidValue;
    // what another stage's wave stored is loaded at agent scope; a wave's own
    // write-back stores are not read back at agent scope
    if (!valid_policy(a.ld_root) || !valid_policy(a.ld_edge) || !valid_policy(a.ld_back) || !valid_policy(a.st_mid)) return hipErrorInvalidValue;
    if (!(a.ld_edge & kAuxAgent)) return hipErrorInvalidValue;
    if (!(a.st_mid & kAuxAgent) && (a.ld_back & kAuxAgent)) return hipErrorInvalidValue;
    const dim3 grid(grid_blocks), block(block_threads);
    const bool usual = a.ld_root == kAuxAgent && a.ld_edge == kAuxAgent && a.ld_back == kAuxCached;
    const int policy = usual && a.st_mid == kAuxAgent ? kPolicyThrough : usual && a.st_mid == kAuxCached ? kPolicyBack : kPolicyArgs;
#define BCAST_LAUNCH_CHAIN(U)                                                                      \
    switch (policy) {                                                                              \
    case kPolicyThrough: BCAST_LAUNCH_VB(chain_kernel, vec_bytes, grid, block, stream, a, U, kPolicyThrough); break; \
    case kPolicyBack: BCAST_LAUNCH_VB(chain_kernel, vec_bytes, grid, block, stream, a, U, kPolicyBack); break;       \
    default: BCAST_LAUNCH_VB(chain_kernel, vec_bytes, grid, block, stream, a, U, kPolicyArgs); break;                \
    }
    switch (a.unroll) {
    case 2: BCAST_LAUNCH_CHAIN(2) break;
    case 3: BCAST_LAUNCH_CHAIN(3) break;
    case 4: BCAST_LAUNCH_CHAIN(4) break;
    case 6: BCAST_LAUNCH_CHAIN(6) break;
    default: return hipErrorInvalidValue;
    }
#undef BCAST_LAUNCH_CHAIN
    return hipGetLastError();
}

size_t rank_chain_lds_bytes(int waves, int unroll, int vec_bytes)
{
    return (size_t)waves * 2 * unroll * kWaveSize * vec_bytes;
}

// A launch with more dynamic LDS than the default allowance has to be announced
// to the runtime once per kernel and device; the largest size announced so far
// is remembered so that a run enqueues nothing but its kernel.
template <int V, int U>
static hipError_t allow_rank_chain_lds(int device, size_t lds)
{
    static std::atomic<size_t> allowed[kStaticMaxDevices];
    constexpr size_t kDefaultAllowance = 48u << 10;
    if (lds <= kDefaultAllowance || lds <= allowed[device].load(std::memory_order_acquire)) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(rank_chain_kernel<V, U>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    size_t seen = allowed[device].load(std::memory_order_relaxed);
    while (seen < lds && !allowed[device].compare_exchange_weak(seen, lds, std::memory_order_release)) {}
    return hipSuccess;
}

hipError_t launch_rank_chain(const ChainArgs &a, int vec_bytes, int grid_blocks, int block_threads, int device, int lds_limit,
                             hipStream_t stream)
{
    if (a.nranks < 2 || a.stages < 1 || a.stages > a.nranks - 1 || a.lanes < 1) return hipErrorInvalidValue;
    // one wave per hop of the longest stage, one workgroup per (stage, lane)
    const unsigned longest = (a.nranks - 1 + a.stages - 1) / a.stages;
    if (longest > (unsigned)kRankWavesMax || block_threads != (int)(longest * kWaveSize)) return hipErrorInvalidValue;
    if ((u64)grid_blocks != (u64)a.stages * a.lanes) return hipErrorInvalidValue;
    if (!(a.mode & kModeFixedSpans)) return hipErrorInvalidValue;  // a wave keeps its position for every chunk
    if (!valid_policy(a.ld_root) || !valid_policy(a.ld_edge) || !valid_policy(a.ld_back) || !valid_policy(a.st_mid)) return hipErrorInvalidValue;
    if (!(a.ld_edge & kAuxAgent)) return hipErrorInvalidValue;
    const dim3 grid(grid_blocks), block(block_threads);
    // LDS hand-off: two trip slots per wave of the workgroup, beside the kernel's own counters
    size_t lds = 0;
    if (a.mode & kModeLdsHandoff) {
        lds = rank_chain_lds_bytes((int)longest, (int)a.unroll, vec_bytes);
        if (device < 0 || device >= kStaticMaxDevices || lds_limit < 0 || lds + kRankStaticLdsBytes > (size_t)lds_limit) return hipErrorInvalidValue;
    }
#define BCAST_LAUNCH_RANK_V(V, U)                                                                                        \
    {                                                                                                                    \
        hipError_t e = allow_rank_chain_lds<V, U>(device, lds);                                                          \
        if (e != hipSuccess) return e;                                                                                   \
        rank_chain_kernel<V, U><<<grid, block, lds, stream>>>(a);                                                        \
    }
#define BCAST_LAUNCH_RANK(U)                        \
    switch (vec_bytes) {                            \
    case 16: BCAST_LAUNCH_RANK_V(16, U) break;      \
    case 8: BCAST_LAUNCH_RANK_V(8, U) break;        \
    case 4: BCAST_LAUNCH_RANK_V(4, U) break;        \
    case 1: BCAST_LAUNCH_RANK_V(1, U) break;        \
    default: return hipErrorInvalidValue;           \
    }
    switch (a.unroll) {
    case 1: BCAST_LAUNCH_RANK(1) break;
    case 2: BCAST_LAUNCH_RANK(2) break;
    case 3: BCAST_LAUNCH_RANK(3) break;
    case 4: BCAST_LAUNCH_RANK(4) break;
    case 6: BCAST_LAUNCH_RANK(6) break;
    case 8: BCAST_LAUNCH_RANK(8) break;
    default: return hipErrorInvalidValue;
    }
#undef BCAST_LAUNCH_RANK
#undef BCAST_LAUNCH_RANK_V
    return hipGetLastError();
}

hipError_t rank_chain_max_blocks_per_cu(int block_threads, int *blocks)
{
    int n[4] = {0, 0, 0, 0};
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n[0], rank_chain_kernel<16, 1>, block_threads, 0);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n[1], rank_chain_kernel<16, 2>, block_threads, 0);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n[2], rank_chain_kernel<16, 3>, block_threads, 0);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n[3], rank_chain_kernel<16, 4>, block_threads, 0);
    *blocks = n[0];
    for (int x : n)
        if (x < *blocks) *blocks = x;
    return e;
}

hipError_t launch_tree(const ChainArgs &a, int vec_bytes, int grid_blocks, hipStream_t stream)
{
    if (grid_blocks < 1 || a.nranks < 2 || a.nranks > BCAST_MAX_RANKS) return hipErrorInvalidValue;
    if ((u64)grid_blocks * kWavesPerBlock < (u64)(a.nranks - 1) * a.lanes) return hipErrorInvalidValue;
    for (unsigned q = 1; q < a.nranks; ++q)
        if (a.parent[q] >= q) return hipErrorInvalidValue;  // a parent lies below its child
    BCAST_LAUNCH_V(tree_kernel, vec_bytes, dim3(grid_blocks), stream, a);
    return hipGetLastError();
}

hipError_t launch_reduce(const ChainArgs &a, int grid_blocks, hipStream_t stream)
{
    if (grid_blocks < 1 || a.nranks < 2 || a.nranks > BCAST_MAX_RANKS || a.stages < 1 || a.stages > a.nranks - 1) return hipErrorInvalidValue;
    if ((u64)grid_blocks * kWavesPerBlock < (u64)a.stages * a.lanes) return hipErrorInvalidValue;
    if (!a.recv || (a.stages > 1 && !a.scratch) || (a.bytes & 3u)) return hipErrorInvalidValue;
    if (a.unroll == (unsigned)kRedUnrollSmall) reduce_kernel<kRedUnrollSmall, 16><<<dim3(grid_blocks), dim3(kBlockThreads), 0, stream>>>(a);
    else if (a.unroll == (unsigned)kRedUnroll) reduce_kernel<kRedUnroll, 4><<<dim3(grid_blocks), dim3(kBlockThreads), 0, stream>>>(a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t tree_max_blocks_per_cu(int *blocks)
{
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, tree_kernel<16>, kBlockThreads, 0);
}

hipError_t reduce_max_blocks_per_cu(int *blocks)
{
    int small = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, reduce_kernel<kRedUnroll, 4>, kBlockThreads, 0);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&small, reduce_kernel<kRedUnrollSmall, 16>, kBlockThreads, 0);
    if (e == hipSuccess && small < *blocks) *blocks = small;
    return e;
}

hipError_t launch_pair_copy(const CopyArgs &a, int vec_bytes, int grid_x, hipStream_t stream)
{
    if (grid_x < 1 || a.npairs < 1 || a.npairs > BCAST_MAX_RANKS / 2) return hipErrorInvalidValue;
    BCAST_LAUNCH_V(pair_copy_kernel, vec_bytes, dim3(grid_x, a.npairs), stream, a);
    return hipGetLastError();
}

hipError_t launch_fanout(const CopyArgs &a, int vec_bytes, int grid_x, hipStream_t stream)
{
    if (grid_x < 1) return hipErrorInvalidValue;
    BCAST_LAUNCH_V(fanout_kernel, vec_bytes, dim3(grid_x), stream, a);
    return hipGetLastError();
}

hipError_t launch_ranged_copy(const RangedCopyArgs &a, int vec_bytes, int grid_x, hipStream_t stream)
{
    if (grid_x < 1 || a.npairs < 1 || a.npairs > BCAST_MAX_RANKS) return hipErrorInvalidValue;
    BCAST_LAUNCH_V(ranged_copy_kernel, vec_bytes, dim3(grid_x, a.npairs), stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Scratch memory that exists without any allocation call: one array in the
// code object's data segment, for the entry point that callers use who cannot
// allocate (bcast_reduce_sum_f32_static).  Layout: the ready flags, the abort
// word and the run counter first (kStaticFlagLines lines of 128 bytes), then the staging area
// for the running sums that cross a stage boundary (kStaticStagingBytes).  Every
// GPU the library runs on holds its own copy, zero-filled when the code object
// is loaded, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: the address of a device's copy is looked up
// once per device, with that device current, and that pointer is what every
// launch, fill and copy uses.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
struct StaticScratchSlot {
    char *ptr = nullptr;
    bool looked_up = false;
};
StaticScratchSlot g_static_slot[kStaticMaxDevices];
std::mutex g_static_mu;
}  // namespace

hipError_t static_scratch_address(int device, char **ptr)
{
    if (!ptr || device < 0 || device >= kStaticMaxDevices) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> g(g_static_mu);
    StaticScratchSlot &slot = g_static_slot[device];
    if (!slot.looked_up) {
        int current = -1;
        hipError_t e = hipGetDevice(&current);
        if (e != hipSuccess) return e;
        if (current != device) return hipErrorInvalidDevice;  // the look-up answers for the current device
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || ((uintptr_t)p & 255u)) return hipErrorInvalidSymbol;
        slot.ptr = (char *)p;
        slot.looked_up = true;
    }
    *ptr = slot.ptr;
    return hipSuccess;
}

// The run counter in device memory, for launches that must be replayable from a
// captured graph (and for the static array, which no host counter could follow
// through replays).  One workgroup, enqueued ahead of every flag kernel that
// reads the counter: it adds one, and when the 32-bit count in the flag words
// would wrap it first clears `clear_words` words at `flags` (ready flags and
// abort word) and starts again at one -- a fill by a kernel, which a graph
// replays correctly, with no allocation.  Stream order puts it after the run
// before and ahead of the run that reads it.
__global__ void __launch_bounds__(kBlockThreads) advance_epoch_kernel(u64 *epoch_word, u64 *flags, u64 clear_words, u64 limit)
{
    u64 epoch = *epoch_word;  // every thread reads it before thread 0 writes it (barrier below)
    if (epoch >= limit) {
        for (u64 i = threadIdx.x; i < clear_words; i += kBlockThreads) flags[i] = 0;
        epoch = 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) *epoch_word = epoch + 1;
}

hipError_t launch_advance_epoch(u64 *epoch_word, u64 *flags, u64 clear_words, u64 limit, hipStream_t stream)
{
    if (!epoch_word || !flags || clear_words == 0) return hipErrorInvalidValue;
    // the counter must lie outside what a wrap clears
    if (epoch_word >= flags && epoch_word < flags + clear_words) return hipErrorInvalidValue;
    advance_epoch_kernel<<<dim3(1), dim3(kBlockThreads), 0, stream>>>(epoch_word, flags, clear_words, limit);
    return hipGetLastError();
}

bool valid_chain_unroll(int unroll) { return unroll == 2 || unroll == 3 || unroll == 4 || unroll == 6; }

hipError_t chain_max_blocks_per_cu(int block_threads, int *blocks)
{
    // the smallest over the trip sizes and policy sets the kernel is built for
    int n[12] = {0};
    hipError_t e = hipSuccess;
    int k = 0;
#define BCAST_CHAIN_OCCUPANCY(U, POLICY) \
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n[k++], chain_kernel<16, U, POLICY>, block_threads, 0);
#define BCAST_CHAIN_OCCUPANCY_U(U) \
    BCAST_CHAIN_OCCUPANCY(U, kPolicyThrough) BCAST_CHAIN_OCCUPANCY(U, kPolicyBack) BCAST_CHAIN_OCCUPANCY(U, kPolicyArgs)
    BCAST_CHAIN_OCCUPANCY_U(2)
    BCAST_CHAIN_OCCUPANCY_U(3)
    BCAST_CHAIN_OCCUPANCY_U(4)
    BCAST_CHAIN_OCCUPANCY_U(6)
#undef BCAST_CHAIN_OCCUPANCY_U
#undef BCAST_CHAIN_OCCUPANCY
    if (e != hipSuccess) return e;
    *blocks = n[0];
    for (int x : n)
        if (x < *blocks) *blocks = x;
    return e;
}

}  // namespace bcast

// gfx950 kernels of the broadcast library.
//
// All kernels move raw bytes between device buffers of one GPU.  The unit of
// work is a wavefront (64 lanes): it copies one contiguous span with 16-byte
// accesses per lane (1 KiB per wave instruction, kUnroll of them in flight),
// and byte accesses for a head/tail that is not 16-byte aligned.  There are no
// workgroup barriers and no LDS: the path is bound by HBM, not by arithmetic.
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
// Pipelined chain (Sec. IV-B).  Wavefront (hop, lane) receives lane's slice of
// every chunk from position hop-1 into position hop and then publishes it to
// position hop+1 -- the receive / store / forward loop of a middle rank.
// Position 0 (the root) only sends: nobody writes its buffer.  The last
// position only receives: it publishes nothing.
//
// Hand-off protocol.  flag(hop, lane) counts the chunks of this run that
// position `hop` has stored for `lane`, as base + count with base = epoch<<32;
// flags only grow, so nothing is reset between runs.  Producer: all lanes'
// stores are drained and written back (agent-scope release fence, executed by
// the whole wave so it covers every lane's stores), then lane 0 stores the
// flag.  Consumer: polls the flag with relaxed agent-scope loads (one address
// per wave), then an agent-scope acquire fence before touching the payload.
//
// Forward progress.  Wavefronts are numbered hop-major, so a wave only ever
// waits for a wave with a lower workgroup index; the host also keeps the grid
// within what the device can hold at once.  Every wait is bounded by a clock
// limit: a wave that gives up records (hop, chunk), raises the abort word so
// that the others stop waiting too, and returns.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void report_timeout(const ChainArgs &a, unsigned hop, unsigned chunk)
{
    const u64 epoch = a.base >> 32;
    const u64 old = __hip_atomic_fetch_max(a.abort_word, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old < epoch && a.status[0] == 0) {  // first wave of this run to give up
        __hip_atomic_store(&a.status[1], ((u64)hop << 32) | chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(&a.status[0], (u64)1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

__device__ __forceinline__ bool wait_ready(const u64 *flag, u64 want, const ChainArgs &a, unsigned hop,
                                           unsigned chunk, unsigned lane)
{
    u64 v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (v < want) {
        const u64 t0 = wall_clock64();
        const u64 epoch = a.base >> 32;
        unsigned spins = 0;
        for (;;) {
            __builtin_amdgcn_s_sleep(1);
            v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v >= want) break;
            if ((++spins & 31u) == 0) {
                if (__hip_atomic_load(a.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= epoch)
                    return false;
                if (wall_clock64() - t0 > a.spin_ticks) {
                    if (lane == 0) report_timeout(a, hop, chunk);
                    return false;
                }
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return true;
}

template <int V>
__global__ void __launch_bounds__(kBlockThreads) chain_kernel(const ChainArgs a)
{
    const unsigned lane = threadIdx.x & (kWaveSize - 1);
    const unsigned gw = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const unsigned nwaves = (a.nranks - 1) * a.lanes;
    if (gw >= nwaves) return;
    const unsigned hop = gw / a.lanes + 1;  // this wave fills chain position `hop`
    const unsigned s = gw - (hop - 1) * a.lanes;

    const char *src = a.buf[hop - 1];
    char *dst = a.buf[hop];
    const u64 *in_flag = hop > 1 ? a.flags + ((u64)(hop - 2) * a.lanes + s) * kFlagStrideWords : nullptr;
    u64 *out_flag = (hop + 1 < a.nranks && hop != a.mute_hop)
                        ? a.flags + ((u64)(hop - 1) * a.lanes + s) * kFlagStrideWords
                        : nullptr;

    u64 chunk_lo = 0;
    for (unsigned c = 0; c < a.nchunks; ++c, chunk_lo += a.chunk_bytes) {
        u64 chunk_hi = chunk_lo + a.chunk_bytes;
        if (chunk_hi > a.bytes) chunk_hi = a.bytes;
        u64 lo = chunk_lo + (u64)s * a.slice_bytes;
        u64 hi = lo + a.slice_bytes;
        if (hi > chunk_hi) hi = chunk_hi;

        if (in_flag && !wait_ready(in_flag, a.base + c + 1, a, hop, c, lane)) return;
        if (lo < hi) copy_span<V>(dst, src, lo, hi, lane);
        if (out_flag) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            if (lane == 0)
                __hip_atomic_store(out_flag, a.base + c + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

// Launch KERNEL<V> for the vector width the host found usable.
#define BCAST_LAUNCH_V(KERNEL, vec_bytes, grid, stream, args)                              \
    switch (vec_bytes) {                                                                   \
    case 16: KERNEL<16><<<grid, dim3(kBlockThreads), 0, stream>>>(args); break;            \
    case 8: KERNEL<8><<<grid, dim3(kBlockThreads), 0, stream>>>(args); break;              \
    case 4: KERNEL<4><<<grid, dim3(kBlockThreads), 0, stream>>>(args); break;              \
    case 1: KERNEL<1><<<grid, dim3(kBlockThreads), 0, stream>>>(args); break;              \
    default: return hipErrorInvalidValue;                                                  \
    }

hipError_t launch_chain(const ChainArgs &a, int vec_bytes, int grid_blocks, hipStream_t stream)
{
    if (grid_blocks < 1) return hipErrorInvalidValue;
    BCAST_LAUNCH_V(chain_kernel, vec_bytes, dim3(grid_blocks), stream, a);
    return hipGetLastError();
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

hipError_t chain_max_blocks_per_cu(int *blocks)
{
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, chain_kernel<16>, kBlockThreads, 0);
}

}  // namespace bcast

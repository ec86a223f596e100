// Placement of buffers in the device's memory (bcast_memory_regions,
// bcast_buffers_alloc, bcast_buffers_free in bcast.h).
//
// Measured on MI355X (288 GB of HBM3E): the device's memory answers as three
// regions, each a third of the physical address range.  A stream of writes whose
// targets all lie in one region runs at 5.9 TB/s; spread over two or three
// regions it runs at 7.1 TB/s.  Reads mixed with writes to the SAME region cost
// far more than their bytes (a reduction that reads 32 x 512 MiB and writes
// 512 MiB takes 3.07 ms with the result next to the inputs, 2.66 ms with the
// result in another region); pure reads are a few percent faster from one
// region than from two.  This is what ranks of DRAM behind shared channels do
// (write-to-read turnaround and refresh are per rank), and twelve-high stacks
// have three.  So a broadcast wants its receiving buffers spread over two
// regions, a reduction its contributions in one region and its result in
// another -- a choice only the allocating side can make.
//
// HIP has no call that allocates at a physical address, and the order in which
// the driver hands memory out depends on everything allocated and freed before,
// by this process and by earlier ones.  Two things hold regardless (measured in
// first and in later processes on a device): an allocation of a power-of-two
// size up to 16 GiB comes out of one region, and whether two allocations lie in
// the same region shows plainly when both are written at once (5.7-6.3 TB/s
// against 6.9-7.2).  bcast_buffers_alloc builds on just these: buffers that
// share a region label are packed into slabs of a power-of-two size; a slab
// whose label differs from that of slabs placed before is accepted only if
// writing to it together with each of them runs at the spread rate; a candidate
// that fails is kept aside, so that the next one is other memory, and freed at
// the end.  Nothing is assumed about addresses, and the verdict is a measurement.
#include <algorithm>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include "bcast_internal.h"

using namespace bcast;

namespace {

constexpr int kRegionCount = 3;
constexpr size_t kMiB = (size_t)1 << 20;
constexpr size_t kGiB = (size_t)1 << 30;
constexpr size_t kBufferAlign = 2 * kMiB;          // buffers start on 2 MiB boundaries inside a slab
constexpr size_t kSlabMax = 16 * kGiB;             // the largest power-of-two allocation seen to lie in one region every time
constexpr size_t kSlabMin = 2 * kGiB;              // the smallest slab a probe can judge: the 256 MiB memory-side cache takes that much of
                                                   // every pass off the memory, which must stay a few percent of what a probe writes
constexpr size_t kProbeWindows = 8;                // windows of a slab that a probe writes to, spread evenly over it
constexpr size_t kProbeWindowMax = 256 * kMiB;
constexpr size_t kProbeMinBytes = 4 * kGiB;        // least bytes a probe of two slabs writes
constexpr size_t kAttempts = 10;                   // allocations tried for one slab, at least, before it is taken as it comes
constexpr size_t kWalkBytes = 112 * kGiB;          // ... and as many as walk past a region (96 GiB) and a margin
constexpr size_t kWalkAllocsMax = 64;              // ... but never more than this
constexpr size_t kProbeEvery = 8 * kGiB;           // small candidates are probed once per this many bytes walked
constexpr int kProbedAgainst = 4;                  // slabs of other labels a candidate is probed against, at most
constexpr double kProbeGain = 1.08;                // two slabs together vs the slower one alone: measured 1.15-1.20 across regions
constexpr size_t kMemorySideCache = 256 * kMiB;
constexpr double kSpreadRateGBps = 6500.0;         // store-only rate: 5700-6300 GB/s into one region, 6900-7200 over two (measured)

size_t round_up(size_t n, size_t to) { return (n + to - 1) / to * to; }

size_t pow2_ceil(size_t n)
{
    size_t p = 1;
    while (p < n) p <<= 1;
    return p;
}

int hip_status(hipError_t e)
{
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? BCAST_ERR_NOMEM : BCAST_ERR_HIP;
}

// One allocation that carries the buffers of one region label.
struct Slab {
    char *base = nullptr;
    size_t bytes = 0;           // allocated size
    int label = 0;
    std::vector<int> members;   // indices of the caller's buffers
    std::vector<size_t> offset; // of each member inside the slab
};

// Slabs handed out, so that bcast_buffers_free can return them: buffer address
// -> slab base, slab base -> buffers still alive.
std::mutex g_mu;
std::map<void *, void *> g_slab_of;
std::map<void *, int> g_live;

// A part of a device allocation as the probes see it: they never write beyond `bytes`.
struct Span {
    void *ptr;
    size_t bytes;
};

// `count` windows spread evenly over a slab; every window lies inside it.
std::vector<Span> windows_of(const Slab &s, size_t count = kProbeWindows)
{
    std::vector<Span> out;
    if (count == 0 || !s.base) return out;
    const size_t step = s.bytes / count / (size_t)kTileBytes * (size_t)kTileBytes;
    const size_t window = std::min(kProbeWindowMax, step);
    if (window == 0) return out;
    for (size_t k = 0; k < count; ++k) {
        const size_t at = k * step;
        if (at + window > s.bytes) break;  // cannot happen (count * step <= bytes): the bound is checked all the same
        out.push_back(Span{s.base + at, window});
    }
    return out;
}

// Milliseconds for one pass of the store-only pattern over the first `window`
// bytes of each span.  Refuses a window that any span does not hold.
int time_store_pattern(const std::vector<Span> &spans, size_t window, hipEvent_t e0, hipEvent_t e1, float *ms)
{
    if (spans.empty() || spans.size() > (size_t)BCAST_MAX_RANKS || window == 0 || window % kTileBytes != 0) return BCAST_ERR_ARG;
    std::vector<void *> bufs;
    for (const Span &s : spans) {
        if (!s.ptr || s.bytes < window) return BCAST_ERR_ARG;  // the kernel writes [0, window) of every buffer
        bufs.push_back(s.ptr);
    }
    int rc = bcast_debug_store_pattern(bufs.data(), (int)bufs.size(), window, nullptr);  // warms up, loads the kernel
    if (rc != BCAST_OK) return rc;
    float best = 1e30f;
    for (int i = 0; i < 3; ++i) {
        if (hipEventRecord(e0, nullptr) != hipSuccess) return BCAST_ERR_HIP;
        rc = bcast_debug_store_pattern(bufs.data(), (int)bufs.size(), window, nullptr);
        if (rc != BCAST_OK) return rc;
        if (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return BCAST_ERR_HIP;
        float t = 0.f;
        if (hipEventElapsedTime(&t, e0, e1) != hipSuccess) return BCAST_ERR_HIP;
        best = std::min(best, t);
    }
    *ms = best;
    return BCAST_OK;
}

// The rate from which a pass that writes `written` bytes counts as spread over
// regions: the memory-side cache keeps the last 256 MiB of every pass off the
// memory, which makes a short pass look faster than the memory is.
double spread_rate_for(size_t written)
{
    // kSpreadRateGBps is what separates the two cases in passes of kProbeMinBytes (4 GiB)
    const double kept_there = (double)kMemorySideCache / (double)kProbeMinBytes;
    const double kept = std::min(0.5, (double)kMemorySideCache / (double)written);
    return kSpreadRateGBps * (1.0 - kept_there) / (1.0 - kept);
}

// Whether writing to slabs a and b together runs at the rate of a write set
// spread over regions: clearly faster, byte for byte, than writing to the slower
// of the two alone, or at the spread rate outright.  *told is false if they are
// too small to tell.
int probe_spread(const Slab &sa, const Slab &sb, bool *told, bool *spread)
{
    *told = *spread = false;
    std::vector<Span> a = windows_of(sa), b = windows_of(sb), both;
    if (a.size() != kProbeWindows || b.size() != kProbeWindows) return BCAST_OK;
    size_t window = kProbeWindowMax;
    for (const Span &s : a) window = std::min(window, s.bytes);
    for (const Span &s : b) window = std::min(window, s.bytes);  // no span is written beyond its size
    window = window / (size_t)kTileBytes * (size_t)kTileBytes;
    if (window == 0 || 2 * kProbeWindows * window < kProbeMinBytes) return BCAST_OK;
    both = a;
    both.insert(both.end(), b.begin(), b.end());
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return BCAST_ERR_HIP;
    }
    // Each alone, both together, each alone again: the faster of its two times counts for a slab alone.  A probe
    // follows allocations during which the device sat idle, and a first measurement taken while its clocks come
    // back up is slow -- which, taken for a slab alone, would make the two together look like a gain.
    float t_a = 0.f, t_b = 0.f, t_both = 0.f, t_a2 = 0.f, t_b2 = 0.f;
    int rc = time_store_pattern(a, window, e0, e1, &t_a);
    if (rc == BCAST_OK) rc = time_store_pattern(b, window, e0, e1, &t_b);
    if (rc == BCAST_OK) rc = time_store_pattern(both, window, e0, e1, &t_both);
    if (rc == BCAST_OK) rc = time_store_pattern(a, window, e0, e1, &t_a2);
    if (rc == BCAST_OK) rc = time_store_pattern(b, window, e0, e1, &t_b2);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != BCAST_OK) return rc;
    t_a = std::min(t_a, t_a2);
    t_b = std::min(t_b, t_b2);
    *told = true;
    // `both` writes twice the bytes of either alone
    const double gain = 2.0 * std::max(t_a, t_b) / t_both;
    const size_t written = 2 * kProbeWindows * window;
    const double rate_gbps = (double)written / (t_both * 1e-3) / 1e9;
    *spread = gain >= kProbeGain || rate_gbps >= spread_rate_for(written);
    return BCAST_OK;
}

// Whether a slab lies in one region: written alone, it stays below the rate of a
// write set spread over regions.  (A power-of-two allocation mostly does; where
// much has been allocated and freed before, the driver may piece one together
// from several regions.)
int probe_one_region(const Slab &s, bool *told, bool *one_region)
{
    *told = *one_region = false;
    // as many bytes as a probe of two slabs writes, where the slab has them
    const size_t count = s.bytes >= 2 * kProbeWindows * kProbeWindowMax ? 2 * kProbeWindows : kProbeWindows;
    std::vector<Span> w = windows_of(s, count);
    if (w.size() != count) return BCAST_OK;
    const size_t window = w[0].bytes / (size_t)kTileBytes * (size_t)kTileBytes;
    const size_t written = count * window;
    if (window == 0 || written < kProbeMinBytes / 2) return BCAST_OK;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return BCAST_ERR_HIP;
    }
    float t = 0.f;
    int rc = time_store_pattern(w, window, e0, e1, &t);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != BCAST_OK) return rc;
    *told = true;
    *one_region = (double)written / (t * 1e-3) / 1e9 < spread_rate_for(written);
    return BCAST_OK;
}

}  // namespace

extern "C" int bcast_memory_regions(int *count, size_t *region_bytes)
{
    if (!count || !region_bytes) return BCAST_ERR_ARG;
    size_t free_bytes = 0, total = 0;
    hipError_t e = hipMemGetInfo(&free_bytes, &total);
    if (e != hipSuccess) return hip_status(e);
    *count = kRegionCount;
    *region_bytes = total / kRegionCount;
    return BCAST_OK;
}

extern "C" int bcast_buffers_free(int n, void *const *ptrs)
{
    if (n < 0 || (n > 0 && !ptrs)) return BCAST_ERR_ARG;
    int rc = BCAST_OK;
    std::lock_guard<std::mutex> g(g_mu);
    for (int i = 0; i < n; ++i) {
        if (!ptrs[i]) continue;
        auto it = g_slab_of.find(ptrs[i]);
        if (it == g_slab_of.end()) {
            rc = BCAST_ERR_ARG;  // not a buffer this library handed out (or freed already)
            continue;
        }
        void *base = it->second;
        g_slab_of.erase(it);
        auto live = g_live.find(base);
        if (live != g_live.end() && --live->second == 0) {
            g_live.erase(live);
            hipError_t e = hipFree(base);
            if (e != hipSuccess) rc = hip_status(e);
        }
    }
    return rc;
}

extern "C" int bcast_buffers_alloc(int n, const size_t *bytes, const int *region, void **ptrs, int *placed)
{
    if (n < 1 || n > (1 << 16) || !bytes || !region || !ptrs) return BCAST_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        if (bytes[i] == 0 || region[i] < 0 || region[i] >= kRegionCount) return BCAST_ERR_ARG;
        ptrs[i] = nullptr;
    }
    if (placed) *placed = BCAST_PLACED_NO;

    // Pack the buffers of each label, in the caller's order, into slabs of at most
    // kSlabMax bytes (a buffer larger than that gets a slab of its own); a slab is
    // allocated at the next power of two, kSlabMin at least.
    std::vector<Slab> slabs;
    int labels_used = 0;
    for (int label = 0; label < kRegionCount; ++label) {
        Slab cur;
        size_t fill = 0;
        const size_t before = slabs.size();
        auto close = [&]() {
            if (cur.members.empty()) return;
            cur.label = label;
            cur.bytes = std::max(kSlabMin, fill <= kSlabMax ? pow2_ceil(fill) : fill);
            slabs.push_back(cur);
            cur = Slab();
            fill = 0;
        };
        for (int i = 0; i < n; ++i) {
            if (region[i] != label) continue;
            const size_t need = round_up(bytes[i], kBufferAlign);
            if (!cur.members.empty() && fill + need > kSlabMax) close();
            cur.members.push_back(i);
            cur.offset.push_back(fill);
            fill += need;
        }
        close();
        if (slabs.size() > before) ++labels_used;
    }

    std::vector<char *> aside;  // candidates that lay in the wrong region, and jumps past them
    auto release = [&](bool slabs_too) {
        for (char *p : aside) (void)hipFree(p);
        aside.clear();
        if (slabs_too)
            for (Slab &s : slabs)
                if (s.base) {
                    (void)hipFree(s.base);
                    s.base = nullptr;
                }
    };

    bool any_told = false, any_failed = false;
    for (size_t k = 0; k < slabs.size(); ++k) {
        Slab &s = slabs[k];
        // the slabs placed so far whose label differs: this one must lie apart from each (the first few are checked)
        std::vector<const Slab *> others;
        for (size_t j = 0; j < k && (int)others.size() < kProbedAgainst; ++j)
            if (slabs[j].label != s.label) others.push_back(&slabs[j]);
        // Candidates are allocations of the slab's own size, taken one after the other
        // and kept aside while they fail: equal allocations are what the driver hands
        // out in order where it has an order, so the walk crosses into another region
        // after at most a region's worth of them; where it has none, the first or
        // second candidate already lies apart.  Small candidates are probed only every
        // kProbeEvery bytes of the walk.
        const size_t stride = std::max<size_t>(1, kProbeEvery / s.bytes);
        const size_t max_allocs = std::min<size_t>(kWalkAllocsMax, std::max<size_t>(kAttempts, kWalkBytes / s.bytes));
        for (size_t alloc = 0;; ++alloc) {
            void *p = nullptr;
            hipError_t e = hipMalloc(&p, s.bytes);
            if (e != hipSuccess) {
                // out of memory with candidates kept aside: give those back and take the next allocation as it comes
                const bool had_aside = !aside.empty();
                (void)hipGetLastError();
                release(false);
                if (!had_aside || hipMalloc(&p, s.bytes) != hipSuccess) {
                    (void)hipGetLastError();
                    release(true);
                    return e == hipErrorOutOfMemory ? BCAST_ERR_NOMEM : BCAST_ERR_HIP;
                }
                s.base = (char *)p;
                if (!others.empty()) any_failed = true;
                break;
            }
            s.base = (char *)p;
            if (labels_used < 2) break;  // one label only: nothing to place
            const bool last = alloc + 1 >= max_allocs;
            bool apart = false;
            if (alloc % stride == 0 || last) {
                // in one region itself, and apart from the slabs of other labels
                bool told = false, one_region = false;
                int rc1 = probe_one_region(s, &told, &one_region);
                if (rc1 != BCAST_OK) {
                    release(true);
                    return rc1;
                }
                any_told = any_told || told;
                apart = !told || one_region;
                for (const Slab *o : others) {
                    if (!apart) break;
                    bool told = false, spread = false;
                    int rc = probe_spread(s, *o, &told, &spread);
                    // a slab is placed for the life of its buffers: what speaks for it is measured twice
                    if (rc == BCAST_OK && told && spread) rc = probe_spread(s, *o, &told, &spread);
                    if (rc != BCAST_OK) {
                        release(true);
                        return rc;
                    }
                    any_told = any_told || told;
                    if (told && !spread) {
                        apart = false;
                        break;
                    }
                }
            }
            if (apart) break;
            if (last) {
                any_failed = true;  // taken where it fell
                break;
            }
            aside.push_back(s.base);  // the wrong region (or not looked at): kept, so that the next allocation is other memory
            s.base = nullptr;
        }
    }
    release(false);

    {
        std::lock_guard<std::mutex> g(g_mu);
        for (const Slab &s : slabs) {
            g_live[s.base] = (int)s.members.size();
            for (size_t m = 0; m < s.members.size(); ++m) {
                ptrs[s.members[m]] = s.base + s.offset[m];
                g_slab_of[ptrs[s.members[m]]] = s.base;
            }
        }
    }
    if (placed) *placed = any_failed ? BCAST_PLACED_NO : (labels_used > 1 && any_told) ? BCAST_PLACED_MEASURED : BCAST_PLACED_BY_ORDER;
    return BCAST_OK;
}

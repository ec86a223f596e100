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
// HIP has no call that allocates at a physical address.  What it does have is
// an allocator that, while the device's memory is not fragmented, hands memory
// out in address order from one end; hipMemGetInfo tells how far it has come.
// bcast_buffers_alloc uses that: it allocates the buffers region by region and,
// between two regions, a temporary filler that pushes the allocator past the
// boundary (plus a margin for what the accounting does not show); the fillers
// are freed before it returns.  The placement is then confirmed by measurement:
// writing to memory on both sides of a boundary together must be clearly faster
// than writing to one side alone -- measured on the fillers next to the groups
// and, where they are large enough (their writes must exceed the memory-side
// cache by far), on the groups themselves.
#include <algorithm>
#include <cstring>
#include <vector>

#include "bcast_internal.h"

using namespace bcast;

namespace {

constexpr int kRegionCount = 3;
constexpr size_t kGiB = (size_t)1 << 30;
constexpr size_t kAllocUnit = (size_t)2 << 20;     // allocations are accounted in 2 MiB units
constexpr size_t kBoundaryMargin = 10 * kGiB;      // how far past a boundary the next group starts
constexpr size_t kFillerPiece = kGiB;              // fillers are allocated in pieces of this size
constexpr size_t kProbePieces = 8;                 // filler pieces on either side of a boundary that a probe writes to
constexpr size_t kProbeMinBytes = 2 * kGiB;        // a probe must write more than the memory-side cache holds (256 MiB), by a wide margin
constexpr size_t kProbeWindowMax = (size_t)256 << 20;
static_assert(kProbeWindowMax <= kFillerPiece, "a probe writes at most one filler piece's size into a piece");
constexpr double kProbeGain = 1.08;                // both sides of a boundary together vs the slower side alone: measured 1.18-1.20
constexpr double kSpreadRateGBps = 6500.0;         // store-only rate: 5800-6000 GB/s into one region, 6900-7200 over two (measured)

size_t round_up_unit(size_t n) { return (n + kAllocUnit - 1) / kAllocUnit * kAllocUnit; }

int hip_status(hipError_t e)
{
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? BCAST_ERR_NOMEM : BCAST_ERR_HIP;
}

// A device allocation as the probes see it: they never write beyond `bytes`.
struct Span {
    void *ptr;
    size_t bytes;
};

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

// Whether writing to spans of a and b together runs at the rate of a write set
// spread over regions: clearly faster, byte for byte, than writing to the slower
// of the two alone, or at the spread rate outright.  *told is false if the sets are
// too small to tell (the writes must exceed the memory-side cache by far).
int probe_spread(const std::vector<Span> &in_a, const std::vector<Span> &in_b, bool *told, bool *spread)
{
    *told = *spread = false;
    const size_t each = std::min<size_t>({in_a.size(), in_b.size(), (size_t)BCAST_MAX_RANKS / 2});
    if (each == 0) return BCAST_OK;
    std::vector<Span> a(in_a.begin(), in_a.begin() + each), b(in_b.begin(), in_b.begin() + each), both(a);
    both.insert(both.end(), b.begin(), b.end());
    size_t window = kProbeWindowMax;
    for (const Span &s : both) window = std::min(window, s.bytes);  // no span is written beyond its size
    window = window / (size_t)kTileBytes * (size_t)kTileBytes;
    if (window == 0 || 2 * each * window < kProbeMinBytes) return BCAST_OK;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return BCAST_ERR_HIP;
    }
    float t_a = 0.f, t_b = 0.f, t_both = 0.f;
    int rc = time_store_pattern(a, window, e0, e1, &t_a);
    if (rc == BCAST_OK) rc = time_store_pattern(b, window, e0, e1, &t_b);
    if (rc == BCAST_OK) rc = time_store_pattern(both, window, e0, e1, &t_both);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != BCAST_OK) return rc;
    *told = true;
    // `both` writes twice the bytes of either alone.  Spread: clearly faster than
    // the slower of the two alone -- or as fast as only writes over more than one
    // region are (where earlier allocations and frees have scattered a group over
    // the regions already, it is no slower alone than together with the other)
    const double gain = 2.0 * std::max(t_a, t_b) / t_both;
    const double rate_gbps = 2.0 * (double)each * (double)window / (t_both * 1e-3) / 1e9;
    *spread = gain >= kProbeGain || rate_gbps >= kSpreadRateGBps;
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
    for (int i = 0; i < n; ++i)
        if (ptrs[i]) {
            hipError_t e = hipFree(ptrs[i]);
            if (e != hipSuccess) rc = hip_status(e);
        }
    return rc;
}

extern "C" int bcast_buffers_alloc(int n, const size_t *bytes, const int *region, void **ptrs, int *placed)
{
    if (n < 1 || n > (1 << 16) || !bytes || !region || !ptrs) return BCAST_ERR_ARG;
    int top = 0;
    for (int i = 0; i < n; ++i) {
        if (bytes[i] == 0 || region[i] < 0 || region[i] >= kRegionCount) return BCAST_ERR_ARG;
        top = std::max(top, region[i]);
        ptrs[i] = nullptr;
    }
    if (placed) *placed = BCAST_PLACED_NO;

    size_t free_bytes = 0, total = 0;
    hipError_t e = hipMemGetInfo(&free_bytes, &total);
    if (e != hipSuccess) return hip_status(e);
    const size_t third = total / kRegionCount;
    const size_t used_now = total - free_bytes;
    const size_t here = used_now / third;  // the third the allocator is handing out now

    // Region 0 of the request is that third if its group still fits there (clear
    // of the next boundary), else the next one.  Can every region asked for be
    // reached from there, fillers and margins included?
    size_t group_bytes[kRegionCount] = {0, 0, 0};
    for (int i = 0; i < n; ++i) group_bytes[region[i]] += round_up_unit(bytes[i]);
    const bool fits_here = used_now - here * third + group_bytes[0] + kBoundaryMargin / 2 <= third;
    const size_t first = fits_here ? here : here + 1;
    bool arrange = first + (size_t)top < (size_t)kRegionCount;
    for (int r = 0; r <= top && arrange; ++r)
        if (group_bytes[r] + 2 * kBoundaryMargin > third) arrange = false;  // a group must fit inside its third
    if (arrange && (first != here || top > 0)) {
        const size_t end = (first + (size_t)top) * third + kBoundaryMargin + group_bytes[top];
        if (end + kGiB > total) arrange = false;
    }

    std::vector<void *> fillers;
    auto release = [&](bool buffers_too) {
        for (void *f : fillers) (void)hipFree(f);
        fillers.clear();
        if (buffers_too)
            for (int i = 0; i < n; ++i)
                if (ptrs[i]) {
                    (void)hipFree(ptrs[i]);
                    ptrs[i] = nullptr;
                }
    };

    bool arranged = arrange;
    bool any_told = false, any_flat = false;
    for (int r = 0; r <= top; ++r) {
        if (arranged && (r > 0 || first != here)) {
            // push the allocator to kBoundaryMargin past the start of third first + r,
            // in pieces of 1 GiB: equal, moderate allocations are what the allocator
            // hands out in order (one huge block it may take from anywhere)
            e = hipMemGetInfo(&free_bytes, &total);
            if (e != hipSuccess) {
                release(true);
                return hip_status(e);
            }
            size_t used = total - free_bytes;
            const size_t target = (first + (size_t)r) * third + kBoundaryMargin;
            const size_t run_begin = fillers.size();
            while (arranged && used < target) {
                // every piece has the full size (the last one overshoots the target by less
                // than a piece): the probe below writes kProbeWindowMax bytes into pieces
                void *filler = nullptr;
                e = hipMalloc(&filler, kFillerPiece);
                if (e == hipSuccess) {
                    fillers.push_back(filler);
                    used += kFillerPiece;
                } else {
                    (void)hipGetLastError();
                    arranged = false;  // no room for the fillers: the rest is allocated where it falls
                }
            }
            // The pieces right after the group before and the pieces just allocated lie
            // on either side of the boundary if the allocator works as assumed: measure it
            // (whole pieces of 1 GiB each, so any set, however small, gets its placement checked).
            const size_t run = fillers.size() - run_begin;
            if (arranged && run >= 2 * kProbePieces + kBoundaryMargin / kFillerPiece) {
                std::vector<Span> before, after;
                for (size_t k = 0; k < kProbePieces; ++k) {
                    before.push_back(Span{fillers[run_begin + k], kFillerPiece});
                    after.push_back(Span{fillers[fillers.size() - kProbePieces + k], kFillerPiece});
                }
                bool told = false, spread = false;
                int rc = probe_spread(before, after, &told, &spread);
                if (rc != BCAST_OK) {
                    release(true);
                    return rc;
                }
                any_told = any_told || told;
                any_flat = any_flat || (told && !spread);
            }
        }
        for (int i = 0; i < n; ++i) {
            if (region[i] != r) continue;
            e = hipMalloc(&ptrs[i], bytes[i]);
            if (e != hipSuccess) {
                release(true);
                return hip_status(e);
            }
        }
    }
    release(false);
    if (!arranged) return BCAST_OK;

    // and the groups themselves, wherever two neighbouring ones are large enough to tell
    for (int r = 0; r + 1 <= top && !any_flat; ++r) {
        std::vector<Span> a, b;
        for (int i = 0; i < n; ++i) {
            if (region[i] != r && region[i] != r + 1) continue;
            (region[i] == r ? a : b).push_back(Span{ptrs[i], bytes[i]});
        }
        if (a.empty() || b.empty()) continue;
        bool told = false, spread = false;
        int rc = probe_spread(a, b, &told, &spread);
        if (rc != BCAST_OK) {
            release(true);
            return rc;
        }
        any_told = any_told || told;
        any_flat = any_flat || (told && !spread);
    }
    if (placed) *placed = any_flat ? BCAST_PLACED_NO : any_told ? BCAST_PLACED_MEASURED : BCAST_PLACED_BY_ORDER;
    return BCAST_OK;
}

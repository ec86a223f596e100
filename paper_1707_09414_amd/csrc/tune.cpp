// Tuning table and the sweep that fills it (Sec. III-B "Discussion", Sec. IV-B
// last paragraph: the best algorithm and chunk size are found by experiment
// per message-size range and process count, and looked up at run time).
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "bcast_internal.h"
#include "tune_table.h"

namespace bcast {

int log2_bucket(size_t bytes)
{
    int b = 0;
    while (bytes > 1) { bytes >>= 1; ++b; }
    return b;
}

static std::mutex g_mu;
static std::map<std::pair<int, int>, TuneEntry> g_table;  // (nranks, bucket)

}  // namespace bcast

using namespace bcast;

static bool valid_algo(int algo) { return algo >= BCAST_ALGO_CHAIN && algo <= BCAST_ALGO_FANOUT; }

extern "C" int bcast_tune_clear(void)
{
    std::lock_guard<std::mutex> g(g_mu);
    g_table.clear();
    return BCAST_OK;
}

extern "C" int bcast_tune_count(void)
{
    std::lock_guard<std::mutex> g(g_mu);
    return (int)g_table.size();
}

extern "C" int bcast_tune_set(int nranks, size_t bytes, int algo, size_t chunk_bytes, double usec)
{
    if (nranks < 1 || nranks > BCAST_MAX_RANKS || !valid_algo(algo) || bytes == 0) return BCAST_ERR_ARG;
    if (algo == BCAST_ALGO_CHAIN && (chunk_bytes == 0 || chunk_bytes % 16 != 0)) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    TuneEntry &e = g_table[{nranks, log2_bucket(bytes)}];
    e.algo = algo;
    e.chunk_bytes = chunk_bytes;
    e.usec = usec;
    if (algo == BCAST_ALGO_CHAIN) {
        e.chain_chunk = chunk_bytes;
        e.chain_usec = usec;
    }
    return BCAST_OK;
}

extern "C" int bcast_tune_set_chain(int nranks, size_t bytes, size_t chunk_bytes, double usec)
{
    if (nranks < 1 || nranks > BCAST_MAX_RANKS || bytes == 0 || chunk_bytes == 0 || chunk_bytes % 16 != 0) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    auto it = g_table.find({nranks, log2_bucket(bytes)});
    if (it == g_table.end()) return BCAST_ERR_UNTUNED;  // the bucket's winner must be set first
    it->second.chain_chunk = chunk_bytes;
    it->second.chain_usec = usec;
    return BCAST_OK;
}

// nearest bucket at or below, else the nearest above, among this nranks' entries
// (caller holds g_mu)
static const TuneEntry *nearest(int nranks, size_t bytes)
{
    const int want = log2_bucket(bytes);
    auto it = g_table.upper_bound({nranks, want});
    if (it != g_table.begin()) {
        auto below = std::prev(it);
        if (below->first.first == nranks) return &below->second;
    }
    if (it != g_table.end() && it->first.first == nranks) return &it->second;
    return nullptr;
}

extern "C" int bcast_tune_lookup(int nranks, size_t bytes, int *algo, size_t *chunk_bytes, double *usec)
{
    if (!algo || !chunk_bytes || nranks < 1 || nranks > BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    const TuneEntry *best = nearest(nranks, bytes);
    if (!best) return BCAST_ERR_UNTUNED;
    *algo = best->algo;
    *chunk_bytes = best->chunk_bytes;
    if (usec) *usec = best->usec;
    return BCAST_OK;
}

extern "C" int bcast_tune_lookup_chain(int nranks, size_t bytes, size_t *chunk_bytes, double *usec)
{
    if (!chunk_bytes || nranks < 1 || nranks > BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    const TuneEntry *best = nearest(nranks, bytes);
    if (!best || best->chain_chunk == 0) return BCAST_ERR_UNTUNED;
    *chunk_bytes = best->chain_chunk;
    if (usec) *usec = best->chain_usec;
    return BCAST_OK;
}

// Text format, one entry per line:
//   nranks log2_bytes algo chunk_bytes usec [chain_chunk_bytes chain_usec]
// Lines starting with '#' are comments.
static const char kHeaderLine[] =
    "# nranks log2_bytes algo(1=chain 2=direct 3=binomial 4=fanout) chunk_bytes usec chain_chunk_bytes chain_usec\n";

extern "C" int bcast_tune_save(const char *path)
{
    if (!path) return BCAST_ERR_ARG;
    FILE *f = fopen(path, "w");
    if (!f) return BCAST_ERR_ARG;
    fprintf(f, "%s", kHeaderLine);
    std::lock_guard<std::mutex> g(g_mu);
    for (const auto &kv : g_table)
        fprintf(f, "%d %d %d %zu %.3f %zu %.3f\n", kv.first.first, kv.first.second, kv.second.algo,
                kv.second.chunk_bytes, kv.second.usec, kv.second.chain_chunk, kv.second.chain_usec);
    fclose(f);
    return BCAST_OK;
}

extern "C" int bcast_tune_load(const char *path)
{
    if (!path) return BCAST_ERR_ARG;
    FILE *f = fopen(path, "r");
    if (!f) return BCAST_ERR_ARG;
    char line[256];
    int rc = BCAST_OK;
    std::vector<std::pair<std::pair<int, int>, TuneEntry>> rows;
    while (fgets(line, sizeof line, f)) {
        const char *s = line;
        while (*s == ' ' || *s == '\t') ++s;
        if (*s == '#' || *s == '\n' || *s == '\0') continue;
        int nranks, bucket, algo;
        unsigned long long chunk, cchunk = 0;
        double usec = 0.0, cusec = 0.0;
        int got = sscanf(s, "%d %d %d %llu %lf %llu %lf", &nranks, &bucket, &algo, &chunk, &usec, &cchunk, &cusec);
        if (got < 4 || nranks < 1 || nranks > BCAST_MAX_RANKS || bucket < 0 || bucket > 62 || !valid_algo(algo) ||
            (algo == BCAST_ALGO_CHAIN && (chunk == 0 || chunk % 16 != 0)) || cchunk % 16 != 0) {
            rc = BCAST_ERR_ARG;
            break;
        }
        if (algo == BCAST_ALGO_CHAIN && cchunk == 0) { cchunk = chunk; cusec = usec; }
        rows.push_back({{nranks, bucket}, TuneEntry{algo, (size_t)chunk, usec, (size_t)cchunk, cusec}});
    }
    fclose(f);
    if (rc != BCAST_OK) return rc;  // a malformed file installs nothing
    std::lock_guard<std::mutex> g(g_mu);
    for (const auto &r : rows) g_table[r.first] = r.second;
    return BCAST_OK;
}

namespace {

struct Scratch {
    std::vector<void *> bufs;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~Scratch()
    {
        for (void *b : bufs)
            if (b) (void)hipFree(b);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

// Microseconds per run of one candidate.  One timed run warms up and sizes
// the batches (about 20 ms each, 2..40 runs); the best of three batches counts.
int time_candidate(int nranks, size_t bytes, int algo, size_t chunk, Scratch &sc, hipStream_t stream, double *usec)
{
    bcast_plan_t *plan = nullptr;
    int rc = bcast_plan_create(&plan, nranks, bytes, chunk, algo);
    if (rc != BCAST_OK) return rc;
    int reps = 1;
    double best = 1e30;
    for (int batch = 0; batch < 4 && rc == BCAST_OK; ++batch) {
        if (hipEventRecord(sc.e0, stream) != hipSuccess) { rc = BCAST_ERR_HIP; break; }
        for (int i = 0; i < reps && rc == BCAST_OK; ++i) rc = bcast_run(plan, sc.bufs.data(), 0, bytes, stream);
        if (rc != BCAST_OK) break;
        if (hipEventRecord(sc.e1, stream) != hipSuccess || hipEventSynchronize(sc.e1) != hipSuccess) { rc = BCAST_ERR_HIP; break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sc.e0, sc.e1) != hipSuccess) { rc = BCAST_ERR_HIP; break; }
        const double us = (double)ms * 1000.0 / reps;
        if (batch == 0)
            reps = (int)std::min(40.0, std::max(2.0, 20000.0 / std::max(us, 1.0)));
        else
            best = std::min(best, us);
    }
    if (rc == BCAST_OK && bcast_plan_status(plan, nullptr) != BCAST_OK) rc = BCAST_ERR_TIMEOUT;
    int rd = bcast_plan_destroy(plan);
    if (rc == BCAST_OK) rc = rd;
    *usec = best;
    return rc;
}

}  // namespace

extern "C" int bcast_tune(int nranks, size_t min_bytes, size_t max_bytes, unsigned algo_mask,
                          bcast_stream_t stream, const char *table_path)
{
    if (nranks < 2 || nranks > BCAST_MAX_RANKS || min_bytes == 0 || max_bytes < min_bytes) return BCAST_ERR_ARG;
    if (algo_mask == 0) algo_mask = (1u << BCAST_ALGO_CHAIN) | (1u << BCAST_ALGO_DIRECT) | (1u << BCAST_ALGO_BINOMIAL);

    Scratch sc;
    sc.bufs.assign(nranks, nullptr);
    for (int r = 0; r < nranks; ++r) {
        hipError_t e = hipMalloc(&sc.bufs[r], max_bytes);
        if (e == hipSuccess) e = hipMemset(sc.bufs[r], r == 0 ? 0x5a : 0xff, max_bytes);
        if (e != hipSuccess) return e == hipErrorOutOfMemory ? BCAST_ERR_NOMEM : BCAST_ERR_HIP;
    }
    if (hipEventCreate(&sc.e0) != hipSuccess || hipEventCreate(&sc.e1) != hipSuccess) return BCAST_ERR_HIP;

    FILE *f = nullptr;
    if (table_path) {
        f = fopen(table_path, "a");
        if (!f) return BCAST_ERR_ARG;
        fprintf(f, "%s", kHeaderLine);
    }

    int rc = BCAST_OK;
    size_t M = (size_t)1 << log2_bucket(min_bytes);
    if (M < min_bytes) M <<= 1;
    for (; M <= max_bytes && rc == BCAST_OK; M <<= 1) {
        TuneEntry best{0, 0, 1e30, 0, 1e30};
        auto consider = [&](int algo, size_t chunk) {
            if (rc != BCAST_OK || !(algo_mask & (1u << algo))) return;
            double us = 0.0;
            rc = time_candidate(nranks, M, algo, chunk, sc, stream, &us);
            if (rc != BCAST_OK) return;
            if (algo == BCAST_ALGO_CHAIN && us < best.chain_usec) {
                best.chain_chunk = chunk;
                best.chain_usec = us;
            }
            if (us < best.usec) {
                best.algo = algo;
                best.chunk_bytes = chunk;
                best.usec = us;
            }
        };
        // chain: the whole message as one chunk (Eq. 2), then every power-of-two
        // chunk size from 8 KiB to 64 MiB that splits the message into at most
        // 4096 chunks (Eq. 5); smaller chunks than that only add hand-offs
        consider(BCAST_ALGO_CHAIN, std::max<size_t>(16, (M + 15) / 16 * 16));
        for (size_t C = 8u << 10; C <= (64u << 20) && C < M; C <<= 1)
            if (M / C <= 4096) consider(BCAST_ALGO_CHAIN, C);
        consider(BCAST_ALGO_DIRECT, 0);
        consider(BCAST_ALGO_BINOMIAL, 0);
        consider(BCAST_ALGO_FANOUT, 0);
        if (rc != BCAST_OK) break;
        rc = bcast_tune_set(nranks, M, best.algo, best.chunk_bytes, best.usec);
        if (rc == BCAST_OK && best.chain_chunk) rc = bcast_tune_set_chain(nranks, M, best.chain_chunk, best.chain_usec);
        if (f) fprintf(f, "%d %d %d %zu %.3f %zu %.3f\n", nranks, log2_bucket(M), best.algo, best.chunk_bytes, best.usec,
                       best.chain_chunk, best.chain_chunk ? best.chain_usec : 0.0);
        if (M > (max_bytes >> 1)) break;  // next doubling would overflow or pass max
    }
    if (f) fclose(f);
    return rc;
}

// Tuning table and the sweep that fills it (Sec. III-B "Discussion", Sec. IV-B
// last paragraph: the best algorithm and chunk size are found by experiment
// per message-size range and process count, and looked up at run time).
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <climits>
#include <map>
#include <mutex>
#include <string>
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
static std::map<std::pair<int, int>, bcast_tune_entry_t> g_table;  // (nranks, bucket)
static std::map<std::pair<int, int>, bcast_reduce_entry_t> g_reduce_table;  // the reduction's own entries
static std::string g_log_path;  // if set, bcast_tune appends every candidate it times

}  // namespace bcast

using namespace bcast;

static bool valid_algo(int algo) { return algo >= BCAST_ALGO_CHAIN && algo <= BCAST_ALGO_KNOMIAL_PIPELINED; }
static bool has_radix(int algo) { return algo == BCAST_ALGO_KNOMIAL || algo == BCAST_ALGO_KNOMIAL_PIPELINED; }

static bool valid_entry(int nranks, const bcast_tune_entry_t &e)
{
    if (nranks < 1 || nranks > BCAST_MAX_RANKS || !valid_algo(e.algo)) return false;
    const bool chunked = e.algo == BCAST_ALGO_CHAIN || e.algo == BCAST_ALGO_KNOMIAL_PIPELINED;
    if (chunked && (e.chunk_bytes == 0 || e.chunk_bytes % 16 != 0)) return false;
    if (e.chain_chunk_bytes % 16 != 0) return false;
    if (e.stages < 0 || e.stages > BCAST_MAX_RANKS || e.chain_stages < 0 || e.chain_stages > BCAST_MAX_RANKS) return false;
    if ((e.rank_waves != 0 && e.rank_waves != 1) || (e.chain_rank_waves != 0 && e.chain_rank_waves != 1)) return false;
    // trip sizes: those the chain kernel of the entry's wave mode is built for
    auto trip_ok = [](int t, int rank_waves) {
        if (t == 0) return true;
        if (t % 1024 != 0) return false;
        const int u = t / 1024;
        return rank_waves ? (u == 1 || u == 2 || u == 3 || u == 4 || u == 6 || u == 8) : valid_chain_unroll(u);
    };
    if (!trip_ok(e.trip_bytes, e.rank_waves) || !trip_ok(e.chain_trip_bytes, e.chain_rank_waves)) return false;
    if (e.rank_waves && e.algo != BCAST_ALGO_CHAIN) return false;
    if (e.stage_store < BCAST_STORE_AUTO || e.stage_store > BCAST_STORE_BACK) return false;
    if (e.chain_stage_store < BCAST_STORE_AUTO || e.chain_stage_store > BCAST_STORE_BACK) return false;
    if (e.stage_store != BCAST_STORE_AUTO && e.algo != BCAST_ALGO_CHAIN) return false;
    // lanes belong to the chain (either kernel), spans to the chain with a wavefront per stage
    if (e.lanes < 0 || e.lanes > 8192 || e.chain_lanes < 0 || e.chain_lanes > 8192) return false;
    if (e.spans < BCAST_SPANS_AUTO || e.spans > BCAST_SPANS_ROTATE || e.chain_spans < BCAST_SPANS_AUTO || e.chain_spans > BCAST_SPANS_ROTATE)
        return false;
    if ((e.lanes != 0 || e.spans != BCAST_SPANS_AUTO) && e.algo != BCAST_ALGO_CHAIN) return false;
    if ((e.spans != BCAST_SPANS_AUTO && e.rank_waves) || (e.chain_spans != BCAST_SPANS_AUTO && e.chain_rank_waves)) return false;
    return true;
}

extern "C" int bcast_tune_clear(void)
{
    std::lock_guard<std::mutex> g(g_mu);
    g_table.clear();
    g_reduce_table.clear();
    return BCAST_OK;
}

extern "C" int bcast_tune_count(void)
{
    std::lock_guard<std::mutex> g(g_mu);
    return (int)g_table.size();
}

extern "C" int bcast_tune_set_log(const char *path)
{
    std::lock_guard<std::mutex> g(g_mu);
    g_log_path = path ? path : "";
    return BCAST_OK;
}

extern "C" int bcast_tune_put(int nranks, size_t bytes, const bcast_tune_entry_t *entry)
{
    if (!entry || bytes == 0 || !valid_entry(nranks, *entry)) return BCAST_ERR_ARG;
    bcast_tune_entry_t e = *entry;
    if (e.algo == BCAST_ALGO_CHAIN && e.chain_chunk_bytes == 0) {  // the winner is the chain: it is its own best
        e.chain_chunk_bytes = e.chunk_bytes;
        e.chain_stages = e.stages;
        e.chain_trip_bytes = e.trip_bytes;
        e.chain_usec = e.usec;
        e.chain_rank_waves = e.rank_waves;
        e.chain_stage_store = e.stage_store;
        e.chain_lanes = e.lanes;
        e.chain_spans = e.spans;
    }
    std::lock_guard<std::mutex> g(g_mu);
    g_table[{nranks, log2_bucket(bytes)}] = e;
    return BCAST_OK;
}

// nearest bucket at or below, else the nearest above, among one rank count's entries
// (caller holds g_mu)
static const bcast_tune_entry_t *nearest_size(int nranks, size_t bytes)
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

// The entry for (nranks, bytes): this rank count's if it has any, else that of
// the measured rank count closest to it in ratio (the larger one on a tie) --
// tables are measured for a few process counts and serve the ranges between
// them (Sec. III-B).  (caller holds g_mu)
static const bcast_tune_entry_t *nearest(int nranks, size_t bytes)
{
    if (const bcast_tune_entry_t *e = nearest_size(nranks, bytes)) return e;
    int best = 0;
    for (auto it = g_table.begin(); it != g_table.end(); it = g_table.upper_bound({it->first.first, INT_MAX})) {
        const int n = it->first.first;
        // n is closer than best if max(n, nranks) / min(n, nranks) is smaller
        auto closer = [&](int a, int b) {
            const long long ra_num = std::max(a, nranks), ra_den = std::min(a, nranks);
            const long long rb_num = std::max(b, nranks), rb_den = std::min(b, nranks);
            return ra_num * rb_den < rb_num * ra_den || (ra_num * rb_den == rb_num * ra_den && a > b);
        };
        if (best == 0 || closer(n, best)) best = n;
    }
    return best ? nearest_size(best, bytes) : nullptr;
}

static bool valid_reduce_entry(int nranks, const bcast_reduce_entry_t &e)
{
    if (nranks < 2 || nranks > BCAST_MAX_RANKS) return false;
    if (e.chunk_bytes == 0 || e.chunk_bytes % 16 != 0) return false;
    if (e.stages < 1 || e.stages > BCAST_MAX_RANKS) return false;
    return e.trip_bytes == 4096 || e.trip_bytes == 1024;
}

extern "C" int bcast_tune_reduce_put(int nranks, size_t bytes, const bcast_reduce_entry_t *entry)
{
    if (!entry || bytes == 0 || !valid_reduce_entry(nranks, *entry)) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    g_reduce_table[{nranks, log2_bucket(bytes)}] = *entry;
    return BCAST_OK;
}

extern "C" int bcast_tune_reduce_get(int nranks, size_t bytes, bcast_reduce_entry_t *entry)
{
    if (!entry || nranks < 1 || nranks > BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    // this rank count's nearest bucket at or below, else the nearest above; no
    // borrowing from other rank counts (a reduction's best stage count depends on it)
    const int want = log2_bucket(bytes);
    auto it = g_reduce_table.upper_bound({nranks, want});
    if (it != g_reduce_table.begin()) {
        auto below = std::prev(it);
        if (below->first.first == nranks) {
            *entry = below->second;
            return BCAST_OK;
        }
    }
    if (it != g_reduce_table.end() && it->first.first == nranks) {
        *entry = it->second;
        return BCAST_OK;
    }
    return BCAST_ERR_UNTUNED;
}

extern "C" int bcast_tune_get(int nranks, size_t bytes, bcast_tune_entry_t *entry)
{
    if (!entry || nranks < 1 || nranks > BCAST_MAX_RANKS) return BCAST_ERR_ARG;
    std::lock_guard<std::mutex> g(g_mu);
    const bcast_tune_entry_t *best = nearest(nranks, bytes);
    if (!best) return BCAST_ERR_UNTUNED;
    *entry = *best;
    return BCAST_OK;
}

extern "C" int bcast_tune_set(int nranks, size_t bytes, int algo, size_t chunk_bytes, double usec)
{
    bcast_tune_entry_t e;
    memset(&e, 0, sizeof e);
    e.algo = algo;
    e.chunk_bytes = chunk_bytes;
    e.usec = usec;
    return bcast_tune_put(nranks, bytes, &e);
}

extern "C" int bcast_tune_lookup(int nranks, size_t bytes, int *algo, size_t *chunk_bytes, double *usec)
{
    if (!algo || !chunk_bytes) return BCAST_ERR_ARG;
    bcast_tune_entry_t e;
    int rc = bcast_tune_get(nranks, bytes, &e);
    if (rc != BCAST_OK) return rc;
    *algo = e.algo;
    *chunk_bytes = (size_t)e.chunk_bytes;
    if (usec) *usec = e.usec;
    return BCAST_OK;
}

static const char kHeaderLine[] =
    "# nranks log2_bytes algo(1=chain 2=direct 3=binomial 4=fanout 5=scatter-allgather 6=knomial 7=pipelined-knomial) chunk_bytes usec "
    "chain_chunk_bytes chain_usec stages chain_stages trip_bytes chain_trip_bytes rank_waves chain_rank_waves "
    "stage_store(0=rule 1=through 2=back) chain_stage_store lanes(0=from the chunk) chain_lanes spans(0=rule 1=fixed 2=rotate) chain_spans\n";

// Text format, one entry per line (columns after usec are optional; for a
// k-nomial winner the stages column holds the radix):
//   nranks log2_bytes algo chunk_bytes usec [chain_chunk_bytes chain_usec [stages chain_stages
//   [trip_bytes chain_trip_bytes [rank_waves chain_rank_waves [stage_store chain_stage_store
//   [lanes chain_lanes spans chain_spans]]]]]]
// Lines starting with '#' are comments.
static void print_entry(FILE *f, int nranks, int bucket, const bcast_tune_entry_t &e)
{
    fprintf(f, "%d %d %d %llu %.3f %llu %.3f %d %d %d %d %d %d %d %d %d %d %d %d\n", nranks, bucket, e.algo,
            (unsigned long long)e.chunk_bytes, e.usec, (unsigned long long)e.chain_chunk_bytes, e.chain_usec, e.stages, e.chain_stages,
            e.trip_bytes, e.chain_trip_bytes, e.rank_waves, e.chain_rank_waves, e.stage_store, e.chain_stage_store, e.lanes,
            e.chain_lanes, e.spans, e.chain_spans);
}

static const char kReduceHeaderLine[] = "# reduce nranks log2_bytes chunk_bytes stages trip_bytes usec   (the chain reduction's own entries)\n";

static void print_reduce_entry(FILE *f, int nranks, int bucket, const bcast_reduce_entry_t &e)
{
    fprintf(f, "reduce %d %d %llu %d %d %.3f\n", nranks, bucket, (unsigned long long)e.chunk_bytes, e.stages, e.trip_bytes, e.usec);
}

extern "C" int bcast_tune_save(const char *path)
{
    if (!path) return BCAST_ERR_ARG;
    FILE *f = fopen(path, "w");
    if (!f) return BCAST_ERR_ARG;
    fprintf(f, "%s", kHeaderLine);
    std::lock_guard<std::mutex> g(g_mu);
    for (const auto &kv : g_table) print_entry(f, kv.first.first, kv.first.second, kv.second);
    if (!g_reduce_table.empty()) fprintf(f, "%s", kReduceHeaderLine);
    for (const auto &kv : g_reduce_table) print_reduce_entry(f, kv.first.first, kv.first.second, kv.second);
    fclose(f);
    return BCAST_OK;
}

extern "C" int bcast_tune_load(const char *path)
{
    if (!path) return BCAST_ERR_ARG;
    FILE *f = fopen(path, "r");
    if (!f) return BCAST_ERR_ARG;
    char line[1024];  // longer than the header line that bcast_tune_save writes
    int rc = BCAST_OK;
    std::vector<std::pair<std::pair<int, int>, bcast_tune_entry_t>> rows;
    std::vector<std::pair<std::pair<int, int>, bcast_reduce_entry_t>> reduce_rows;
    while (fgets(line, sizeof line, f)) {
        const char *s = line;
        while (*s == ' ' || *s == '\t') ++s;
        if (*s == '#' || *s == '\n' || *s == '\0') continue;
        if (strncmp(s, "reduce ", 7) == 0) {
            int nranks, bucket;
            unsigned long long chunk = 0;
            bcast_reduce_entry_t e;
            memset(&e, 0, sizeof e);
            int got = sscanf(s + 7, "%d %d %llu %d %d %lf", &nranks, &bucket, &chunk, &e.stages, &e.trip_bytes, &e.usec);
            e.chunk_bytes = chunk;
            if (got < 5 || bucket < 0 || bucket > 62 || !valid_reduce_entry(nranks, e)) {
                rc = BCAST_ERR_ARG;
                break;
            }
            reduce_rows.push_back({{nranks, bucket}, e});
            continue;
        }
        int nranks, bucket;
        unsigned long long chunk = 0, cchunk = 0;
        bcast_tune_entry_t e;
        memset(&e, 0, sizeof e);
        int got = sscanf(s, "%d %d %d %llu %lf %llu %lf %d %d %d %d %d %d %d %d %d %d %d %d", &nranks, &bucket, &e.algo, &chunk, &e.usec,
                         &cchunk, &e.chain_usec, &e.stages, &e.chain_stages, &e.trip_bytes, &e.chain_trip_bytes, &e.rank_waves,
                         &e.chain_rank_waves, &e.stage_store, &e.chain_stage_store, &e.lanes, &e.chain_lanes, &e.spans, &e.chain_spans);
        e.chunk_bytes = chunk;
        e.chain_chunk_bytes = cchunk;
        if (got < 4 || bucket < 0 || bucket > 62 || !valid_entry(nranks, e)) {
            rc = BCAST_ERR_ARG;
            break;
        }
        if (e.algo == BCAST_ALGO_CHAIN && e.chain_chunk_bytes == 0) {
            e.chain_chunk_bytes = e.chunk_bytes;
            e.chain_stages = e.stages;
            e.chain_trip_bytes = e.trip_bytes;
            e.chain_usec = e.usec;
            e.chain_rank_waves = e.rank_waves;
            e.chain_stage_store = e.stage_store;
            e.chain_lanes = e.lanes;
            e.chain_spans = e.spans;
        }
        rows.push_back({{nranks, bucket}, e});
    }
    fclose(f);
    if (rc != BCAST_OK) return rc;  // a malformed file installs nothing
    std::lock_guard<std::mutex> g(g_mu);
    for (const auto &r : rows) g_table[r.first] = r.second;
    for (const auto &r : reduce_rows) g_reduce_table[r.first] = r.second;
    return BCAST_OK;
}

namespace {

struct Scratch {
    std::vector<void *> bufs;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~Scratch()
    {
        if (!bufs.empty()) (void)bcast_buffers_free((int)bufs.size(), bufs.data());  // they come from bcast_buffers_alloc
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

// Microseconds per run of one candidate.  One timed run warms up and sizes
// the batches (about 20 ms each, 2..40 runs); the best of three batches counts.
int time_candidate(int nranks, size_t bytes, int algo, size_t chunk, int stages, int trip, int rank_waves, int stage_store,
                   int lanes, int spans, Scratch &sc, hipStream_t stream, double *usec)
{
    bcast_plan_t *plan = nullptr;
    int rc = bcast_plan_create(&plan, nranks, bytes, chunk, algo);
    if (rc != BCAST_OK) return rc;
    rc = has_radix(algo) ? bcast_plan_set_radix(plan, stages) : bcast_plan_set_stages(plan, stages);
    if (rc == BCAST_OK && algo == BCAST_ALGO_CHAIN) rc = bcast_plan_set_trip(plan, trip);
    if (rc == BCAST_OK && algo == BCAST_ALGO_CHAIN)
        rc = bcast_plan_set_chain_waves(plan, rank_waves ? BCAST_CHAIN_WAVE_PER_RANK : BCAST_CHAIN_WAVE_PER_STAGE);
    if (rc == BCAST_OK && algo == BCAST_ALGO_CHAIN) rc = bcast_plan_set_stage_store(plan, stage_store);
    if (rc == BCAST_OK && algo == BCAST_ALGO_CHAIN && lanes > 0) rc = bcast_plan_set_lanes(plan, lanes);
    if (rc == BCAST_OK && algo == BCAST_ALGO_CHAIN && spans != BCAST_SPANS_AUTO)
        rc = bcast_plan_set_mode(plan, spans == BCAST_SPANS_ROTATE ? BCAST_MODE_ROTATE_SPANS : BCAST_MODE_FIXED_SPANS);
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
    if ((algo_mask & ~(BCAST_TUNE_FOLDED | BCAST_TUNE_NO_RANK_WAVES)) == 0)
        algo_mask |= (1u << BCAST_ALGO_CHAIN) | (1u << BCAST_ALGO_DIRECT) | (1u << BCAST_ALGO_BINOMIAL);

    // rank buffers placed as the library recommends for a broadcast: the two halves
    // of the chain in two regions of the device's memory (see memory.cpp)
    Scratch sc;
    sc.bufs.assign(nranks, nullptr);
    {
        std::vector<size_t> sizes(nranks, max_bytes);
        std::vector<int> region(nranks, 0);
        for (int r = nranks / 2; r < nranks; ++r) region[r] = 1;
        int rc_alloc = bcast_buffers_alloc(nranks, sizes.data(), region.data(), sc.bufs.data(), nullptr);
        if (rc_alloc != BCAST_OK) return rc_alloc;
    }
    for (int r = 0; r < nranks; ++r) {
        hipError_t e = hipMemset(sc.bufs[r], r == 0 ? 0x5a : 0xff, max_bytes);
        if (e != hipSuccess) return BCAST_ERR_HIP;
    }
    if (hipEventCreate(&sc.e0) != hipSuccess || hipEventCreate(&sc.e1) != hipSuccess) return BCAST_ERR_HIP;

    FILE *log = nullptr;
    {
        std::lock_guard<std::mutex> g(g_mu);
        if (!g_log_path.empty()) log = fopen(g_log_path.c_str(), "a");
    }
    if (log) fprintf(log, "# nranks bytes algo chunk_bytes stages usec trip_bytes rank_waves stage_store lanes spans\n");
    struct LogCloser {
        FILE *f;
        ~LogCloser() { if (f) fclose(f); }
    } log_closer{log};

    FILE *f = nullptr;
    if (table_path) {
        f = fopen(table_path, "a");
        if (!f) return BCAST_ERR_ARG;
        fprintf(f, "%s", kHeaderLine);
    }

    // Stage counts to try for the chain: one stage per receiving rank (every
    // rank has wavefronts of its own), then fewer, larger stages.  A single
    // stage has no flag hand-off at all and is only tried on request.
    const int hops = nranks - 1;
    std::vector<int> stage_counts;
    for (int s : {hops, 16, 8, 4, 2, 1}) {
        if (s > hops || (s == 1 && hops > 1 && !(algo_mask & BCAST_TUNE_FOLDED))) continue;
        if (std::find(stage_counts.begin(), stage_counts.end(), s) == stage_counts.end()) stage_counts.push_back(s);
    }

    int rc = BCAST_OK;
    size_t M = (size_t)1 << log2_bucket(min_bytes);
    if (M < min_bytes) M <<= 1;
    for (; M <= max_bytes && rc == BCAST_OK; M <<= 1) {
        bcast_tune_entry_t best;
        memset(&best, 0, sizeof best);
        best.usec = best.chain_usec = 1e30;
        // the best setting of the chain with a wavefront per stage alone, and the best candidate of all but
        // the wave-per-rank chains of several stages (see the end of the sweep)
        bcast_tune_entry_t relay, runner;
        memset(&relay, 0, sizeof relay);
        memset(&runner, 0, sizeof runner);
        relay.usec = runner.usec = 1e30;
        auto consider = [&](int algo, size_t chunk, int stages, int trip = 0, int rank_waves = 0, int stage_store = BCAST_STORE_AUTO,
                            int lanes = 0, int spans = BCAST_SPANS_AUTO) {
            if (rc != BCAST_OK || !(algo_mask & (1u << algo))) return;
            double us = 0.0;
            rc = time_candidate(nranks, M, algo, chunk, stages, trip, rank_waves, stage_store, lanes, spans, sc, stream, &us);
            if (rc != BCAST_OK) return;
            if (log)
                fprintf(log, "%d %zu %d %zu %d %.3f %d %d %d %d %d\n", nranks, M, algo, chunk, stages, us, trip, rank_waves, stage_store, lanes,
                        spans);
            if (algo == BCAST_ALGO_CHAIN && !rank_waves && us < relay.usec) {
                relay.chunk_bytes = chunk;
                relay.stages = stages;
                relay.trip_bytes = trip;
                relay.stage_store = stage_store;
                relay.lanes = lanes;
                relay.spans = spans;
                relay.usec = us;
            }
            if (!(algo == BCAST_ALGO_CHAIN && rank_waves && stages >= 2) && us < runner.usec) {
                runner.algo = algo;
                runner.chunk_bytes = chunk;
                runner.stages = (algo == BCAST_ALGO_CHAIN || has_radix(algo)) ? stages : 0;
                runner.trip_bytes = algo == BCAST_ALGO_CHAIN ? trip : 0;
                runner.rank_waves = algo == BCAST_ALGO_CHAIN ? rank_waves : 0;
                runner.stage_store = algo == BCAST_ALGO_CHAIN ? stage_store : BCAST_STORE_AUTO;
                runner.lanes = algo == BCAST_ALGO_CHAIN ? lanes : 0;
                runner.spans = algo == BCAST_ALGO_CHAIN ? spans : BCAST_SPANS_AUTO;
                runner.usec = us;
            }
            if (algo == BCAST_ALGO_CHAIN && us < best.chain_usec) {
                best.chain_chunk_bytes = chunk;
                best.chain_stages = stages;
                best.chain_trip_bytes = trip;
                best.chain_rank_waves = rank_waves;
                best.chain_stage_store = stage_store;
                best.chain_lanes = lanes;
                best.chain_spans = spans;
                best.chain_usec = us;
            }
            if (us < best.usec) {
                best.algo = algo;
                best.chunk_bytes = chunk;
                best.stages = (algo == BCAST_ALGO_CHAIN || has_radix(algo)) ? stages : 0;
                best.trip_bytes = algo == BCAST_ALGO_CHAIN ? trip : 0;
                best.rank_waves = algo == BCAST_ALGO_CHAIN ? rank_waves : 0;
                best.stage_store = algo == BCAST_ALGO_CHAIN ? stage_store : BCAST_STORE_AUTO;
                best.lanes = algo == BCAST_ALGO_CHAIN ? lanes : 0;
                best.spans = algo == BCAST_ALGO_CHAIN ? spans : BCAST_SPANS_AUTO;
                best.usec = us;
            }
        };
        // chain: for every stage count, the whole message as one chunk (Eq. 2)
        // and chunk sizes lanes * trip for power-of-two lane counts (Eq. 5): a
        // chunk gives every lane one trip, so the chunk size is also the number
        // of waves that run, and that is what has an optimum (see chain_kernel).
        // 4 KiB trips span 8 KiB .. 64 MiB chunks; 3 KiB trips are only tried
        // where they can matter (messages of a few MiB and more).  At most 4096
        // chunks per message.
        for (int stages : stage_counts) {
            size_t lanes_max = 1;
            while (lanes_max * 2 * stages <= 8192) lanes_max *= 2;
            consider(BCAST_ALGO_CHAIN, std::max<size_t>(16, (M + 15) / 16 * 16), stages, 4096);
            for (int trip : {4096, 3072}) {
                if (trip == 3072 && M < (4u << 20)) continue;
                for (size_t lanes = 2; lanes <= lanes_max * 32; lanes <<= 1) {
                    const size_t C = lanes * (size_t)trip;
                    if (C >= M || M / C > 4096 || C > (64u << 20)) continue;
                    if (trip == 3072 && lanes * (size_t)stages < 512) continue;
                    consider(BCAST_ALGO_CHAIN, C, stages, trip);
                    // the same with write-back stores inside the stages where the message streams (below
                    // that the library's rule already stores write-back): the cache acknowledges them
                    // sooner, so fewer waves fill the memory system
                    if (M >= ((size_t)4 << 20) && stages <= 4 && lanes * (size_t)stages >= 256 && lanes * (size_t)stages <= 2048)
                        consider(BCAST_ALGO_CHAIN, C, stages, trip, 0, BCAST_STORE_BACK);
                }
            }
        }
        // The chain with a wavefront per rank: as few stages as 8 and as 16 ranks
        // per workgroup allow; 4 and 8 KiB trips; chunks of one trip per lane for
        // lane counts around 64 KiB of trips in flight per compute unit (the
        // library's rule), half and twice that, from 16 MiB also with several trips per
        // lane and chunk; and the whole message as one chunk.
        if (!(algo_mask & BCAST_TUNE_NO_RANK_WAVES)) {
            std::vector<int> rank_stages;
            for (int per : {8, 16}) {
                const int st = (hops + per - 1) / per;
                if (std::find(rank_stages.begin(), rank_stages.end(), st) == rank_stages.end()) rank_stages.push_back(st);
            }
            for (int stages : rank_stages) {
                const int waves = (hops + stages - 1) / stages;
                for (int trip : {4096, 8192}) {
                    consider(BCAST_ALGO_CHAIN, std::max<size_t>(16, (M + 15) / 16 * 16), stages, trip, 1);
                    size_t rule = 1;
                    while (rule * 2 * (size_t)trip * waves * stages <= ((size_t)64 << 10) * 256) rule *= 2;
                    for (size_t lanes : {rule / 2, rule, rule * 2}) {
                        const size_t C = lanes * (size_t)trip;
                        if (lanes < 1 || C >= M || M / C > 4096) continue;
                        consider(BCAST_ALGO_CHAIN, C, stages, trip, 1);
                        // messages that stream: the same lanes with 4 and 8 trips per lane and chunk (a chunk
                        // is what crosses a workgroup boundary, one flag hand-off each)
                        if (M < ((size_t)16 << 20) || stages < 2) continue;
                        for (size_t mult : {(size_t)4, (size_t)8})
                            if (C * mult < M) consider(BCAST_ALGO_CHAIN, C * mult, stages, trip, 1, BCAST_STORE_AUTO, (int)lanes);
                    }
                }
            }
        }
        // Refinement around the best staged chain of a message that streams: the same
        // lanes with several trips per lane and chunk (fewer flag hand-offs), and,
        // where the stages are unequal, the extra hop kept in place or passed round.
        if (M >= ((size_t)16 << 20) && best.chain_chunk_bytes != 0 && !best.chain_rank_waves && best.chain_trip_bytes != 0 &&
            best.chain_chunk_bytes < M) {
            const bcast_tune_entry_t base = best;
            // the lanes that setting ran with: one per trip of its chunk, up to the power of two its stage count allows
            u64 lanes_max = 1;
            while (lanes_max * 2 * (u64)base.chain_stages <= 8192) lanes_max *= 2;
            const int lanes = (int)std::min<u64>(lanes_max, base.chain_chunk_bytes / (u64)base.chain_trip_bytes);
            if (lanes >= 1 && base.chain_chunk_bytes % ((u64)lanes * (u64)base.chain_trip_bytes) == 0) {
                const bool unequal = hops % base.chain_stages != 0;
                for (int spans : {BCAST_SPANS_AUTO, BCAST_SPANS_FIXED, BCAST_SPANS_ROTATE}) {
                    if (spans != BCAST_SPANS_AUTO && !unequal) continue;
                    for (int mult : {1, 2, 4, 8}) {
                        if (mult == 1 && spans == BCAST_SPANS_AUTO) continue;  // that is `base` itself
                        const size_t C = (size_t)base.chain_chunk_bytes * mult;
                        if (C >= M) continue;
                        consider(BCAST_ALGO_CHAIN, C, base.chain_stages, base.chain_trip_bytes, 0, base.chain_stage_store, lanes, spans);
                    }
                }
            }
        }
        consider(BCAST_ALGO_DIRECT, 0, 0);
        consider(BCAST_ALGO_BINOMIAL, 0, 0);
        consider(BCAST_ALGO_FANOUT, 0, 0);
        consider(BCAST_ALGO_SCATTER_ALLGATHER, 0, 0);
        for (int k : {4, 8})
            if (k < nranks) consider(BCAST_ALGO_KNOMIAL, 0, k);  // radix travels in the stages column
        // the same trees in one launch, chunked: the whole message as one chunk,
        // and 64 KiB and 512 KiB chunks where the message is longer.  The last
        // radix is the rank count itself: the flat tree, one level, every
        // position pulls from the root (Eq. 3 with ceil(log_k n) = 1).  On one
        // die nothing serialises at the root, and measured it is the fastest
        // tree from 256 KiB to a few MiB (64 ranks, 1 MiB: 11.7 us against 14.8
        // at radix 8).
        int tried[5];
        int ntried = 0;
        for (int k : {2, 4, 8, 16, nranks}) {
            if (k > nranks && k != 2) continue;
            if (std::find(tried, tried + ntried, k) != tried + ntried) continue;
            tried[ntried++] = k;
            consider(BCAST_ALGO_KNOMIAL_PIPELINED, std::max<size_t>(16, (M + 15) / 16 * 16), k);
            for (size_t C : {(size_t)64 << 10, (size_t)512 << 10})
                if (C < M && M / C <= 4096) consider(BCAST_ALGO_KNOMIAL_PIPELINED, C, k);
        }
        if (rc != BCAST_OK) break;
        // A wave-per-rank chain of several stages must win clearly.  Its time moves more with where the rank
        // buffers happen to lie than the wave-per-stage chain's does (the same shape at 64 ranks x 1 GiB: 10.1 to
        // 10.9 ms from one set of placed buffers to the next, the wave-per-stage chain 10.2 to 10.5), and the
        // tuner sees one set only.  Within kRankWavesMargin the steadier kernel keeps the entry.
        constexpr double kRankWavesMargin = 1.05;
        if (best.algo == BCAST_ALGO_CHAIN && best.rank_waves && best.stages >= 2 && runner.usec <= best.usec * kRankWavesMargin) {
            best.algo = runner.algo;
            best.chunk_bytes = runner.chunk_bytes;
            best.stages = runner.stages;
            best.trip_bytes = runner.trip_bytes;
            best.rank_waves = runner.rank_waves;
            best.stage_store = runner.stage_store;
            best.lanes = runner.lanes;
            best.spans = runner.spans;
            best.usec = runner.usec;
        }
        if (best.chain_rank_waves && best.chain_stages >= 2 && relay.usec <= best.chain_usec * kRankWavesMargin) {
            best.chain_chunk_bytes = relay.chunk_bytes;
            best.chain_stages = relay.stages;
            best.chain_trip_bytes = relay.trip_bytes;
            best.chain_rank_waves = 0;
            best.chain_stage_store = relay.stage_store;
            best.chain_lanes = relay.lanes;
            best.chain_spans = relay.spans;
            best.chain_usec = relay.usec;
        }
        if (best.chain_chunk_bytes == 0) best.chain_usec = 0.0;
        rc = bcast_tune_put(nranks, M, &best);
        if (f) print_entry(f, nranks, log2_bucket(M), best);
        if (M > (max_bytes >> 1)) break;  // next doubling would overflow or pass max
    }
    if (f) fclose(f);
    return rc;
}

// The reduction's sweep: stage counts 1, 2, 4; trips of 4 KiB and (up to a few
// MiB) 1 KiB; chunks of one trip per lane for power-of-two lane counts, and the
// whole message as one chunk.  Timed like the broadcast's candidates.
extern "C" int bcast_tune_reduce(int nranks, size_t min_bytes, size_t max_bytes, bcast_stream_t stream, const char *table_path)
{
    if (nranks < 2 || nranks > BCAST_MAX_RANKS || min_bytes < 4 || max_bytes < min_bytes) return BCAST_ERR_ARG;
    // placed as the library recommends for a reduction: the contributions in one
    // region of the device's memory, the result in another (see memory.cpp)
    Scratch sc;
    sc.bufs.assign(nranks + 1, nullptr);
    {
        std::vector<size_t> sizes(nranks + 1, max_bytes);
        std::vector<int> region(nranks + 1, 0);
        region[nranks] = 1;
        int rc_alloc = bcast_buffers_alloc(nranks + 1, sizes.data(), region.data(), sc.bufs.data(), nullptr);
        if (rc_alloc != BCAST_OK) return rc_alloc;
    }
    for (int r = 0; r <= nranks; ++r) {
        hipError_t e = hipMemset(sc.bufs[r], 0, max_bytes);  // fp32 zeros: sums stay finite
        if (e != hipSuccess) return BCAST_ERR_HIP;
    }
    if (hipEventCreate(&sc.e0) != hipSuccess || hipEventCreate(&sc.e1) != hipSuccess) return BCAST_ERR_HIP;
    FILE *log = nullptr;
    {
        std::lock_guard<std::mutex> g(g_mu);
        if (!g_log_path.empty()) log = fopen(g_log_path.c_str(), "a");
    }
    if (log) fprintf(log, "# reduce nranks bytes chunk_bytes stages trip_bytes usec\n");
    struct Closer {
        FILE *f;
        ~Closer() { if (f) fclose(f); }
    } log_closer{log};
    FILE *f = nullptr;
    if (table_path) {
        f = fopen(table_path, "a");
        if (!f) return BCAST_ERR_ARG;
        fprintf(f, "%s", kReduceHeaderLine);
    }
    Closer table_closer{f};
    const int hops = nranks - 1;
    int rc = BCAST_OK;
    size_t M = (size_t)1 << log2_bucket(min_bytes);
    if (M < min_bytes) M <<= 1;
    for (; M <= max_bytes && rc == BCAST_OK; M <<= 1) {
        bcast_reduce_entry_t best;
        memset(&best, 0, sizeof best);
        best.usec = 1e30;
        auto consider = [&](size_t chunk, int stages, int trip) {
            if (rc != BCAST_OK) return;
            bcast_plan_t *plan = nullptr;
            rc = bcast_plan_create(&plan, nranks, M, chunk, BCAST_ALGO_CHAIN);
            if (rc != BCAST_OK) return;
            rc = bcast_plan_set_stages(plan, stages);
            if (rc == BCAST_OK) rc = bcast_plan_set_reduce_trip(plan, trip);
            if (rc == BCAST_OK) rc = bcast_plan_reserve_reduce(plan, M / sizeof(float), stages);
            int reps = 1;
            double fastest = 1e30;
            for (int batch = 0; batch < 4 && rc == BCAST_OK; ++batch) {
                if (hipEventRecord(sc.e0, stream) != hipSuccess) { rc = BCAST_ERR_HIP; break; }
                for (int i = 0; i < reps && rc == BCAST_OK; ++i)
                    rc = bcast_reduce_sum_f32(plan, sc.bufs.data(), sc.bufs[nranks], 0, M / sizeof(float), stream);
                if (rc != BCAST_OK) break;
                if (hipEventRecord(sc.e1, stream) != hipSuccess || hipEventSynchronize(sc.e1) != hipSuccess) { rc = BCAST_ERR_HIP; break; }
                float ms = 0.f;
                if (hipEventElapsedTime(&ms, sc.e0, sc.e1) != hipSuccess) { rc = BCAST_ERR_HIP; break; }
                const double us = (double)ms * 1000.0 / reps;
                if (batch == 0) reps = (int)std::min(40.0, std::max(2.0, 20000.0 / std::max(us, 1.0)));
                else fastest = std::min(fastest, us);
            }
            if (rc == BCAST_OK && bcast_plan_status(plan, nullptr) != BCAST_OK) rc = BCAST_ERR_TIMEOUT;
            int rd = bcast_plan_destroy(plan);
            if (rc == BCAST_OK) rc = rd;
            if (rc != BCAST_OK) return;
            if (log) fprintf(log, "reduce %d %zu %zu %d %d %.3f\n", nranks, M, chunk, stages, trip, fastest);
            if (fastest < best.usec) {
                best.chunk_bytes = chunk;
                best.stages = stages;
                best.trip_bytes = trip;
                best.usec = fastest;
            }
        };
        const size_t whole = std::max<size_t>(16, (M + 15) / 16 * 16);
        for (int stages : {1, 2, 4}) {
            if (stages > hops) continue;
            for (int trip : {4096, 1024}) {
                if (trip == 1024 && M > ((size_t)8 << 20)) continue;
                consider(whole, stages, trip);
                for (size_t lanes = 64; lanes * (size_t)stages <= 8192; lanes <<= 1) {
                    const size_t C = lanes * (size_t)trip;
                    if (C >= M || M / C > 4096) continue;
                    consider(C, stages, trip);
                }
            }
        }
        if (rc != BCAST_OK) break;
        rc = bcast_tune_reduce_put(nranks, M, &best);
        if (f) print_reduce_entry(f, nranks, log2_bucket(M), best);
        if (M > (max_bytes >> 1)) break;
    }
    return rc;
}

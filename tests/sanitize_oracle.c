/*
 * Driver for the sanitizer pass over the CPU oracle (test infrastructure).
 * Built by tests/test_oracle_sanitizers.py together with oracle/bcast_oracle.c
 * under -fsanitize=address,undefined and run as a plain executable: every
 * schedule of the oracle on every small configuration (ranks, roots, sizes,
 * chunk sizes, radices, traces of every capacity), its end state compared with
 * row replication written out here.  AddressSanitizer and UBSan abort the run
 * on an out-of-bounds access, a leak, an overflow or a misaligned access; a
 * wrong end state or count exits with status 1.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "bcast_oracle.h"

static int failures = 0;
#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            if (failures++ < 20) {                         \
                fprintf(stderr, "FAIL %s:%d: ", __FILE__, __LINE__); \
                fprintf(stderr, __VA_ARGS__);              \
                fprintf(stderr, "\n");                     \
            }                                              \
        }                                                  \
    } while (0)

typedef struct {
    unsigned char **rows;
    unsigned char *want;
    int P;
    size_t cap;
} bufs_t;

/* P rows of exactly cap bytes each (separate allocations, so that one byte too
 * far is a sanitizer report), root filled with a pattern, others 0xFF */
static bufs_t make(int P, int root, size_t M, size_t cap, unsigned seed)
{
    bufs_t b;
    b.P = P;
    b.cap = cap;
    b.rows = (unsigned char **)malloc(sizeof(unsigned char *) * (size_t)P);
    b.want = (unsigned char *)malloc(cap ? cap : 1);
    for (int r = 0; r < P; ++r) {
        b.rows[r] = (unsigned char *)malloc(cap ? cap : 1);
        memset(b.rows[r], 0xFF, cap);
    }
    for (size_t i = 0; i < cap; ++i) b.want[i] = 0xFF;
    for (size_t i = 0; i < M; ++i) {
        seed = seed * 1103515245u + 12345u;
        b.rows[root][i] = b.want[i] = (unsigned char)(seed >> 16);
    }
    for (size_t i = M; i < cap; ++i) b.rows[root][i] = 0xFF;
    return b;
}

static void expect_replicated(const bufs_t *b, const char *what, int P, int root, size_t M, size_t C, int k)
{
    for (int r = 0; r < b->P; ++r)
        CHECK(memcmp(b->rows[r], b->want, b->cap) == 0, "%s P=%d root=%d M=%zu C=%zu k=%d: rank %d differs", what, P, root, M, C, k, r);
}

static void drop(bufs_t *b)
{
    for (int r = 0; r < b->P; ++r) free(b->rows[r]);
    free(b->rows);
    free(b->want);
}

static long ceil_log(long P, long k)
{
    long rounds = 0;
    for (long reach = 1; reach < P; reach *= k) ++rounds;
    return rounds;
}

int main(void)
{
    long runs = 0;
    for (int P = 1; P <= 9; ++P)
        for (int root = 0; root < P; ++root)
            for (size_t M = 0; M <= 24; M += (M < 6 ? 1 : 3)) {
                const size_t cap = M + 2;  /* two guard bytes behind the message */
                /* chain over every chunk size, with traces of several capacities */
                for (size_t C = 1; C <= M + 2; ++C) {
                    bufs_t b = make(P, root, M, cap, (unsigned)(P * 131 + root * 17 + M));
                    const size_t nchunks = M ? (M + C - 1) / C : 0;
                    const size_t cap_x = (size_t)((P + (int)M + (int)C) % 7);  /* often too small on purpose */
                    const size_t cap_h = (size_t)((P + root) % 4);
                    oracle_trace_t tr;
                    memset(&tr, 0, sizeof tr);
                    tr.xfers = cap_x ? (oracle_xfer_t *)malloc(sizeof(oracle_xfer_t) * cap_x) : NULL;
                    tr.xfers_cap = cap_x;
                    tr.have = cap_h ? (long *)malloc(sizeof(long) * cap_h * (size_t)P) : NULL;
                    tr.have_cap_steps = cap_h;
                    long steps = oracle_chain_bcast(b.rows, P, root, M, C, &tr);
                    long want_steps = (P < 2 || M == 0) ? 0 : (long)nchunks + P - 2;
                    CHECK(steps == want_steps, "chain steps P=%d M=%zu C=%zu: %ld != %ld", P, M, C, steps, want_steps);
                    CHECK(tr.bytes_copied == (unsigned long long)(P < 2 ? 0 : (size_t)(P - 1) * M), "chain bytes");
                    CHECK(tr.xfers_len == (P < 2 ? 0 : (size_t)(P - 1) * nchunks), "chain transfers");
                    expect_replicated(&b, "chain", P, root, M, C, 0);
                    free(tr.xfers);
                    free(tr.have);
                    drop(&b);
                    ++runs;
                    /* schedule only */
                    CHECK(oracle_chain_bcast(NULL, P, root, M, C, NULL) == want_steps, "chain schedule-only steps");
                    for (int k = 2; k <= 4; ++k) {
                        bufs_t t = make(P, root, M, cap, 7u + (unsigned)M);
                        long s = oracle_knomial_pipeline_bcast(t.rows, P, root, M, C, k, NULL);
                        long w = (P < 2 || M == 0) ? 0 : (long)nchunks * ceil_log(P, k);
                        CHECK(s == w, "pipelined k-nomial steps P=%d M=%zu C=%zu k=%d: %ld != %ld", P, M, C, k, s, w);
                        expect_replicated(&t, "knomial_pipeline", P, root, M, C, k);
                        drop(&t);
                        ++runs;
                    }
                }
                {
                    bufs_t b = make(P, root, M, cap, 3u);
                    CHECK(oracle_naive_bcast(b.rows, P, root, M) == 0, "naive rc");
                    expect_replicated(&b, "naive", P, root, M, 0, 0);
                    drop(&b);
                    b = make(P, root, M, cap, 4u);
                    CHECK(oracle_direct_bcast(b.rows, P, root, M, NULL) == P - 1, "direct sends");
                    expect_replicated(&b, "direct", P, root, M, 0, 0);
                    drop(&b);
                    b = make(P, root, M, cap, 5u);
                    CHECK(oracle_binomial_bcast(b.rows, P, root, M, NULL) == ceil_log(P, 2), "binomial rounds");
                    expect_replicated(&b, "binomial", P, root, M, 0, 0);
                    drop(&b);
                    for (int k = 2; k <= 10; ++k) {
                        b = make(P, root, M, cap, 6u);
                        CHECK(oracle_knomial_bcast(b.rows, P, root, M, k, NULL) == ceil_log(P, k), "k-nomial rounds");
                        expect_replicated(&b, "knomial", P, root, M, 0, k);
                        drop(&b);
                    }
                    b = make(P, root, M, cap, 8u);
                    long sr = -1, rs = -1;
                    long total = oracle_scatter_allgather_bcast(b.rows, P, root, M, &sr, &rs, NULL);
                    CHECK(total == sr + rs && rs == (P > 1 ? P - 1 : 0) && sr == ceil_log(P, 2), "scatter+allgather counts P=%d: %ld %ld %ld", P, total, sr, rs);
                    expect_replicated(&b, "scatter_allgather", P, root, M, 0, 0);
                    drop(&b);
                    runs += 13;
                }
                /* chain reduction: small integers sum exactly in fp32 whatever the order */
                for (size_t chunk = 1; chunk <= M + 1; chunk += 2) {
                    const size_t count = M;
                    float **send = (float **)malloc(sizeof(float *) * (size_t)P);
                    float *recv = (float *)malloc(sizeof(float) * (count ? count : 1));
                    for (int r = 0; r < P; ++r) {
                        send[r] = (float *)malloc(sizeof(float) * (count ? count : 1));
                        for (size_t i = 0; i < count; ++i) send[r][i] = (float)((int)((r * 7 + i * 3) % 23) - 11);
                    }
                    long steps = oracle_chain_reduce_f32((const float *const *)send, recv, P, root, count, chunk, NULL);
                    const size_t nchunks = count ? (count + chunk - 1) / chunk : 0;
                    CHECK(steps == ((P < 2 || count == 0) ? 0 : (long)nchunks + P - 2), "reduce steps");
                    for (size_t i = 0; i < count; ++i) {
                        long sum = 0;
                        for (int r = 0; r < P; ++r) sum += (long)((int)((r * 7 + i * 3) % 23) - 11);
                        CHECK(recv[i] == (float)sum, "reduce P=%d root=%d count=%zu chunk=%zu element %zu: %g != %ld", P, root, count, chunk, i, (double)recv[i], sum);
                    }
                    /* in place at the root */
                    steps = oracle_chain_reduce_f32((const float *const *)send, send[root], P, root, count, chunk, NULL);
                    for (size_t i = 0; i < count; ++i) CHECK(send[root][i] == recv[i], "reduce in place");
                    for (int r = 0; r < P; ++r) free(send[r]);
                    free(send);
                    free(recv);
                    ++runs;
                }
            }
    /* argument errors return -1 and touch nothing */
    CHECK(oracle_chain_bcast(NULL, 4, 4, 10, 2, NULL) == -1, "root out of range");
    CHECK(oracle_chain_bcast(NULL, 4, 0, 10, 0, NULL) == -1, "zero chunk");
    CHECK(oracle_knomial_bcast(NULL, 4, 0, 10, 1, NULL) == -1, "radix 1");
    CHECK(oracle_naive_bcast(NULL, 0, 0, 1) == -1, "no ranks");
    /* the model functions on ordinary arguments */
    CHECK(fabs(oracle_model_chain_pipeline(8, 64e6, 4e6, 2e-6, 5e12) - (16 + 6) * (2e-6 + 4e6 / 5e12)) < 1e-12, "Eq. 5");
    CHECK(oracle_model_direct(8, 1e6, 1e-6, 1e12) > 0 && oracle_model_chain(8, 1e6, 1e-6, 1e12) > 0 &&
              oracle_model_knomial(8, 2, 1e6, 1e-6, 1e12) > 0 && oracle_model_scatter_allgather(8, 1e6, 1e-6, 1e12) > 0 &&
              oracle_model_knomial_pipeline(8, 2, 1e6, 1e5, 1e-6, 1e12) > 0,
          "models");
    printf("sanitize_oracle: %ld runs, %d failures\n", runs, failures);
    return failures ? 1 : 0;
}

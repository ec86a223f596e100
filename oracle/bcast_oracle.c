/*
 * CPU oracle for rooted broadcast schedules -- TEST INFRASTRUCTURE ONLY.
 * See bcast_oracle.h for the contract.  Plain C, single thread, memcpy for
 * payload; nothing here is blocked, fused or reordered beyond what each
 * schedule's description in the paper states.
 */
#include "bcast_oracle.h"

#include <stdlib.h>
#include <string.h>

/* rank that sits at chain position k when the broadcast root is `root` */
static int rank_at(int root, int k, int P) { return (root + k) % P; }

static int bad_common(int P, int root) { return P < 1 || root < 0 || root >= P; }

static void trace_reset(oracle_trace_t *tr)
{
    if (!tr) return;
    tr->xfers_len = 0;
    tr->bytes_copied = 0;
}

/* Perform (or, with bufs == NULL, only account for) one transfer. */
static void transfer(unsigned char **bufs, oracle_trace_t *tr, long step, int src_rank,
                     int dst_rank, long chunk, size_t lo, size_t hi)
{
    if (bufs && hi > lo) memcpy(bufs[dst_rank] + lo, bufs[src_rank] + lo, hi - lo);
    if (tr) {
        if (tr->xfers && tr->xfers_len < tr->xfers_cap) {
            oracle_xfer_t *x = &tr->xfers[tr->xfers_len];
            x->step = step;
            x->src_rank = src_rank;
            x->dst_rank = dst_rank;
            x->chunk = chunk;
            x->lo = lo;
            x->hi = hi;
        }
        tr->xfers_len++;
        tr->bytes_copied += hi - lo;
    }
}

int oracle_naive_bcast(unsigned char **bufs, int P, int root, size_t M)
{
    if (bad_common(P, root) || !bufs) return -1;
    for (int r = 0; r < P; r++)
        if (r != root && M) memcpy(bufs[r], bufs[root], M);
    return 0;
}

long oracle_chain_bcast(unsigned char **bufs, int P, int root, size_t M, size_t C,
                        oracle_trace_t *tr)
{
    if (bad_common(P, root) || C == 0) return -1;
    trace_reset(tr);
    if (P < 2 || M == 0) return 0;

    /* number of chunks: the last one may be short (Eq. 5's M/C, rounded up) */
    long nchunks = (long)(M / C) + (M % C ? 1 : 0);

    /* have[k] = how many chunks position k holds; always the prefix 0..have[k)-1 */
    long *have = calloc((size_t)P, sizeof *have);
    long *seen = calloc((size_t)P, sizeof *seen);
    if (!have || !seen) { free(have); free(seen); return -1; }
    have[0] = nchunks; /* the root starts with the whole message */

    long steps = 0;
    for (;;) {
        int unfinished = 0;
        for (int k = 1; k < P; k++)
            if (have[k] < nchunks) unfinished = 1;
        if (!unfinished) break;

        /* every link looks at the state as it was when the step began, so a
         * chunk advances by exactly one hop per step */
        memcpy(seen, have, (size_t)P * sizeof *have);
        for (int k = 1; k < P; k++) {
            long c = seen[k];                 /* next chunk position k is missing */
            if (c < nchunks && seen[k - 1] > c) {
                size_t lo = (size_t)c * C;
                size_t hi = lo + C < M ? lo + C : M;
                /* received from the LEFT NEIGHBOUR, which forwards what it stored */
                transfer(bufs, tr, steps, rank_at(root, k - 1, P), rank_at(root, k, P), c, lo, hi);
                have[k] = c + 1;
            }
        }
        if (tr && tr->have && (size_t)steps < tr->have_cap_steps)
            memcpy(tr->have + (size_t)steps * (size_t)P, have, (size_t)P * sizeof *have);
        steps++;
    }
    free(have);
    free(seen);
    return steps;
}

long oracle_direct_bcast(unsigned char **bufs, int P, int root, size_t M, oracle_trace_t *tr)
{
    if (bad_common(P, root)) return -1;
    trace_reset(tr);
    long sends = 0;
    for (int k = 1; k < P; k++) {
        transfer(bufs, tr, sends, root, rank_at(root, k, P), 0, 0, M);
        sends++;
    }
    return sends;
}

long oracle_binomial_bcast(unsigned char **bufs, int P, int root, size_t M, oracle_trace_t *tr)
{
    if (bad_common(P, root)) return -1;
    trace_reset(tr);
    long rounds = 0;
    /* before round j the holders are exactly positions 0 .. 2^j - 1 */
    for (long reach = 1; reach < P; reach *= 2) {
        for (long q = 0; q < reach; q++) {
            long child = q + reach;
            if (child < P)
                transfer(bufs, tr, rounds, rank_at(root, (int)q, P), rank_at(root, (int)child, P),
                         0, 0, M);
        }
        rounds++;
    }
    return rounds;
}

long oracle_knomial_bcast(unsigned char **bufs, int P, int root, size_t M, int k, oracle_trace_t *tr)
{
    if (bad_common(P, root) || k < 2) return -1;
    trace_reset(tr);
    long rounds = 0;
    /* before round j the holders are exactly positions 0 .. reach - 1, reach = k^j */
    for (long reach = 1; reach < P; reach *= k) {
        for (long q = 0; q < reach; q++)
            for (long i = 1; i < k; i++) {
                long child = q + i * reach;
                if (child < P)
                    transfer(bufs, tr, rounds, rank_at(root, (int)q, P), rank_at(root, (int)child, P),
                             0, 0, M);
            }
        rounds++;
    }
    return rounds;
}

long oracle_knomial_pipeline_bcast(unsigned char **bufs, int P, int root, size_t M, size_t C, int k,
                                   oracle_trace_t *tr)
{
    if (bad_common(P, root) || k < 2 || C == 0) return -1;
    trace_reset(tr);
    if (P < 2 || M == 0) return 0;
    long pieces = (long)(M / C);
    if (M % C) pieces++; /* a short last chunk is a chunk */
    long steps = 0;
    /* level by level as in the k-nomial tree; inside a level the message goes
     * out one chunk per step, to all children of the level at once */
    for (long span = 1; span < P; span *= k) {
        for (long ch = 0; ch < pieces; ch++) {
            size_t from = (size_t)ch * C;
            size_t to = from + C < M ? from + C : M;
            for (long holder = 0; holder < span; holder++)
                for (long d = 1; d < k; d++) {
                    long target = holder + d * span;
                    if (target < P)
                        transfer(bufs, tr, steps, rank_at(root, (int)holder, P),
                                 rank_at(root, (int)target, P), ch, from, to);
                }
            steps++;
        }
    }
    return steps;
}

long oracle_scatter_allgather_bcast(unsigned char **bufs, int P, int root, size_t M,
                                    long *scatter_rounds, long *ring_steps, oracle_trace_t *tr)
{
    if (bad_common(P, root)) return -1;
    trace_reset(tr);
    if (scatter_rounds) *scatter_rounds = 0;
    if (ring_steps) *ring_steps = 0;
    if (P < 2) return 0;

    size_t piece = M / (size_t)P + (M % (size_t)P ? 1 : 0); /* ceil(M / P) */
#define PIECE_LO(q) ((size_t)(q) * piece < M ? (size_t)(q) * piece : M)

    /* Binomial scatter: a position that is a multiple of 2*stride holds the
     * pieces of positions [q, q + 2*stride); it hands the upper half of that
     * range to position q + stride.  Strides go from the top power of two down. */
    long top = 1;
    while (top < P) top *= 2;
    long rounds = 0;
    for (long stride = top / 2; stride >= 1; stride /= 2) {
        for (long q = 0; q + stride < P; q += 2 * stride) {
            long last = q + 2 * stride < P ? q + 2 * stride : P;
            transfer(bufs, tr, rounds, rank_at(root, (int)q, P), rank_at(root, (int)(q + stride), P),
                     q + stride, PIECE_LO(q + stride), PIECE_LO(last));
        }
        rounds++;
    }

    /* Ring allgather with wrap-around: in step t position q passes piece
     * (q - t) mod P to position q + 1.  What would arrive at position 0 is
     * data the root already owns, and the root's buffer is input only, so
     * that one transfer per step is not performed. */
    long steps = 0;
    for (long t = 0; t < P - 1; t++) {
        for (long q = 0; q < P; q++) {
            long dst = (q + 1) % P;
            if (dst == 0) continue;
            long pc = ((q - t) % P + P) % P;
            transfer(bufs, tr, rounds + steps, rank_at(root, (int)q, P), rank_at(root, (int)dst, P),
                     pc, PIECE_LO(pc), PIECE_LO(pc + 1));
        }
        steps++;
    }
#undef PIECE_LO
    if (scatter_rounds) *scatter_rounds = rounds;
    if (ring_steps) *ring_steps = steps;
    return rounds + steps;
}

long oracle_chain_reduce_f32(const float *const *send, float *recv, int P, int root, size_t count,
                             size_t chunk_elems, oracle_trace_t *tr)
{
    if (bad_common(P, root) || chunk_elems == 0) return -1;
    if (count && (!send || !recv) && (send || recv)) return -1; /* both or neither */
    trace_reset(tr);
    if (count == 0) return 0;
    const int payload = send != NULL;
    if (P == 1) {
        if (payload) memmove(recv, send[root], count * sizeof(float));
        return 0;
    }
    long nchunks = (long)(count / chunk_elems) + (count % chunk_elems ? 1 : 0);

    /* partial[k] = running sum held by chain position k: position P-1 starts
     * with its own contribution, every other position adds its own to what its
     * RIGHT neighbour (k + 1) hands over, and position 0 is the root */
    float *partial = payload ? malloc((size_t)P * count * sizeof(float)) : NULL;
    long *got = calloc((size_t)P, sizeof *got);   /* chunks of its partial that position k holds */
    long *before = calloc((size_t)P, sizeof *before);
    if ((payload && !partial) || !got || !before) { free(partial); free(got); free(before); return -1; }
    if (payload) memcpy(partial + (size_t)(P - 1) * count, send[rank_at(root, P - 1, P)], count * sizeof(float));
    got[P - 1] = nchunks;

    long steps = 0;
    while (got[0] < nchunks) {
        memcpy(before, got, (size_t)P * sizeof *got); /* all links decide from the start of the step */
        for (int k = P - 2; k >= 0; k--) {
            long c = before[k];
            if (c < nchunks && before[k + 1] > c) {
                size_t e0 = (size_t)c * chunk_elems;
                size_t e1 = e0 + chunk_elems < count ? e0 + chunk_elems : count;
                if (payload) {
                    const float *mine = send[rank_at(root, k, P)];
                    const float *in = partial + (size_t)(k + 1) * count;
                    float *out = partial + (size_t)k * count;
                    for (size_t i = e0; i < e1; i++) out[i] = mine[i] + in[i]; /* one fp32 addition */
                }
                /* account for the hand-over as a transfer of the partial's bytes */
                transfer(NULL, tr, steps, rank_at(root, k + 1, P), rank_at(root, k, P), c,
                         e0 * sizeof(float), e1 * sizeof(float));
                got[k] = c + 1;
            }
        }
        steps++;
    }
    if (payload) memcpy(recv, partial, count * sizeof(float));
    free(partial);
    free(got);
    free(before);
    return steps;
}

/* smallest r with k^r >= n */
static int ceil_log(int n, int k)
{
    int r = 0;
    long reach = 1;
    while (reach < n) { reach *= k; r++; }
    return r;
}

double oracle_model_direct(int n, double M, double ts, double B) { return n * (ts + M / B); }

double oracle_model_chain(int n, double M, double ts, double B) { return (n - 1) * (ts + M / B); }

double oracle_model_knomial(int n, int k, double M, double ts, double B)
{
    return ceil_log(n, k) * (ts + M / B);
}

double oracle_model_knomial_pipeline(int n, int k, double M, double C, double ts, double B)
{
    return (M / C * ceil_log(n, k)) * (ts + C / B);
}

double oracle_model_scatter_allgather(int n, double M, double ts, double B)
{
    return (ceil_log(n, 2) + n - 1) * ts + 2.0 * ((n - 1) * M / n) / B;
}

double oracle_model_chain_pipeline(int n, double M, double C, double ts, double B)
{
    return (M / C + (n - 2)) * (ts + C / B);
}

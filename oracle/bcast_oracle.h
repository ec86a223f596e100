/*
 * CPU oracle for rooted broadcast schedules -- TEST INFRASTRUCTURE ONLY.
 *
 * This is the slow, plain reference that the GPU library is checked against.
 * It is not part of the product: only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the HIP
 * path and includes no GPU header.
 *
 * "Rank" r owns host buffer bufs[r].  The broadcast root is `root`; chain
 * position k (0 <= k < P) is rank (root + k) mod P, so the chain runs
 * root -> root+1 -> ... -> root-1 and never wraps back to the root
 * (paper Sec. III-A, "Chain and Ring Algorithms").
 *
 * Every function may be called with bufs == NULL: it then walks the same
 * schedule without touching payload (used for step counts at sizes whose
 * payload does not fit in host memory).
 *
 * Parity status: every function here is pinned by tests that do not use this
 * file's own arithmetic (numpy row replication for the end state, the paper's
 * closed-form step counts for the schedules, hand-worked values of the cost
 * models, parent and step of every transfer derived independently in the test,
 * and a set of planted mistakes that the pins must reject).  Nothing is
 * "parity unpinned".
 */
#ifndef BCAST_ORACLE_H
#define BCAST_ORACLE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One point-to-point transfer performed by a schedule. */
typedef struct {
    long step;               /* 0-based step (chain), round (binomial), or send index (direct) */
    int src_rank;            /* rank whose buffer was read  */
    int dst_rank;            /* rank whose buffer was written */
    long chunk;              /* chunk index (0 for unchunked schedules) */
    unsigned long long lo;   /* first byte offset copied */
    unsigned long long hi;   /* one past the last byte offset copied */
} oracle_xfer_t;

/* Optional recording of what a schedule did.  Zero-initialise, then set the
 * capacities and caller-owned arrays you want filled. */
typedef struct {
    oracle_xfer_t *xfers;    /* caller-owned array, may be NULL */
    size_t xfers_cap;        /* entries available in xfers */
    size_t xfers_len;        /* OUT: transfers performed (may exceed cap; extra ones are not stored) */
    long *have;              /* caller-owned [have_cap_steps][P]; row s = chunks held per chain position after step s */
    size_t have_cap_steps;   /* rows available in have */
    unsigned long long bytes_copied; /* OUT: total payload bytes moved */
} oracle_trace_t;

/* The definition of MPI_Bcast's result (paper Sec. I, Sec. III-A "Direct
 * Algorithm"): every non-root buffer's first M bytes become the root's.
 * Returns 0, or -1 on bad arguments. */
int oracle_naive_bcast(unsigned char **bufs, int P, int root, size_t M);

/* Pipelined chain broadcast (paper Sec. IV-B, Eq. 5) as a synchronous
 * step simulation: in one step every link (k-1 -> k) moves at most one chunk,
 * and all links decide from the state at the start of the step.
 * C >= M gives the unpipelined chain (Eq. 2).  Returns the number of steps,
 * 0 when P < 2 or M == 0, or -1 on bad arguments (C == 0, root out of range). */
long oracle_chain_bcast(unsigned char **bufs, int P, int root, size_t M, size_t C,
                        oracle_trace_t *tr);

/* Direct algorithm (Sec. III-A, Eq. 1): the root sends the whole message to
 * each other rank, one after another, in chain-position order.
 * Returns the number of sends (P - 1), or -1 on bad arguments. */
long oracle_direct_bcast(unsigned char **bufs, int P, int root, size_t M,
                         oracle_trace_t *tr);

/* Binomial tree (Sec. III-A, Eq. 3 with k = 2): in round j every chain
 * position q < 2^j that holds the message sends all of it to q + 2^j
 * (if that position exists).  Returns the number of rounds, ceil(log2 P),
 * or -1 on bad arguments. */
long oracle_binomial_bcast(unsigned char **bufs, int P, int root, size_t M,
                           oracle_trace_t *tr);

/* K-nomial tree (Sec. III-A, Eq. 3, general radix k >= 2): before round j the
 * holders are chain positions 0 .. k^j - 1; in round j every holder q sends the
 * whole message to q + i * k^j for i = 1 .. k-1 (where that position exists).
 * All sends of a round count as one step of Eq. 3.  k = 2 is the binomial tree.
 * Returns the number of rounds, ceil(log_k P), or -1 on bad arguments. */
long oracle_knomial_bcast(unsigned char **bufs, int P, int root, size_t M, int k,
                          oracle_trace_t *tr);

/* Pipelined k-nomial tree: the k-nomial levels of Eq. 3 with the message cut
 * into chunks of C bytes as in Sec. IV-B.  The paper pipelines the chain only;
 * this is the build's own extension of the same chunking to the tree, taken
 * level by level: a sender needs ceil(M/C) steps to push the message to its
 * children of one level and there are ceil(log_k n) levels, so
 * (ceil(M/C) * ceil(log_k n)) steps of (t_s + C/B) each.
 * This function walks exactly that: level after level, and inside a level one
 * step per chunk in which every holder sends that chunk to each of its k - 1
 * children of the level.  C >= M is oracle_knomial_bcast.  Returns the number
 * of steps, ceil(M/C) * ceil(log_k P), 0 when P < 2 or M == 0, or -1 on bad
 * arguments. */
long oracle_knomial_pipeline_bcast(unsigned char **bufs, int P, int root, size_t M, size_t C, int k,
                                   oracle_trace_t *tr);

/* Scatter + ring allgather (Sec. III-A, Eq. 4): the message is cut into P
 * pieces of ceil(M/P) bytes (piece q may be short or empty); a binomial
 * scatter leaves position q holding piece q, then P - 1 ring steps pass
 * pieces around (with wrap-around) until everyone holds all of them.
 * *scatter_rounds and *ring_steps (nullable) receive the two counts.
 * Returns their sum, or -1 on bad arguments. */
long oracle_scatter_allgather_bcast(unsigned char **bufs, int P, int root, size_t M,
                                    long *scatter_rounds, long *ring_steps,
                                    oracle_trace_t *tr);

/* Pipelined chain REDUCTION (sum, fp32): the collective the paper names as the
 * next one to receive the pipelined chain (Sec. VII); the paper gives no
 * schedule, so this is the broadcast chain of Sec. IV-B run backwards.  Chain
 * position k is rank (root + k) mod P as before.  Position P-1 starts the
 * running sum with its own contribution; every position k < P-1 receives the
 * running sum of a chunk from its right neighbour k+1, adds its own
 * contribution with ONE fp32 addition per element (own + incoming) and hands the
 * result to k-1; position 0, the root, stores it in recv.  Hence
 *   recv[i] = x_0[i] + (x_1[i] + ( ... + (x_{P-2}[i] + x_{P-1}[i]))),
 * every addition rounded to fp32 (round to nearest even), x_k = send[(root+k)%P].
 * One step moves at most one chunk (chunk_elems elements, the last one short)
 * per link, all links deciding from the state at the start of the step, so the
 * step count is chunks + P - 2 as in Eq. 5.  send == recv == NULL walks the
 * schedule only.  recv may be send[root].  Returns the steps, 0 when P == 1
 * (recv = send[root]) or count == 0, -1 on bad arguments. */
long oracle_chain_reduce_f32(const float *const *send, float *recv, int P, int root, size_t count,
                             size_t chunk_elems, oracle_trace_t *tr);

/* Cost models of Sec. III-A and IV-B, evaluated literally as printed
 * (Eq. 1: direct, Eq. 2: chain, Eq. 3: k-nomial, Eq. 4: scatter-allgather,
 * Eq. 5: pipelined chain).  n ranks, M message bytes, C chunk bytes,
 * ts start-up seconds, B bytes per second, k tree radix. */
double oracle_model_direct(int n, double M, double ts, double B);
double oracle_model_chain(int n, double M, double ts, double B);
double oracle_model_knomial(int n, int k, double M, double ts, double B);
double oracle_model_scatter_allgather(int n, double M, double ts, double B);
/* the level-by-level pipelined k-nomial tree (the build's extension, see above): (M/C * ceil(log_k n)) (t_s + C/B) */
double oracle_model_knomial_pipeline(int n, int k, double M, double C, double ts, double B);
double oracle_model_chain_pipeline(int n, double M, double C, double ts, double B);

#ifdef __cplusplus
}
#endif
#endif

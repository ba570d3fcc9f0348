/*
 * CPU oracle for round-optimal broadcast schedules (Träff, arXiv 2407.18004).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * step-by-step transcription of the paper's definitions into sequential C
 * (int64 arithmetic, recursion, linked lists), written to be checked against
 * the paper by eye.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper
 * with the HIP library.
 *
 * Domain: 1 <= p < 2^40 for schedules; the digest needs q <= 31 (p <= 2^31).
 * q = ceil(log2 p) computed with integers (Section 2).
 *
 * What pins each function to something other than itself is listed next to
 * the tests; nothing here is "parity unpinned" except the hashes of orc_digest
 * and orc_edgecheck (definitions of this build, not of the paper: the digest's
 * flags and the edge check's equality are pinned, the hash values are not).
 */
#ifndef BCAST_ORACLE_H
#define BCAST_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_MAXQ 40

/* Counters of the receive-schedule search (Algorithm 4), for the complexity
 * lemmas of Section 2.2 and for the anomaly checks the tests make. */
typedef struct {
    int64_t scans;       /* iterations of the while loop over all calls      */
    int64_t calls;       /* recursive calls (first invocation not counted)   */
    int64_t max_depth;   /* deepest recursion reached (first call = depth 0) */
    int64_t anomalies;   /* an index pushed while already on the path, an
                            index accepted twice, or k reaching q inside a
                            frame whose index is still linked: none of these
                            may happen if the paper's invariants hold        */
} orc_recv_stats;

/* Outcome of the round-by-round broadcast simulation (Algorithm 1). */
typedef struct {
    uint32_t flags;               /* bit0 dup recv, bit1 unheld send, bit2 edge
                                     mismatch, bit3 incomplete rank           */
    uint32_t rounds;              /* communication rounds executed           */
    uint64_t n_bad_recv_dup;      /* (round, receiver) pairs: block already held */
    uint64_t n_bad_send_unheld;   /* (round, sender) pairs: block not yet held   */
    uint64_t n_edge_mismatch;     /* (round, receiver) pairs: recv != sender's send */
    uint64_t n_incomplete_ranks;  /* ranks missing a block at the end        */
    uint64_t first_bad;           /* min over failures of round<<32 | physical
                                     rank; UINT64_MAX if none                */
} orc_verdict;

/* q = ceil(log2 p), by integers only; -1 if p < 1. */
int orc_q(int64_t p);

/* Algorithm 2: skip[q] = p, skip[k-1] = skip[k] - skip[k]/2.  Writes q+1
 * entries, returns q (or -1). */
int orc_skips(int64_t p, int64_t *skip);

/* Algorithm 3: baseblock of rank r (root 0); q for r = 0. */
int orc_baseblock(int64_t p, int64_t r);

/* Algorithm 5 (which calls Algorithm 4): receive schedule of rank r for
 * root 0.  recv gets q entries in [-q, q-1].  stats may be NULL.
 * Returns the number of entries the search produced (q when all is well). */
int orc_recvschedule(int64_t p, int64_t r, int32_t *recv, orc_recv_stats *stats);

/* Send schedule by its definition (Section 2.2, the sentence that defines
 * sendblock[k]_r as recvblock[k] of the to-processor; Condition 2):
 * q calls of orc_recvschedule. */
int orc_sendschedule_def(int64_t p, int64_t r, int32_t *send);

/* Algorithm 6: send schedule in O(q) with at most a few "violations", each
 * resolved by one receive schedule of the to-processor.  violations and
 * viol_mask (bit k set when round k was a violation) may be NULL. */
int orc_sendschedule(int64_t p, int64_t r, int32_t *send, int *violations,
                     uint32_t *viol_mask);

/* Schedules for physical ranks [r_begin, r_end) with the given root
 * (Section 2: renumber by subtracting the root modulo p).  Entry (r,k) goes
 * to recv[(r-r_begin)*ld + k] and send[(r-r_begin)*ld + k].
 * send_mode 0: send by definition (tier 1).  send_mode 1: Algorithm 6 (tier 2).
 * threads <= 1: sequential; otherwise an OpenMP loop over ranks. */
int orc_schedules(int64_t p, int64_t root, int64_t r_begin, int64_t r_end,
                  int32_t *recv, int32_t *send, int64_t ld, int send_mode,
                  int threads);

/* Same for an arbitrary list of m physical ranks; row j = {recv[0..q-1],
 * send[0..q-1]} at out + j*2q. */
int orc_schedules_ranks(int64_t p, int64_t root, const uint32_t *ranks,
                        int64_t m, int32_t *out, int send_mode, int threads);

/* Digest and invariant flags over physical ranks [r_begin, r_end).
 *
 * Hash (a definition of this build): sm64 is the published SplitMix64 output
 * function.  Fields f_j = recv[j]+32 for j<q and send[j-q]+32 for q<=j<2q,
 * six bits each; words w_i = sum_{t<10} f_{10i+t} << 6t for i < ceil(2q/10);
 * h = sm64((p << 32) ^ r); then h = sm64(h ^ w_i) for each i in order.
 * digest = XOR of h over the ranks.
 *
 * Flags (OR over the ranks), each from the paper's correctness conditions:
 *  bit0 Condition 3 fails: {recv[k]} != ({-1..-q} minus {b-q}) plus {b}
 *       (root: a permutation of -1..-q);
 *  bit1 send[0] != b-q (root: send[k] != k for some k);
 *  bit2 Condition 4 fails for a non-root: some send[k], k>=1, is neither b-q
 *       nor one of recv[0..k-1];
 *  bit3 Algorithm 6 met more than 4 violations (send_mode 1 only);
 *  bit4 the receive search produced fewer than q entries;
 *  bit5 an entry lies outside [-q, q-1].
 */
int orc_digest(int64_t p, int64_t root, int64_t r_begin, int64_t r_end,
               uint64_t *digest, uint32_t *flags, int send_mode, int threads);

/* The hash primitive alone, so that tests can hold it against the published
 * SplitMix64 output sequence. */
uint64_t orc_sm64(uint64_t z);

/* Digest of one given row (same hash and flags), for known-answer tests and
 * for planting mistakes on the CPU.  viol_count feeds bit3; produced feeds bit4. */
int orc_digest_row(int64_t p, int64_t root, int64_t r, const int32_t *recv,
                   const int32_t *send, int viol_count, int produced,
                   uint64_t *hash, uint32_t *flags);

/* Conditions 1 and 2 over a rank range without a table (a definition of this
 * build).  Every rank r contributes, for each round k,
 *     xor_recv ^= g(r, k, recv[k]_r)      what r expects to receive in round k
 *     xor_send ^= g(t, k, send[k]_r)      what r sends to t = (r + skip[k]) mod p
 * with g(rank, k, val) = sm64(rank << 11 | k << 6 | (val + 32)).  Over ALL ranks
 * of an instance the two multisets of (rank, k, block) triples are equal exactly
 * when every receive entry matches the send entry of its from-processor, so
 * the two XORs must then be equal; ranges combine by XOR. */
int orc_edgecheck(int64_t p, int64_t root, int64_t r_begin, int64_t r_end,
                  uint64_t *xor_recv, uint64_t *xor_send, int send_mode, int threads);

/* The same two XORs of a given table sched[p][2q] (all ranks, physical order). */
int orc_edgecheck_table(int64_t p, const int32_t *sched, uint64_t *xor_recv, uint64_t *xor_send);

/* Algorithm 1 with possession marks instead of payload: n blocks, root,
 * schedules sched[r*2q + k] = recv, sched[r*2q + q + k] = send for physical
 * rank r (raw entries, not yet shifted by x); sched == NULL recomputes them
 * (Algorithm 5 + 6).  Every round first checks all ranks against the state
 * before the round, then applies that round's receives. */
int orc_simulate(int64_t p, int64_t n, int64_t root, const int32_t *sched,
                 orc_verdict *verdict);

/* Reduction to the root by running the rounds of Algorithm 1 backwards with
 * all communication reversed (Section 2, observation on reduction), over "sent"
 * marks.  n_bad_recv_dup counts sends of a block already sent, n_bad_send_unheld
 * partial results that arrive after (or while) the block is sent on, the other
 * members as in orc_simulate; rounds carry their forward numbers. */
int orc_simulate_reduce(int64_t p, int64_t n, int64_t root, const int32_t *sched,
                        orc_verdict *verdict);

#ifdef __cplusplus
}
#endif
#endif

/*
 * bcast.h -- C ABI of the MI355X (gfx950) library that computes round-optimal
 * broadcast schedules on a circulant graph, after J. L. Traff, "Optimal
 * Broadcast Schedules in Logarithmic Time ..." (arXiv 2407.18004).
 *
 * Problem statement (Section 2): p processors 0..p-1, a root, n indivisible
 * blocks, n-1+q communication rounds with q = ceil(log2 p).  In round i every
 * processor r sends to (r + skip[k]) mod p and receives from (r - skip[k]) mod p
 * with k = i mod q.  Which block it receives and sends is given by two arrays
 * of q entries, recvblock[] and sendblock[], that each processor computes for
 * itself in O(q) steps.  This library computes them for many ranks at once,
 * one GPU lane per rank.
 *
 * Conventions for every entry point
 *  - "host" pointers are dereferenced by the calling thread, before the call
 *    returns; "device" pointers are only passed to kernels.  The caller owns
 *    every buffer and the stream; the library allocates nothing and keeps no
 *    state between calls.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued on it and the call returns without waiting; results are
 *    valid once the caller has synchronised the stream.
 *  - Return value: BCAST_OK, or a negative BCAST_E* code.  Nothing is thrown
 *    and nothing aborts.  Arguments are checked before anything is launched:
 *    on BCAST_EINVAL and BCAST_ENOMEM no kernel has run.  BCAST_EHIP means the
 *    HIP runtime refused a launch; kernels launched before it may have run.
 *  - Domain: 1 <= p <= 2^31 - 1, so q <= 31.  p = 1 has q = 0: rows are empty.
 *  - Schedule entries are the raw values of Algorithms 5 and 6, in [-q, q-1]:
 *    exactly one receive entry of a non-root rank is non-negative (its
 *    baseblock, Condition 3).  They are NOT shifted by the x dummy rounds of
 *    Algorithm 1; that shift belongs to whoever runs the rounds.
 *  - A root other than 0 renumbers the ranks: the schedule of physical rank r
 *    is the root-0 schedule of (r - root + p) mod p (Section 2).
 */
#ifndef BCAST_H
#define BCAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BCAST_OK       0
#define BCAST_EINVAL  (-1)  /* argument outside the documented domain          */
#define BCAST_ENOMEM  (-2)  /* workspace smaller than bcast_simulate_workspace */
#define BCAST_EHIP    (-3)  /* the HIP runtime refused a launch or a copy      */

#define BCAST_MAX_P   2147483647u
#define BCAST_MAX_N   268435456u   /* blocks in bcast_simulate: 2^28 (the rounds run on 32-bit block numbers) */

/* Flags of bcast_schedules_digest, OR-ed over the ranks (Section 2, the four
 * correctness conditions, and Theorem 3). */
#define BCAST_F_COND3      (1u << 0) /* recv[] is not ({-1..-q} minus {b-q}) plus {b}   */
#define BCAST_F_SEND0      (1u << 1) /* send[0] != b-q (root: send[k] != k)             */
#define BCAST_F_COND4      (1u << 2) /* a send[k] is neither b-q nor an earlier recv[j] */
#define BCAST_F_VIOLATIONS (1u << 3) /* more than four violations in Algorithm 6        */
#define BCAST_F_SEARCH     (1u << 4) /* the receive search ended early or left its
                                        expected shape (explained at recv_search in the source) */
#define BCAST_F_RANGE      (1u << 5) /* an entry outside [-q, q-1]                      */

/* Flags of bcast_verdict.flags. */
#define BCAST_V_RECV_DUP     (1u << 0)
#define BCAST_V_SEND_UNHELD  (1u << 1)
#define BCAST_V_EDGE         (1u << 2)
#define BCAST_V_INCOMPLETE   (1u << 3)

/* Outcome of one simulated broadcast (Algorithm 1 over possession bits).
 * All members are order-independent reductions over (round, rank) events. */
typedef struct bcast_verdict {
    uint32_t flags;               /* BCAST_V_* */
    uint32_t rounds;              /* rounds executed: n-1+q (0 for p = 1)        */
    uint64_t n_bad_recv_dup;      /* receives of a block already held            */
    uint64_t n_bad_send_unheld;   /* sends of a block not held before the round  */
    uint64_t n_edge_mismatch;     /* receiver's block != its from-processor's    */
    uint64_t n_incomplete_ranks;  /* ranks that miss a block after the last round */
    uint64_t first_bad;           /* min of (round << 32 | physical rank) over all
                                     failures, UINT64_MAX if none; a rank that is
                                     incomplete at the end counts as round = rounds */
} bcast_verdict;

/* q = ceil(log2 p) by integer arithmetic (Section 2).  Returns BCAST_EINVAL
 * for p = 0 or p > BCAST_MAX_P. */
int bcast_q(uint32_t p);

/* Algorithm 2: the skips of the circulant graph.  Writes skip[0..q] (q+1 values,
 * skip[q] = p, skip[k-1] = ceil(skip[k] / 2)) to the host array `skips`, which
 * must hold at least 32 entries, and q to *q_out (may be NULL).  Host only. */
int bcast_skips(uint32_t p, uint32_t *skips, int *q_out);

/* Algorithms 3, 5 (with 4) and 6 for the physical ranks r in [r_begin, r_end).
 * Device output, int32: entry (r, k), k < q, goes to
 *     recv[(r - r_begin) * ld + k]   and   send[(r - r_begin) * ld + k].
 * Two layouts take the coalesced path: one table [ranks][2q] (send == recv + q,
 * ld == 2q) and two tables [ranks][q] (ld == q, disjoint); any other ld >= q
 * with rows that do not overlap is served by a slower row-wise path.
 * Errors: p outside the domain, root >= p, r_begin > r_end, r_end > p, NULL
 * pointers (unless the range is empty or q = 0), ld < q, overlapping rows. */
int bcast_schedules(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                    int32_t *recv, int32_t *send, int64_t ld, void *stream);

/* The same computation folded into a digest instead of being stored, for
 * rank ranges too large to materialise.  Per rank, with sm64 the published
 * SplitMix64 output function and the 2q entries as six-bit fields
 * f_j = recv[j] + 32 (j < q), f_{q+j} = send[j] + 32:
 *     w_i = sum_{t<10} f_{10 i + t} << 6 t,            i < ceil(2q / 10)
 *     h   = sm64((p << 32) ^ r);  h = sm64(h ^ w_i) for i = 0, 1, ...
 * *digest (device, one uint64) = XOR of h over the ranks; *flags (device, one
 * uint32) = OR of the BCAST_F_* checks of every rank.  Both are overwritten.
 * Digests of disjoint ranges combine by XOR, flags by OR.  Errors as above. */
int bcast_schedules_digest(uint32_t p, uint32_t root, uint64_t r_begin,
                           uint64_t r_end, uint64_t *digest, uint32_t *flags,
                           void *stream);

/* Conditions 1 and 2 (every receive entry equals the send entry of its
 * from-processor) for rank ranges too large to materialise.  For each rank r of
 * the range and each round k, with g(rank, k, val) = sm64(rank << 11 | k << 6 |
 * (val + 32)):
 *     xors[0] ^= g(r, k, recv[k]_r)                       what r expects in round k
 *     xors[1] ^= g((r + skip[k]) mod p, k, send[k]_r)     what r sends, filed under its to-processor
 * xors (device, two uint64) is overwritten.  Results of disjoint ranges combine
 * by XOR; once they cover all p ranks of an instance, xors[0] == xors[1] holds
 * exactly when the two multisets of (rank, round, block) triples agree, i.e.
 * when both conditions hold on every edge (up to a 2^-64 hash collision).
 * Errors as for bcast_schedules_digest. */
int bcast_schedules_edgecheck(uint32_t p, uint32_t root, uint64_t r_begin,
                              uint64_t r_end, uint64_t *xors, void *stream);

/* bcast_schedules, bcast_schedules_digest and bcast_schedules_edgecheck with a
 * device workspace of at least bcast_schedules_workspace(p) bytes (164 KB of
 * tables and a list of about p bytes, at most 32 MB; contents irrelevant on
 * entry, overwritten): same arguments, same results, less work per rank.
 * The levels of Algorithms 3, 4 and 5 with the small skips (below 1,024) see
 * of a rank only what Algorithm 3 has left of it after the larger skips, a
 * number below 2,050, so that part of every rank's computation (the
 * baseblock, the first receive entries, the state in which the search of
 * Algorithm 4 goes on, the violations of Algorithm 6 in these rounds) is
 * computed once per such number, into the workspace, by a small kernel ahead
 * of the main one, and looked up by some p / 1,500 ranks each; violations of
 * Algorithm 6 are answered from the same table where the to-processor's entry
 * holds the round in question.  p below 16,384 has too few large skips, and
 * for ranges of fewer than 2^20 ranks the small kernel costs more than it
 * saves: then the tables are not used.  The list: entries of the send
 * schedule that the main kernel of bcast_schedules_ws cannot take from rows it
 * still holds are not searched for; their places are listed in the workspace,
 * and a last kernel copies each from the finished table (Section 2:
 * sendblock[k] of r is recvblock[k] of its to-processor), searching only for
 * to-processors outside the range of the call.  The workspace may be reused by
 * the next call on the same stream; calls that are in flight at the same time
 * (on different streams) need one each.  Errors as for the plain calls;
 * workspace NULL: BCAST_EINVAL; too small: BCAST_ENOMEM. */
size_t bcast_schedules_workspace(uint32_t p);
int bcast_schedules_ws(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                       int32_t *recv, int32_t *send, int64_t ld, void *workspace,
                       size_t workspace_bytes, void *stream);
int bcast_schedules_digest_ws(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                              uint64_t *digest, uint32_t *flags, void *workspace,
                              size_t workspace_bytes, void *stream);
int bcast_schedules_edgecheck_ws(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                                 uint64_t *xors, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* bcast_schedules_digest for every chunk of a rank range in one call: chunk i
 * holds the ranks r_begin + i * chunk_ranks up to (not including) the smaller
 * of r_begin + (i + 1) * chunk_ranks and r_end, and digests[i], flags[i]
 * (device arrays of ceil((r_end - r_begin) / chunk_ranks) elements, overwritten)
 * are what bcast_schedules_digest gives for that chunk.  One launch works
 * through the whole range, so the chunks do not each pay for the first tiles of
 * a launch and for its last wavefronts (the 32 chunks of 2^26 ranks of
 * p = 2^31 - 1: 55 ms in one call against 61 ms in 32).  chunk_ranks: a power
 * of two, at least 64.  workspace: as for bcast_schedules_digest_ws, or NULL
 * with workspace_bytes = 0 (then as bcast_schedules_digest).  Errors as for
 * bcast_schedules_digest; chunk_ranks not as described or more than 2^32
 * chunks: BCAST_EINVAL; a workspace that is too small: BCAST_ENOMEM. */
int bcast_schedules_digest_chunks(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                                  uint64_t chunk_ranks, uint64_t *digests, uint32_t *flags,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* Observations 1 and 5: the table for 2p processors from the table for p, both
 * for root 0.  `in` is a device table int32 [p][2q] (row r = recv then send of
 * rank r, as bcast_schedules writes it with ld = 2q), `out` a device table
 * int32 [2p][2(q+1)]; they must not overlap.  Rank r < p and rank r + p are
 * both derived from row r: negative entries drop by one, and a last round is
 * added (receive: -1 for r < p, the new block q for r = p, the rank's
 * non-negative block for r > p, which then leaves -1 behind; send: the rank's
 * baseblock for r < p; for r >= p every non-negative entry and the new one
 * are -1).  The result equals what bcast_schedules computes for 2p.  Pure
 * data movement: 8q bytes read and 16(q+1) bytes written per given rank.
 * Errors: p outside [1, (2^31-1)/2], NULL pointers (in may be NULL for p = 1),
 * overlapping tables. */
int bcast_schedules_double(uint32_t p, const int32_t *in, int32_t *out, void *stream);

/* The baseblocks of all p processors in linear time, as in the proof of
 * Lemma 4: starting from the list of one rank, the list for the first skip[k+1]
 * ranks is the list for the first skip[k] ranks followed by a copy of its first
 * skip[k+1] - skip[k] entries, with the root's entry raised to k + 1 afterwards
 * (0 -> 10 -> 201 -> 301201 -> ...).  list: device, p bytes, list[r] = b_r in
 * [0, q] (q for the root, as Algorithm 3 returns it).  One copy per skip, 2p
 * bytes moved in all; no search and no per-rank loop.  Errors: p outside the
 * domain, NULL. */
int bcast_baseblocks(uint32_t p, uint8_t *list, void *stream);

/* The whole table for root 0, int32 [p][2q] as bcast_schedules writes it with
 * ld = 2q, by Observations 1 and 5 wherever they apply: with p = m 2^j, m odd,
 * the table of m is computed by Algorithms 3, 5 and 6 and doubled j times
 * (bcast_schedules_double), so the O(p log p) search runs for p / 2^j ranks
 * only and the rest is data movement.  Odd p: the same as bcast_schedules.
 * workspace: device, at least bcast_schedules_doubling_workspace(p) bytes (the
 * tables of p/2 and p/4), contents irrelevant on entry, must not overlap out.
 * Errors: p outside the domain, NULL pointers, overlap; BCAST_ENOMEM when the
 * workspace is too small. */
size_t bcast_schedules_doubling_workspace(uint32_t p);
int bcast_schedules_doubling(uint32_t p, int32_t *out, void *workspace, size_t workspace_bytes,
                             void *stream);

/* Algorithms 3, 5 (with 4) and 6 for listed ranks of many instances at once (the
 * skips of Algorithm 2 per instance): instance i has p[i] processors, root[i]
 * (renumbering as in Section 2), and asks for the m physical ranks
 * ranks[i*m .. i*m+m).  Row j of instance i, 2*q(p[i]) int32
 * {recvblock[0..q-1], sendblock[0..q-1]} of that rank, is written at
 *     out[row_off[i] + j * 2*q(p[i])].
 * p, root, ranks, row_off (n_inst+1 prefix sums, in int32 elements) and out are
 * device arrays; out holds out_elems elements.  Nothing can be validated on
 * the host without a copy, so the kernel does it: an instance with p outside
 * the domain, root >= p, a row_off step other than m*2q, or rows beyond
 * out_elems writes nothing, and a rank >= p[i] gets a row of INT32_MIN; each
 * such instance or rank adds one to *n_rejected (device uint32, overwritten;
 * may be NULL).  Errors: NULL pointers, m = 0 with n_inst > 0. */
int bcast_schedules_batched(uint32_t n_inst, const uint32_t *p, const uint32_t *root,
                            const uint32_t *ranks, uint32_t m,
                            const uint64_t *row_off, int32_t *out,
                            uint64_t out_elems, uint32_t *n_rejected, void *stream);

/* Bytes of device workspace bcast_simulate and bcast_simulate_reduce need for
 * the replay of Algorithm 1 with n blocks from n_roots roots on p processors:
 * the roots, the schedule table of Algorithms 5 and 6 twice (by rows and by
 * columns, 8q bytes per processor each) and one possession bit per root,
 * processor and block.  0 when an argument is outside the domain documented at
 * bcast_simulate or the size does not fit size_t. */
size_t bcast_simulate_workspace(uint32_t p, uint32_t n, uint32_t n_roots);

/* Algorithm 1 (and, for several roots side by side, Algorithm 7) replayed over
 * possession bits: n blocks travel from each of the n_roots roots (host array
 * `roots`) through n-1+q rounds.  In every round each non-root rank that
 * expects a block checks that its from-processor sends that block and that
 * it does not hold it yet, each rank that sends checks that it held the block
 * before the round, and then the received block is marked.  Blocks < 0 are
 * neither sent nor received, blocks > n-1 count as n-1, nothing is sent to
 * the root.  After the last round every rank must hold all n blocks.
 * sched: device int32 [n_roots][p][2q] (row r = recv then send of physical
 * rank r for that root), or NULL to have the schedules computed here.
 * workspace: device, at least bcast_simulate_workspace bytes, contents
 * irrelevant on entry.  verdict: device, n_roots structs, overwritten.
 * Errors: domain of p, n = 0 or n > BCAST_MAX_N, n_roots = 0 or > 65535, a root >= p, NULL
 * pointers, workspace too small (BCAST_ENOMEM). */
int bcast_simulate(uint32_t p, uint32_t n, const uint32_t *roots, uint32_t n_roots,
                   const int32_t *sched, void *workspace, size_t workspace_bytes,
                   bcast_verdict *verdict, void *stream);

/* Reduction to the root over the same schedules (Section 2, the observation on
 * reduction): the rounds of Algorithm 1 from the last one down to the first,
 * with every communication reversed.  In reversed round i a non-root rank sends
 * its partial result for the block it would have received to its
 * from-processor and is then done with that block; it receives, from its
 * to-processor, a partial result for the block it would have sent.  Bits mean
 * "already sent on".  Checked: sender and receiver agree on the block; no block
 * is sent twice (counted in n_bad_recv_dup, flag BCAST_V_RECV_DUP); no partial
 * result arrives for a block that has been sent on, this round's send included
 * (n_bad_send_unheld, BCAST_V_SEND_UNHELD); at the end every non-root has sent
 * all n blocks (n_incomplete_ranks).  Rounds in first_bad carry their forward
 * numbers.  Arguments, workspace and errors exactly as for bcast_simulate. */
int bcast_simulate_reduce(uint32_t p, uint32_t n, const uint32_t *roots, uint32_t n_roots,
                          const int32_t *sched, void *workspace, size_t workspace_bytes,
                          bcast_verdict *verdict, void *stream);

/* bcast_simulate for callers that cannot allocate device memory and so cannot
 * bring a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The same replay with the same kernels; the
 * workspace is an array of BCAST_NOALLOC_SCRATCH_BYTES bytes that the library
 * holds in the memory of every GPU it is used on, from the first call on that
 * GPU until the process ends.  The call allocates and frees nothing and does
 * not wait.  Instances that need more (bcast_simulate_workspace(p, n, n_roots)
 * > BCAST_NOALLOC_SCRATCH_BYTES) are refused with BCAST_ENOMEM before anything
 * is launched: p = 65,537 with n = 256 and one root needs 20 MB and fits, the
 * same with 64 roots does not.  All calls on one GPU share the one array, which
 * keeps what the last call left in it (nothing in it has to be cleared between
 * calls); calls that overlap in time on one GPU, e.g. on two streams, race and
 * give undefined verdicts: order them.  Other arguments and errors as for
 * bcast_simulate; BCAST_EHIP also when the array's address cannot be had. */
#define BCAST_NOALLOC_SCRATCH_BYTES (32u * 1024u * 1024u)
int bcast_simulate_noalloc(uint32_t p, uint32_t n, const uint32_t *roots, uint32_t n_roots,
                           const int32_t *sched, bcast_verdict *verdict, void *stream);

/* Text for a return code; never NULL. */
const char *bcast_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif

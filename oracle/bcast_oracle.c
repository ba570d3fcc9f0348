/*
 * CPU oracle for round-optimal broadcast schedules (Träff, arXiv 2407.18004).
 * TEST INFRASTRUCTURE ONLY -- see bcast_oracle.h.  Plain sequential C, int64,
 * the paper's algorithms taken step by step in the paper's notation.
 */
#include "bcast_oracle.h"

#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- skips -- */

int orc_q(int64_t p)
{
    if (p < 1 || p >= ((int64_t)1 << ORC_MAXQ)) return -1;
    int q = 0;
    while (((int64_t)1 << q) < p) q++;      /* smallest q with 2^q >= p */
    return q;
}

/* Algorithm 2: from skip[q] = p downwards, every skip is the one above it
 * halved with rounding up (what is left after taking away the rounded-down
 * half). */
int orc_skips(int64_t p, int64_t *skip)
{
    int q = orc_q(p);
    if (q < 0) return -1;
    skip[q] = p;
    for (int k = q; k > 0; k--) {
        int64_t lower_half = skip[k] / 2;
        skip[k - 1] = skip[k] - lower_half;
    }
    return q;
}

/* ------------------------------------------------------------ baseblock -- */

/* Algorithm 3 on a given skip table.  For p = 1 (q = 0) the repeat loop has
 * no skip to look at; the only rank is the root and its baseblock is q. */
static int baseblock_sk(const int64_t *skip, int q, int64_t r)
{
    int64_t rp = 0;                       /* r': the skips taken so far */
    for (int k = q - 1; k >= 0; k--) {
        int64_t with_k = rp + skip[k];
        if (with_k == r) return k;        /* the sum closes on r: k is its smallest index */
        if (with_k < r) rp = with_k;      /* still short of r: the skip is part of the sequence */
    }
    return q;                             /* nothing closed: r = 0 */
}

int orc_baseblock(int64_t p, int64_t r)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || r < 0 || r >= p) return -1;
    return baseblock_sk(skip, q, r);
}

/* ------------------------------------------------- receive schedule ------ */

/* State shared by all recursive calls of Algorithm 4: the skips, the target
 * rank R = p + r, the doubly linked list of remaining skip indices in
 * decreasing order (index -1 is the list head, so the arrays are used with an
 * offset of one), and the output. */
typedef struct {
    const int64_t *skip;
    int q;
    int64_t R;
    int nextl[ORC_MAXQ + 3];   /* nextl[e+1] = next smaller remaining index */
    int prevl[ORC_MAXQ + 3];
    int linked[ORC_MAXQ + 3];  /* bookkeeping for the anomaly counter only  */
    int onpath[ORC_MAXQ + 3];  /* ditto                                      */
    int idx[ORC_MAXQ + 2];     /* accepted skip indices, in order of k      */
    orc_recv_stats st;
} recv_ctx;

#define NEXT(c, e) ((c)->nextl[(e) + 1])
#define PREV(c, e) ((c)->prevl[(e) + 1])

static void unlink_index(recv_ctx *c, int e)
{
    if (!c->linked[e + 1]) c->st.anomalies++;
    c->linked[e + 1] = 0;
    NEXT(c, PREV(c, e)) = NEXT(c, e);
    PREV(c, NEXT(c, e)) = PREV(c, e);
}

/* Algorithm 4: the depth-first search for processor R = p + r.  A call stands
 * at intermediate processor rp (r') and goes down the list of remaining skip
 * indices from e on.  R, rp, s and e belong to the call; the round k it has
 * got to is handed back as its result; idx[] and the list are common to all
 * calls.
 *
 * The one place the algorithm leaves open: once q indices are accepted there
 * is no skip[k+1] to compare with.  The list is empty by then and the loop
 * ends anyway; the test after a call that comes back with k = q is therefore
 * "return", and it counts as an anomaly if the call's own index were still in
 * the list (it never is). */
static int allblocks(recv_ctx *c, int64_t rp, int64_t s, int e, int k, int depth)
{
    const int64_t *skip = c->skip;
    const int64_t R = c->R;
    const int q = c->q;
    if (depth > c->st.max_depth) c->st.max_depth = depth;
    for (; e != -1; e = NEXT(c, e)) {
        c->st.scans++;
        if (k >= q) continue;                    /* nothing left to find; the list is empty */
        const int64_t via_e = rp + skip[e];      /* the processor one skip[e] further on */
        /* of use for round k: no later than the from-processor of that round,
         * and before the processor the round before settled on */
        if (!(via_e <= R - skip[k] && via_e < s)) continue;
        if (via_e <= R - skip[k + 1]) {          /* room to get closer from there */
            if (c->onpath[e + 1]) c->st.anomalies++;
            c->onpath[e + 1]++;
            c->st.calls++;
            k = allblocks(c, via_e, s, e, k, depth + 1);
            c->onpath[e + 1]--;
        }
        if (k >= q) {                            /* see above */
            if (c->linked[e + 1]) c->st.anomalies++;
            return k;
        }
        if (rp > R - skip[k + 1]) return k;      /* this call stands too far on for round k by now */
        s = via_e;                               /* via_e is r'_k ... */
        c->idx[k] = e;                           /* ... and e, the smallest index on the way there, its block */
        k = k + 1;
        unlink_index(c, e);
    }
    return k;
}

/* Algorithm 5 on a given skip table. */
static int recvschedule_sk(const int64_t *skip, int q, int64_t p, int64_t r,
                           int32_t *recv, orc_recv_stats *stats)
{
    recv_ctx c;
    memset(&c, 0, sizeof c);
    c.skip = skip;
    c.q = q;
    c.R = p + r;
    if (q == 0) {                     /* p = 1: empty schedule */
        if (stats) *stats = c.st;
        return 0;
    }
    for (int e = 0; e <= q; e++) {
        NEXT(&c, e) = e - 1;
        PREV(&c, e) = e + 1;
        c.linked[e + 1] = 1;
    }
    PREV(&c, q) = -1;
    NEXT(&c, -1) = q;
    PREV(&c, -1) = 0;
    c.linked[0] = 1;

    int b = baseblock_sk(skip, q, r);
    unlink_index(&c, b);

    for (int k = 0; k < q; k++) c.idx[k] = -1 - q;   /* "nothing stored" mark */
    int produced = allblocks(&c, 0, p + p, q, 0, 0);

    for (int k = 0; k < q; k++) {
        if (c.idx[k] == q) recv[k] = b;              /* the one non-negative block */
        else recv[k] = c.idx[k] - q;
    }
    if (stats) *stats = c.st;
    return produced;
}

int orc_recvschedule(int64_t p, int64_t r, int32_t *recv, orc_recv_stats *stats)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || r < 0 || r >= p) return -1;
    skip[q + 1] = 0;   /* never read: see the guard in allblocks */
    return recvschedule_sk(skip, q, p, r, recv, stats);
}

/* ---------------------------------------------------- send schedule ------ */

/* Definition: what r sends in round k is what its to-processor receives in
 * round k (Condition 2). */
static int sendschedule_def_sk(const int64_t *skip, int q, int64_t p, int64_t r,
                               int32_t *send)
{
    int32_t block[ORC_MAXQ + 1];
    for (int k = 0; k < q; k++) {
        int64_t t = (r + skip[k]) % p;
        recvschedule_sk(skip, q, p, t, block, NULL);
        send[k] = block[k];
    }
    return q;
}

int orc_sendschedule_def(int64_t p, int64_t r, int32_t *send)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || r < 0 || r >= p) return -1;
    return sendschedule_def_sk(skip, q, p, r, send);
}

/* Algorithm 6 on a given skip table. */
static int sendschedule_sk(const int64_t *skip, int q, int64_t p, int64_t r,
                           int32_t *send, int *violations, uint32_t *viol_mask)
{
    int nviol = 0;
    uint32_t vmask = 0;
    int32_t block[ORC_MAXQ + 1];
    if (r == 0) {
        for (int k = 0; k < q; k++) send[k] = k;
    } else {
        /* rp (r') is the rank within the range [0, e) that is still being
         * halved, c the block the rank means to send */
        int b = baseblock_sk(skip, q, r);
        int64_t rp = r, e = p;
        int32_t c = b;
        for (int k = q - 1; k >= 1; k--) {
            const int in_lower_half = rp < skip[k];
            int known;                       /* does the structure say what the to-processor lacks? */
            if (in_lower_half) {
                /* keeps sending c as long as the to-processor is inside the
                 * range, or the range is too small for it to have c */
                known = rp + skip[k] < e || e < skip[k - 1] || (k == 1 && b > 0);
            } else {
                c = k - q;
                known = k == 1 || rp > skip[k] || e - skip[k] < skip[k - 1] ||
                        !(rp + skip[k] > e);
            }
            if (known) {
                send[k] = c;
            } else {                         /* a violation: ask the to-processor's own schedule */
                recvschedule_sk(skip, q, p, (r + skip[k]) % p, block, NULL);
                send[k] = block[k];
                nviol++;
                vmask |= (uint32_t)1 << k;
            }
            if (in_lower_half) {
                if (e > skip[k]) e = skip[k];
            } else {
                rp = rp - skip[k];
                e = e - skip[k];
            }
        }
        if (q > 0) send[0] = b - q;
    }
    if (violations) *violations = nviol;
    if (viol_mask) *viol_mask = vmask;
    return q;
}

int orc_sendschedule(int64_t p, int64_t r, int32_t *send, int *violations,
                     uint32_t *viol_mask)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || r < 0 || r >= p) return -1;
    return sendschedule_sk(skip, q, p, r, send, violations, viol_mask);
}

/* ------------------------------------------------------ batch drivers ---- */

static int64_t virtual_rank(int64_t r, int64_t root, int64_t p)
{
    return (r - root + p) % p;       /* renumber so that the root is rank 0 */
}

int orc_schedules(int64_t p, int64_t root, int64_t r_begin, int64_t r_end,
                  int32_t *recv, int32_t *send, int64_t ld, int send_mode,
                  int threads)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || root < 0 || root >= p || r_begin < 0 || r_begin > r_end ||
        r_end > p || ld < q)
        return -1;
    skip[q + 1] = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static, 1024) num_threads(threads > 1 ? threads : 1)
#endif
    for (int64_t r = r_begin; r < r_end; r++) {
        int64_t v = virtual_rank(r, root, p);
        recvschedule_sk(skip, q, p, v, recv + (r - r_begin) * ld, NULL);
        if (send_mode == 0)
            sendschedule_def_sk(skip, q, p, v, send + (r - r_begin) * ld);
        else
            sendschedule_sk(skip, q, p, v, send + (r - r_begin) * ld, NULL, NULL);
    }
    return q;
}

int orc_schedules_ranks(int64_t p, int64_t root, const uint32_t *ranks,
                        int64_t m, int32_t *out, int send_mode, int threads)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || root < 0 || root >= p || m < 0) return -1;
    for (int64_t j = 0; j < m; j++)
        if ((int64_t)ranks[j] >= p) return -1;
    skip[q + 1] = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static, 256) num_threads(threads > 1 ? threads : 1)
#endif
    for (int64_t j = 0; j < m; j++) {
        int64_t v = virtual_rank((int64_t)ranks[j], root, p);
        int32_t *row = out + j * 2 * q;
        recvschedule_sk(skip, q, p, v, row, NULL);
        if (send_mode == 0)
            sendschedule_def_sk(skip, q, p, v, row + q);
        else
            sendschedule_sk(skip, q, p, v, row + q, NULL, NULL);
    }
    return q;
}

/* ------------------------------------------------------------- digest ---- */

/* Output function of SplitMix64 (Steele, Lea, Flood 2014), modulo 2^64. */
static uint64_t sm64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t orc_sm64(uint64_t z) { return sm64(z); }

static void digest_row_sk(const int64_t *skip, int q, int64_t p, int64_t root,
                          int64_t r, const int32_t *recv, const int32_t *send,
                          int viol_count, int produced, uint64_t *hash,
                          uint32_t *flags)
{
    int64_t v = virtual_rank(r, root, p);
    int b = baseblock_sk(skip, q, v);
    uint32_t fl = 0;

    /* hash */
    uint64_t h = sm64(((uint64_t)p << 32) ^ (uint64_t)r);
    int nfields = 2 * q;
    for (int i = 0; 10 * i < nfields; i++) {
        uint64_t w = 0;
        for (int t = 0; t < 10 && 10 * i + t < nfields; t++) {
            int j = 10 * i + t;
            int32_t val = j < q ? recv[j] : send[j - q];
            uint64_t f = (uint64_t)(val + 32) & 63u;
            w |= f << (6 * t);
        }
        h = sm64(h ^ w);
    }

    /* bit5: range */
    for (int k = 0; k < q; k++) {
        if (recv[k] < -q || recv[k] > q - 1) fl |= 1u << 5;
        if (send[k] < -q || send[k] > q - 1) fl |= 1u << 5;
    }

    /* bit0: Condition 3 as a multiset comparison */
    {
        int cnt[2 * ORC_MAXQ + 2];
        memset(cnt, 0, sizeof cnt);
        for (int k = 0; k < q; k++)
            if (recv[k] >= -q && recv[k] <= q - 1) cnt[recv[k] + q]++;
        int ok = 1;
        for (int val = -q; val <= q - 1; val++) {
            int want;
            if (v == 0) want = val < 0 ? 1 : 0;
            else if (val < 0) want = (val == b - q) ? 0 : 1;
            else want = (val == b) ? 1 : 0;
            if (cnt[val + q] != want) ok = 0;
        }
        if (!ok) fl |= 1u << 0;
    }

    /* bit1: first send */
    if (v == 0) {
        for (int k = 0; k < q; k++)
            if (send[k] != k) fl |= 1u << 1;
    } else if (q > 0 && send[0] != b - q) {
        fl |= 1u << 1;
    }

    /* bit2: Condition 4 for non-roots */
    if (v != 0) {
        for (int k = 1; k < q; k++) {
            int ok = (send[k] == b - q);
            for (int j = 0; j < k; j++)
                if (send[k] == recv[j]) ok = 1;
            if (!ok) fl |= 1u << 2;
        }
    }

    if (viol_count > 4) fl |= 1u << 3;
    if (produced != q) fl |= 1u << 4;

    *hash = h;
    *flags = fl;
}

int orc_digest_row(int64_t p, int64_t root, int64_t r, const int32_t *recv,
                   const int32_t *send, int viol_count, int produced,
                   uint64_t *hash, uint32_t *flags)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || q > 31 || root < 0 || root >= p || r < 0 || r >= p) return -1;
    digest_row_sk(skip, q, p, root, r, recv, send, viol_count, produced, hash, flags);
    return q;
}

int orc_digest(int64_t p, int64_t root, int64_t r_begin, int64_t r_end,
               uint64_t *digest, uint32_t *flags, int send_mode, int threads)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || q > 31 || root < 0 || root >= p || r_begin < 0 ||
        r_begin > r_end || r_end > p)
        return -1;
    skip[q + 1] = 0;
    uint64_t dg = 0;
    uint32_t fl = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static, 4096) reduction(^ : dg) reduction(| : fl) \
    num_threads(threads > 1 ? threads : 1)
#endif
    for (int64_t r = r_begin; r < r_end; r++) {
        int32_t recv[ORC_MAXQ + 1], send[ORC_MAXQ + 1];
        int64_t v = virtual_rank(r, root, p);
        int nviol = 0;
        int produced = recvschedule_sk(skip, q, p, v, recv, NULL);
        if (send_mode == 0)
            sendschedule_def_sk(skip, q, p, v, send);
        else
            sendschedule_sk(skip, q, p, v, send, &nviol, NULL);
        uint64_t h;
        uint32_t f;
        digest_row_sk(skip, q, p, root, r, recv, send, nviol, produced, &h, &f);
        dg ^= h;
        fl |= f;
    }
    *digest = dg;
    *flags = fl;
    return q;
}

/* --------------------------------------------------------- edge check ---- */

static uint64_t edge_hash(int64_t rank, int k, int32_t val)
{
    return sm64(((uint64_t)rank << 11) | ((uint64_t)k << 6) | ((uint64_t)(val + 32) & 63u));
}

static void edge_row(const int64_t *skip, int q, int64_t p, int64_t r, const int32_t *recv,
                     const int32_t *send, uint64_t *xr, uint64_t *xs)
{
    for (int k = 0; k < q; k++) {
        int64_t t = (r + skip[k]) % p;              /* to-processor of physical rank r */
        *xr ^= edge_hash(r, k, recv[k]);
        *xs ^= edge_hash(t, k, send[k]);
    }
}

int orc_edgecheck(int64_t p, int64_t root, int64_t r_begin, int64_t r_end,
                  uint64_t *xor_recv, uint64_t *xor_send, int send_mode, int threads)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || q > 31 || root < 0 || root >= p || r_begin < 0 || r_begin > r_end || r_end > p)
        return -1;
    skip[q + 1] = 0;
    uint64_t xr = 0, xs = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static, 4096) reduction(^ : xr, xs) \
    num_threads(threads > 1 ? threads : 1)
#endif
    for (int64_t r = r_begin; r < r_end; r++) {
        int32_t recv[ORC_MAXQ + 1], send[ORC_MAXQ + 1];
        int64_t v = virtual_rank(r, root, p);
        recvschedule_sk(skip, q, p, v, recv, NULL);
        if (send_mode == 0) sendschedule_def_sk(skip, q, p, v, send);
        else sendschedule_sk(skip, q, p, v, send, NULL, NULL);
        edge_row(skip, q, p, r, recv, send, &xr, &xs);
    }
    *xor_recv = xr;
    *xor_send = xs;
    return q;
}

int orc_edgecheck_table(int64_t p, const int32_t *sched, uint64_t *xor_recv, uint64_t *xor_send)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || q > 31 || !sched) return -1;
    uint64_t xr = 0, xs = 0;
    for (int64_t r = 0; r < p; r++)
        edge_row(skip, q, p, r, sched + r * 2 * q, sched + r * 2 * q + q, &xr, &xs);
    *xor_recv = xr;
    *xor_send = xs;
    return q;
}

/* ---------------------------------------------------------- simulator ---- */

static void note_bad(orc_verdict *vd, int64_t round, int64_t rank)
{
    uint64_t key = ((uint64_t)round << 32) | (uint64_t)rank;
    if (key < vd->first_bad) vd->first_bad = key;
}

int orc_simulate(int64_t p, int64_t n, int64_t root, const int32_t *sched,
                 orc_verdict *vd)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || n < 1 || root < 0 || root >= p || !vd) return -1;
    skip[q + 1] = 0;
    memset(vd, 0, sizeof *vd);
    vd->first_bad = UINT64_MAX;
    if (q == 0) return 0;            /* p = 1: the root has everything, no rounds */

    /* schedules by virtual rank: vs[v*2q + k] recv, vs[v*2q + q + k] send */
    int32_t *vs = (int32_t *)malloc((size_t)p * 2 * q * sizeof(int32_t));
    unsigned char *held = (unsigned char *)calloc((size_t)p * (size_t)n, 1);
    int64_t *mark_v = (int64_t *)malloc((size_t)p * sizeof(int64_t));
    int64_t *mark_b = (int64_t *)malloc((size_t)p * sizeof(int64_t));
    if (!vs || !held || !mark_v || !mark_b) {
        free(vs); free(held); free(mark_v); free(mark_b);
        return -2;
    }
    for (int64_t v = 0; v < p; v++) {
        int64_t r = (v + root) % p;
        if (sched) {
            memcpy(vs + v * 2 * q, sched + r * 2 * q, (size_t)2 * q * sizeof(int32_t));
        } else {
            recvschedule_sk(skip, q, p, v, vs + v * 2 * q, NULL);
            sendschedule_sk(skip, q, p, v, vs + v * 2 * q + q, NULL, NULL);
        }
    }
    for (int64_t j = 0; j < n; j++) held[j] = 1;       /* the root (v = 0) has all blocks */

    /* Algorithm 1: x dummy rounds are skipped; in round i the entry for
     * k = i mod q has been advanced by q once per earlier use, which gives
     * raw[k] - x + q*floor(i/q) in both cases of the adjustment loop. */
    int64_t x = (q - (n - 1) % q) % q;
    for (int64_t i = x; i <= (n + q - 1 + x) - 1; i++) {
        int k = (int)(i % q);
        int64_t shift = -x + (int64_t)q * (i / q);
        int64_t round = i - x;
        int64_t nmarks = 0;
        for (int64_t v = 0; v < p; v++) {
            int64_t r = (v + root) % p;
            int64_t t = (v + skip[k]) % p;
            int64_t f = (v - skip[k] + p) % p;
            if (v != 0) {                               /* nothing is sent to the root */
                int64_t rb = (int64_t)vs[v * 2 * q + k] + shift;
                int64_t sb = (int64_t)vs[f * 2 * q + q + k] + shift;
                int has_r = rb >= 0, has_s = sb >= 0;
                if (rb > n - 1) rb = n - 1;
                if (sb > n - 1) sb = n - 1;
                if (has_r != has_s || (has_r && rb != sb)) {
                    vd->n_edge_mismatch++;
                    vd->flags |= 1u << 2;
                    note_bad(vd, round, r);
                }
                if (has_r) {
                    if (held[v * n + rb]) {
                        vd->n_bad_recv_dup++;
                        vd->flags |= 1u << 0;
                        note_bad(vd, round, r);
                    } else {
                        mark_v[nmarks] = v;
                        mark_b[nmarks] = rb;
                        nmarks++;
                    }
                }
            }
            if (v != 0 && t != 0) {                     /* the root holds all it sends */
                int64_t sb = (int64_t)vs[v * 2 * q + q + k] + shift;
                if (sb >= 0) {
                    if (sb > n - 1) sb = n - 1;
                    if (!held[v * n + sb]) {
                        vd->n_bad_send_unheld++;
                        vd->flags |= 1u << 1;
                        note_bad(vd, round, r);
                    }
                }
            }
        }
        for (int64_t m = 0; m < nmarks; m++) held[mark_v[m] * n + mark_b[m]] = 1;
        vd->rounds++;
    }
    for (int64_t v = 0; v < p; v++) {
        int64_t have = 0;
        for (int64_t j = 0; j < n; j++) have += held[v * n + j];
        if (have != n) {
            vd->n_incomplete_ranks++;
            vd->flags |= 1u << 3;
            note_bad(vd, vd->rounds, (v + root) % p);
        }
    }
    free(vs); free(held); free(mark_v); free(mark_b);
    return 0;
}

/* Reduction by running the broadcast backwards (Section 2, the observation on
 * reduction): rounds from the last down to round x, all communication
 * reversed.  In reversed round i a non-root v sends its partial result for the
 * block it would have received, to its from-processor, and is then done with
 * that block; it receives, from its to-processor, a partial result for the
 * block it would have sent.  "Sent" marks take the place of possession marks:
 * a block may be sent once only, and a partial result that arrives when the
 * block has already been sent (this round's send included: send and receive
 * are simultaneous) would be lost.  At the end every non-root must have sent
 * all n blocks.  Verdict members: n_bad_recv_dup counts repeated sends,
 * n_bad_send_unheld counts lost arrivals, the others as in orc_simulate;
 * rounds are numbered as in the forward direction. */
int orc_simulate_reduce(int64_t p, int64_t n, int64_t root, const int32_t *sched,
                        orc_verdict *vd)
{
    int64_t skip[ORC_MAXQ + 2];
    int q = orc_skips(p, skip);
    if (q < 0 || n < 1 || root < 0 || root >= p || !vd) return -1;
    skip[q + 1] = 0;
    memset(vd, 0, sizeof *vd);
    vd->first_bad = UINT64_MAX;
    if (q == 0) return 0;
    int32_t *vs = (int32_t *)malloc((size_t)p * 2 * q * sizeof(int32_t));
    unsigned char *sent = (unsigned char *)calloc((size_t)p * (size_t)n, 1);
    if (!vs || !sent) { free(vs); free(sent); return -2; }
    for (int64_t v = 0; v < p; v++) {
        int64_t r = (v + root) % p;
        if (sched) {
            memcpy(vs + v * 2 * q, sched + r * 2 * q, (size_t)2 * q * sizeof(int32_t));
        } else {
            recvschedule_sk(skip, q, p, v, vs + v * 2 * q, NULL);
            sendschedule_sk(skip, q, p, v, vs + v * 2 * q + q, NULL, NULL);
        }
    }
    int64_t x = (q - (n - 1) % q) % q;
    for (int64_t i = (n + q - 1 + x) - 1; i >= x; i--) {
        int k = (int)(i % q);
        int64_t shift = -x + (int64_t)q * (i / q);
        int64_t round = i - x;
        /* first every send of this round, then every arrival */
        for (int64_t v = 1; v < p; v++) {
            int64_t r = (v + root) % p;
            int64_t f = (v - skip[k] + p) % p;
            int64_t rb = (int64_t)vs[v * 2 * q + k] + shift;       /* v sends this block to f */
            int64_t sb = (int64_t)vs[f * 2 * q + q + k] + shift;   /* f expects this block   */
            int has_r = rb >= 0, has_s = sb >= 0;
            if (rb > n - 1) rb = n - 1;
            if (sb > n - 1) sb = n - 1;
            if (has_r != has_s || (has_r && rb != sb)) {
                vd->n_edge_mismatch++;
                vd->flags |= 1u << 2;
                note_bad(vd, round, r);
            }
            if (has_r) {
                if (sent[v * n + rb]) {
                    vd->n_bad_recv_dup++;
                    vd->flags |= 1u << 0;
                    note_bad(vd, round, r);
                } else {
                    sent[v * n + rb] = 1;
                }
            }
        }
        for (int64_t v = 1; v < p; v++) {
            int64_t r = (v + root) % p;
            int64_t t = (v + skip[k]) % p;
            if (t == 0) continue;                      /* the root sends nothing */
            int64_t sb = (int64_t)vs[v * 2 * q + q + k] + shift;   /* arrives at v from t */
            if (sb >= 0) {
                if (sb > n - 1) sb = n - 1;
                if (sent[v * n + sb]) {
                    vd->n_bad_send_unheld++;
                    vd->flags |= 1u << 1;
                    note_bad(vd, round, r);
                }
            }
        }
        vd->rounds++;
    }
    for (int64_t v = 1; v < p; v++) {
        int64_t have = 0;
        for (int64_t j = 0; j < n; j++) have += sent[v * n + j];
        if (have != n) {
            vd->n_incomplete_ranks++;
            vd->flags |= 1u << 3;
            note_bad(vd, vd->rounds, (v + root) % p);
        }
    }
    free(vs); free(sent);
    return 0;
}

/*
 * CPU oracle for the Allgather schedules of the Sparbit paper.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow,
 * single-threaded p-rank message-passing simulation: every virtual rank runs
 * the paper's per-process program, posts non-blocking single-block sends and
 * receives, and a "wait-all" phase matches and delivers them.  It shares no
 * code, header, table or helper with the HIP library and neither includes the
 * other.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.
 *
 * What it simulates
 *   - MPI_Allgather post-condition (Section II): block of rank j ends in slot
 *     j of every rank's receive buffer.  oracle_naive_allgather() is that
 *     definition written out.  oracle_allgatherv() is the same simulation with
 *     per-rank block sizes and displacements (MPI_Allgatherv, the extension
 *     named in the paper's conclusion).
 *   - Sparbit (Section III-B, Algorithm 1): in every step each rank forwards
 *     the blocks it holds, nearest origin first, to the rank d ahead, and d
 *     halves.  How many it forwards follows from the blocks it really holds
 *     (counted from its buffer) and from the sub-tree rule of the section's
 *     prose: everything on a tree-expansion step and below the smallest
 *     sub-tree, all but the farthest-travelled block otherwise.
 *   - Ring, Recursive Doubling and Bruck as described in Section II-A
 *     (context schedules).
 *
 * Readings of the paper taken here (the paper is silent or garbled there):
 *   - Algorithm 1 tests "ignore_vector" but declares "ignore_steps": one and
 *     the same mask.
 *   - "rank + d % p" means (rank + d) mod p (Figure 3 text: wrap-around).
 *   - The loop runs ceil(log2 p) times (loop header and cost formula), not
 *     log2 p as one sentence of the prose says.
 *   - Algorithm 1 never places the rank's own block: it is put into slot
 *     `rank` before step 0 (required by the Allgather post-condition and by
 *     the Figure 3 text, where step 0 sends the "original block").  With a
 *     NULL send buffer the call is "in place": slot `rank` already holds it.
 *   - p = 1: zero steps, the result is the own block.
 *   - Displacements are reduced with a true mathematical modulo.
 *   - Each Isend/Irecv carries one block (count argument 1); a step's
 *     messages are all posted before any is delivered (Waitall), so sends see
 *     the pre-step buffer.  The simulation stages every payload in a mailbox
 *     between the two phases.
 *   - Ring: in step s rank r sends slot (r - s) mod p to r + 1 and receives
 *     slot (r - 1 - s) mod p from r - 1 (own block first, then the block
 *     received in the previous step).
 *   - Recursive Doubling: before step s rank r holds the aligned group of 2^s
 *     slots that contains r and exchanges that whole group with r xor 2^s.
 *   - Bruck: each rank works in a rotated buffer (working slot i holds block
 *     (r + i) mod p); in step s it sends its first min(2^s, p - 2^s) working
 *     slots to r - 2^s and appends what r + 2^s sends; a final local rotation
 *     by r restores rank order.  The paper names only the partner, the volume
 *     and the "memory shifts"; the layout is the textbook one: parity unpinned
 *     for Bruck's intermediate working-buffer layout (its final state, step
 *     count and per-step volume are pinned).
 *
 * Checks made while simulating (any violation aborts with an error code):
 *   - every posted send is matched by exactly one posted receive and vice
 *     versa, in posting order per (source, destination) pair;
 *   - a send never reads a slot that was not yet written;
 *   - a receive never lands in a slot that is already written or that is a
 *     send source in the same step (each of the p*p slots is written once);
 *   - for Sparbit the receiver's displacement equals the sender's.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_SPARBIT 0
#define ORACLE_RING 1
#define ORACLE_RECURSIVE_DOUBLING 2
#define ORACLE_BRUCK 3
#define ORACLE_NAIVE 4

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_NOMEM (-2)
#define ORACLE_ERR_UNMATCHED (-3)      /* a send or receive found no counterpart */
#define ORACLE_ERR_READ_UNWRITTEN (-4) /* a send read a slot nobody wrote yet */
#define ORACLE_ERR_DOUBLE_WRITE (-5)   /* a receive hit a slot already written */
#define ORACLE_ERR_READ_WRITE (-6)     /* slot both sent and received in one step */
#define ORACLE_ERR_SLOT_MISMATCH (-7)  /* Sparbit: send and receive displacement differ */
#define ORACLE_ERR_UNSUPPORTED (-8)    /* Recursive Doubling with p not a power of two */
#define ORACLE_ERR_TRACE_FULL (-9)

typedef struct {
    int peer;
    int slot;
} post_t;

typedef struct {
    int p;
    size_t row_bytes;      /* distance between two ranks' receive buffers */
    const size_t *off;     /* [p] byte offset of slot k inside a receive buffer */
    const size_t *len;     /* [p] bytes of slot k (uniform B for MPI_Allgather) */
    uint8_t *recv;         /* p receive buffers, caller's memory */
    uint8_t *written; /* p * p: 0 = poison, 1 = holds a block */
    uint8_t *sent_now; /* p * p: slot is a send source in the current step */
    post_t *sends;    /* [p][cap] in posting order */
    post_t *recvs;    /* [p][cap] */
    int *nsends, *nrecvs;
    int cap;
    int step;
    uint8_t *mailbox; /* payload staging of the current step, grown on demand */
    size_t mailbox_cap;
    /* optional trace, rows of 5 int32: step, src, dst, src_slot, dst_slot */
    int32_t *trace;
    size_t trace_cap, trace_len;
} sim_t;

static long long mod_ll(long long x, long long p)
{
    long long m = x % p;
    return m < 0 ? m + p : m;
}

static int ceil_log2_int(int p)
{
    int l = 0;
    while ((1LL << l) < (long long)p)
        l++;
    return l;
}

static uint8_t *slot_ptr(sim_t *s, int rank, int slot)
{
    return s->recv + (size_t)rank * s->row_bytes + s->off[slot];
}

static void post_isend(sim_t *s, int rank, int peer, int slot)
{
    post_t *q = &s->sends[(size_t)rank * s->cap + s->nsends[rank]++];
    q->peer = peer;
    q->slot = slot;
}

static void post_irecv(sim_t *s, int rank, int peer, int slot)
{
    post_t *q = &s->recvs[(size_t)rank * s->cap + s->nrecvs[rank]++];
    q->peer = peer;
    q->slot = slot;
}

/* Wait-all: phase 1 stages every posted send's payload (reading the pre-step
 * buffers), phase 2 delivers each posted receive from the oldest unconsumed
 * send of that source addressed to this rank. */
static int waitall(sim_t *s, int require_same_slot)
{
    const int p = s->p;
    size_t total = 0, payload = 0;
    int r, j;
    for (r = 0; r < p; r++) {
        total += (size_t)s->nsends[r];
        for (j = 0; j < s->nsends[r]; j++)
            payload += s->len[s->sends[(size_t)r * s->cap + j].slot];
    }
    if (total == 0) {
        for (r = 0; r < p; r++)
            if (s->nrecvs[r])
                return ORACLE_ERR_UNMATCHED;
        return ORACLE_OK;
    }
    uint8_t *mailbox;
    if (s->mailbox_cap < payload + 1) {
        free(s->mailbox);
        s->mailbox = (uint8_t *)malloc(payload + 1);
        s->mailbox_cap = s->mailbox ? payload + 1 : 0;
    }
    mailbox = s->mailbox;
    size_t *base = (size_t *)malloc((size_t)p * sizeof(size_t));
    size_t *where = (size_t *)malloc(total * sizeof(size_t)); /* mailbox offset of each staged message */
    uint8_t *consumed = (uint8_t *)calloc(total, 1);
    int *cursor = (int *)calloc((size_t)p, sizeof(int));
    int rc = ORACLE_OK;
    if (!mailbox || !base || !where || !consumed || !cursor) {
        rc = ORACLE_ERR_NOMEM;
        goto out;
    }
    memset(s->sent_now, 0, (size_t)p * p);
    {
        size_t k = 0, at = 0;
        for (r = 0; r < p; r++) {
            base[r] = k;
            for (j = 0; j < s->nsends[r]; j++, k++) {
                post_t *q = &s->sends[(size_t)r * s->cap + j];
                if (!s->written[(size_t)r * p + q->slot]) {
                    rc = ORACLE_ERR_READ_UNWRITTEN;
                    goto out;
                }
                s->sent_now[(size_t)r * p + q->slot] = 1;
                where[k] = at;
                memcpy(mailbox + at, slot_ptr(s, r, q->slot), s->len[q->slot]);
                at += s->len[q->slot];
            }
        }
    }
    for (r = 0; r < p; r++) {
        for (j = 0; j < s->nrecvs[r]; j++) {
            post_t *rq = &s->recvs[(size_t)r * s->cap + j];
            int src = rq->peer;
            int k, found = -1;
            while (cursor[src] < s->nsends[src] && consumed[base[src] + cursor[src]])
                cursor[src]++;
            for (k = cursor[src]; k < s->nsends[src]; k++) {
                if (!consumed[base[src] + k] &&
                    s->sends[(size_t)src * s->cap + k].peer == r) {
                    found = k;
                    break;
                }
            }
            if (found < 0) {
                rc = ORACLE_ERR_UNMATCHED;
                goto out;
            }
            consumed[base[src] + found] = 1;
            {
                int src_slot = s->sends[(size_t)src * s->cap + found].slot;
                if (require_same_slot && src_slot != rq->slot) {
                    rc = ORACLE_ERR_SLOT_MISMATCH;
                    goto out;
                }
                if (s->written[(size_t)r * p + rq->slot]) {
                    rc = ORACLE_ERR_DOUBLE_WRITE;
                    goto out;
                }
                if (s->sent_now[(size_t)r * p + rq->slot]) {
                    rc = ORACLE_ERR_READ_WRITE;
                    goto out;
                }
                if (s->len[src_slot] != s->len[rq->slot]) {
                    rc = ORACLE_ERR_SLOT_MISMATCH;
                    goto out;
                }
                memcpy(slot_ptr(s, r, rq->slot), mailbox + where[base[src] + found], s->len[rq->slot]);
                s->written[(size_t)r * p + rq->slot] = 1;
                if (s->trace) {
                    if (s->trace_len >= s->trace_cap) {
                        rc = ORACLE_ERR_TRACE_FULL;
                        goto out;
                    }
                    int32_t *t = s->trace + 5 * s->trace_len++;
                    t[0] = s->step;
                    t[1] = src;
                    t[2] = r;
                    t[3] = src_slot;
                    t[4] = rq->slot;
                }
            }
        }
    }
    {
        size_t k;
        for (k = 0; k < total; k++)
            if (!consumed[k]) {
                rc = ORACLE_ERR_UNMATCHED;
                goto out;
            }
    }
out:
    free(base);
    free(where);
    free(consumed);
    free(cursor);
    for (r = 0; r < p; r++)
        s->nsends[r] = s->nrecvs[r] = 0;
    return rc;
}

/* ---- Sparbit (Section III-B) --------------------------------------------------
 * The p binomial trees advance one level per step: the step with distance d
 * carries a block from every rank that holds it to the rank d further on.  A
 * tree over p ranks is made of power-of-two sub-trees, one per set bit of p,
 * largest first.  Whether a rank forwards everything it holds in a step, or
 * keeps back the one block that has nowhere left to go, is read off p's binary
 * representation as the section describes it:
 *   - d equal to a sub-tree size other than the smallest: a tree expansion,
 *     every held block is forwarded;
 *   - d below the smallest sub-tree: the distributions are local to complete
 *     power-of-two trees, every held block is forwarded;
 *   - any other d (no sub-tree of that size, or the smallest one): the block
 *     that travelled farthest arrived at a leaf and is kept back. */
static int sparbit_forwards_everything(int p, int d)
{
    int smallest_subtree = 1;
    while ((p & smallest_subtree) == 0)
        smallest_subtree <<= 1;
    if (d < smallest_subtree)
        return 1;
    if (d == smallest_subtree)
        return 0;
    return (p & d) != 0;
}

/* Blocks rank `rank` holds right now, counted from its receive buffer. */
static int blocks_held(const sim_t *s, int rank)
{
    int k, n = 0;
    for (k = 0; k < s->p; k++)
        n += s->written[(size_t)rank * s->p + k];
    return n;
}

/* One rank's postings for the step with distance d.  The blocks a rank holds
 * came from the ranks 0, d', 2d', ... behind it (d' = 2d, the previous
 * distance), so stripe j is the block of origin rank - 2jd, kept in the slot
 * of that number; at the receiver, d further on, it is the block from
 * (2j + 1) d behind.  The stripe kept back, if any, is the last one. */
static int sparbit_post_step(sim_t *s, int rank, int d)
{
    const int p = s->p;
    const int keep_back = sparbit_forwards_everything(p, d) ? 0 : 1;
    const int stripes = blocks_held(s, rank) - keep_back;
    const int ahead = (int)mod_ll((long long)rank + d, p);
    const int behind = (int)mod_ll((long long)rank - d, p);
    int j;
    for (j = 0; j < stripes; j++) {
        const long long origin = (long long)rank - 2LL * j * d;
        post_isend(s, rank, ahead, (int)mod_ll(origin, p));
        post_irecv(s, rank, behind, (int)mod_ll(origin - d, p));
    }
    return keep_back;
}

/* Number of communication steps of a schedule (Section II-A cost formulas,
 * Algorithm 1 loop bound).  -1 if the schedule does not support p. */
int oracle_num_steps(int algo, int p)
{
    if (p < 1)
        return -1;
    switch (algo) {
    case ORACLE_SPARBIT:
    case ORACLE_BRUCK:
        return ceil_log2_int(p);
    case ORACLE_RING:
        return p - 1;
    case ORACLE_RECURSIVE_DOUBLING:
        return (p & (p - 1)) ? -1 : ceil_log2_int(p);
    case ORACLE_NAIVE:
        return 0;
    default:
        return -1;
    }
}

/* MPI_Allgather by definition (Section II): recv[r][k] = send[k]. */
int oracle_naive_allgather(int p, size_t B, const void *send, void *recv)
{
    int r, k;
    if (p < 1 || B == 0 || !send || !recv)
        return ORACLE_ERR_ARG;
    for (r = 0; r < p; r++)
        for (k = 0; k < p; k++)
            memcpy((uint8_t *)recv + ((size_t)r * p + k) * B, (const uint8_t *)send + (size_t)k * B, B);
    return ORACLE_OK;
}

/* The simulation proper.  Slot k of every receive buffer sits at byte off[k]
 * and holds len[k] bytes; rank r's receive buffer starts at r * row_bytes; the
 * send buffer is laid out like one receive buffer (rank r's block at off[r]).
 * `uniform_block` is the common block size when all slots have one (needed by
 * Bruck's rotated working buffer), else 0. */
static int run_schedule(int algo, int p, size_t row_bytes, const size_t *off, const size_t *len,
                        size_t uniform_block, const void *send, void *recv, int max_steps,
                        int32_t *step_info, int64_t *sent_per_rank, int32_t *trace,
                        size_t trace_cap, size_t *trace_len)
{
    sim_t s;
    int rc = ORACLE_OK, r, step, nsteps;
    int sparbit_d = 0, sparbit_kept_back = 0;
    int *bruck_have = NULL;

    nsteps = oracle_num_steps(algo, p);
    if (nsteps < 0)
        return (algo == ORACLE_RECURSIVE_DOUBLING) ? ORACLE_ERR_UNSUPPORTED : ORACLE_ERR_ARG;
    if (algo == ORACLE_BRUCK && !send)
        return ORACLE_ERR_ARG; /* the rotated working buffer has no in-place form */
    if (algo == ORACLE_BRUCK && !uniform_block)
        return ORACLE_ERR_UNSUPPORTED; /* rotated layout is defined for equal blocks only */

    memset(&s, 0, sizeof s);
    s.p = p;
    s.row_bytes = row_bytes;
    s.off = off;
    s.len = len;
    s.recv = (uint8_t *)recv;
    s.cap = p;
    s.trace = trace;
    s.trace_cap = trace_cap;
    s.written = (uint8_t *)calloc((size_t)p * p, 1);
    s.sent_now = (uint8_t *)calloc((size_t)p * p, 1);
    s.sends = (post_t *)malloc((size_t)p * s.cap * sizeof(post_t));
    s.recvs = (post_t *)malloc((size_t)p * s.cap * sizeof(post_t));
    s.nsends = (int *)calloc((size_t)p, sizeof(int));
    s.nrecvs = (int *)calloc((size_t)p, sizeof(int));
    bruck_have = (int *)calloc((size_t)p, sizeof(int));
    if (!s.written || !s.sent_now || !s.sends || !s.recvs || !s.nsends || !s.nrecvs || !bruck_have) {
        rc = ORACLE_ERR_NOMEM;
        goto out;
    }
    if (sent_per_rank)
        memset(sent_per_rank, 0, (size_t)p * sizeof(int64_t));

    /* own block: slot `rank` (working slot 0 for Bruck) */
    for (r = 0; r < p; r++) {
        int own = (algo == ORACLE_BRUCK) ? 0 : r;
        if (send)
            memcpy(slot_ptr(&s, r, own), (const uint8_t *)send + off[r], len[r]);
        s.written[(size_t)r * p + own] = 1;
        bruck_have[r] = 1;
    }

    if (max_steps < 0 || max_steps > nsteps)
        max_steps = nsteps;
    if (algo == ORACLE_SPARBIT && nsteps > 0)
        sparbit_d = 1 << (nsteps - 1); /* the first level of the trees spans half of 2^ceil(log2 p) */
    for (step = 0; step < max_steps; step++) {
        s.step = step;
        for (r = 0; r < p; r++) {
            int j;
            switch (algo) {
            case ORACLE_SPARBIT:
                sparbit_kept_back = sparbit_post_step(&s, r, sparbit_d);
                break;
            case ORACLE_RING:
                post_isend(&s, r, (int)mod_ll(r + 1, p), (int)mod_ll((long long)r - step, p));
                post_irecv(&s, r, (int)mod_ll(r - 1, p), (int)mod_ll((long long)r - 1 - step, p));
                break;
            case ORACLE_RECURSIVE_DOUBLING: {
                int w = 1 << step, peer = r ^ w;
                int mine = r & ~(w - 1), theirs = peer & ~(w - 1);
                for (j = 0; j < w; j++) {
                    post_isend(&s, r, peer, mine + j);
                    post_irecv(&s, r, peer, theirs + j);
                }
                break;
            }
            case ORACLE_BRUCK: {
                int w = 1 << step;
                int n = (w < p - w) ? w : p - w; /* min(2^s, p - 2^s) */
                for (j = 0; j < n; j++) {
                    post_isend(&s, r, (int)mod_ll((long long)r - w, p), j);
                    post_irecv(&s, r, (int)mod_ll((long long)r + w, p), bruck_have[r] + j);
                }
                bruck_have[r] += n;
                break;
            }
            }
            if (sent_per_rank)
                sent_per_rank[r] += s.nsends[r];
        }
        if (step_info) {
            int32_t *si = step_info + 3 * step;
            si[1] = 0;
            si[2] = s.nsends[0];
            switch (algo) {
            case ORACLE_SPARBIT:
                si[0] = sparbit_d;
                si[1] = sparbit_kept_back;
                break;
            case ORACLE_RING:
                si[0] = 1;
                break;
            default:
                si[0] = 1 << step;
                break;
            }
        }
        rc = waitall(&s, algo == ORACLE_SPARBIT);
        if (rc != ORACLE_OK)
            goto out;
        sparbit_d /= 2;
    }

    if (algo == ORACLE_BRUCK && max_steps == nsteps) {
        /* local memory shift: working slot i of rank r is block (r + i) mod p */
        const size_t B = uniform_block;
        uint8_t *row = (uint8_t *)malloc((size_t)p * B);
        if (!row) {
            rc = ORACLE_ERR_NOMEM;
            goto out;
        }
        for (r = 0; r < p; r++) {
            int i;
            memcpy(row, slot_ptr(&s, r, 0), (size_t)p * B);
            for (i = 0; i < p; i++)
                memcpy(slot_ptr(&s, r, (int)mod_ll((long long)r + i, p)), row + (size_t)i * B, B);
        }
        free(row);
    }
out:
    if (trace_len)
        *trace_len = s.trace_len;
    free(s.mailbox);
    free(s.written);
    free(s.sent_now);
    free(s.sends);
    free(s.recvs);
    free(s.nsends);
    free(s.nrecvs);
    free(bruck_have);
    return rc;
}

/*
 * MPI_Allgather: run `algo` for p ranks with blocks of B bytes.
 *   send      p blocks (rank r at byte r*B), or NULL for in-place: recv[r][r]
 *             already holds rank r's block.
 *   recv      p*p blocks, rank r's buffer at byte r*p*B.  Slots that are never
 *             written keep whatever the caller put there (poison).
 *   max_steps run only the first max_steps communication steps (negative =
 *             all).  Bruck's final rotation happens only when all steps ran.
 *   step_info optional, [num_steps][3] int32: per step the distance d, the
 *             ignore flag (Sparbit; 0 otherwise) and the number of blocks rank
 *             0 sent.
 *   sent_per_rank optional, [p] int64: total blocks each rank sent.
 *   trace     optional, rows of 5 int32 (step, src, dst, src_slot, dst_slot),
 *             one per delivered message; trace_cap rows available, *trace_len
 *             receives the number written.
 * Returns ORACLE_OK or a negative ORACLE_ERR_* code.
 */
int oracle_allgather(int algo, int p, size_t B, const void *send, void *recv, int max_steps,
                     int32_t *step_info, int64_t *sent_per_rank, int32_t *trace, size_t trace_cap,
                     size_t *trace_len)
{
    size_t *off, *len;
    int k, rc;
    if (p < 1 || B == 0 || !recv)
        return ORACLE_ERR_ARG;
    if (algo == ORACLE_NAIVE)
        return oracle_naive_allgather(p, B, send, recv);
    off = (size_t *)malloc((size_t)p * sizeof(size_t));
    len = (size_t *)malloc((size_t)p * sizeof(size_t));
    if (!off || !len) {
        free(off);
        free(len);
        return ORACLE_ERR_NOMEM;
    }
    for (k = 0; k < p; k++) {
        off[k] = (size_t)k * B;
        len[k] = B;
    }
    rc = run_schedule(algo, p, (size_t)p * B, off, len, B, send, recv, max_steps, step_info,
                      sent_per_rank, trace, trace_cap, trace_len);
    free(off);
    free(len);
    return rc;
}

/*
 * MPI_Allgatherv over the same schedules (the extension the paper's
 * conclusion names): rank k contributes counts[k] bytes (zero allowed), which
 * land at byte displs[k] of every receive buffer; receive buffers are
 * row_bytes apart; the send buffer is laid out like one receive buffer (rank
 * r's block at displs[r]) or NULL for in place.  Bytes of a receive buffer
 * that belong to no block are never touched.  Bruck is not defined here (its
 * rotated buffer assumes equal blocks).  ORACLE_NAIVE gives the definition.
 */
int oracle_allgatherv(int algo, int p, const size_t *counts, const size_t *displs, size_t row_bytes,
                      const void *send, void *recv, int max_steps, int32_t *step_info,
                      int64_t *sent_per_rank, int32_t *trace, size_t trace_cap, size_t *trace_len)
{
    int r, k;
    if (p < 1 || !counts || !displs || !recv)
        return ORACLE_ERR_ARG;
    for (k = 0; k < p; k++)
        if (displs[k] + counts[k] > row_bytes)
            return ORACLE_ERR_ARG;
    if (algo == ORACLE_NAIVE) {
        if (!send)
            return ORACLE_ERR_ARG;
        for (r = 0; r < p; r++)
            for (k = 0; k < p; k++)
                memcpy((uint8_t *)recv + (size_t)r * row_bytes + displs[k],
                       (const uint8_t *)send + displs[k], counts[k]);
        return ORACLE_OK;
    }
    return run_schedule(algo, p, row_bytes, displs, counts, 0, send, recv, max_steps, step_info,
                        sent_per_rank, trace, trace_cap, trace_len);
}

const char *oracle_strerror(int code)
{
    switch (code) {
    case ORACLE_OK:
        return "ok";
    case ORACLE_ERR_ARG:
        return "bad argument";
    case ORACLE_ERR_NOMEM:
        return "out of host memory";
    case ORACLE_ERR_UNMATCHED:
        return "a send or receive has no counterpart";
    case ORACLE_ERR_READ_UNWRITTEN:
        return "a send reads a slot that was never written";
    case ORACLE_ERR_DOUBLE_WRITE:
        return "a receive lands in a slot that is already written";
    case ORACLE_ERR_READ_WRITE:
        return "a slot is sent and received in the same step";
    case ORACLE_ERR_SLOT_MISMATCH:
        return "Sparbit: receive displacement differs from send displacement";
    case ORACLE_ERR_UNSUPPORTED:
        return "schedule does not support this number of ranks";
    case ORACLE_ERR_TRACE_FULL:
        return "trace buffer too small";
    default:
        return "unknown oracle error";
    }
}

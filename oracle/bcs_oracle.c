/*
 * bcs_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow CPU statement of the round-optimal broadcast schedule
 * construction on a p-processor circulant graph (Traff, arXiv 2205.10072,
 * Section 2).  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.  It shares no code with the HIP library and neither side
 * includes the other.
 *
 * Every function follows one passage of the paper, named in its comment.
 * Where the paper leaves a gap the reading taken is stated next to the code.
 *
 * Pins (tests/, CPU only): the five printed tables (Tables 1-5), the printed
 * skips, brute-force scanning of rank ranges for every p <= 2048, the power
 * of two closed form, the row-permutation property (Section 2, end) and an
 * independent round-by-round broadcast simulator.
 *
 * Conventions that are not the paper's: the expand sentinel -1 ("no block
 * this round") and the batch layout (row stride 32, padding INT32_MIN).
 *
 * All entry points return 0 (or a non-negative value) on success and a
 * negative code on failure; nothing here aborts the process.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_EINVAL   (-1)   /* argument outside its domain                 */
#define ORC_ENOBLOCK (-2)   /* Alg. 4 found no new block in either range   */
#define ORC_ELAST    (-3)   /* Alg. 4: {0..q-1} \ B not a singleton at q-1 */
#define ORC_ENOMEM   (-4)

#define ORC_MAXQ 31
#define ORC_BATCH_STRIDE 32

/* q = ceil(log2 p) (Section 2, first paragraph); p = 1 gives 0. */
int orc_q(int32_t p)
{
    if (p < 1) return ORC_EINVAL;
    int q = 0;
    while (((int64_t)1 << q) < (int64_t)p) q++;
    return q;
}

/* Alg. 1: skips[q] = p, then repeated ceil-halving down to skips[0] = 1.
 * skips must have room for q+1 entries.  Returns q. */
int orc_skips(int32_t p, int32_t *skips)
{
    int q = orc_q(p);
    if (q < 0) return q;
    skips[q] = p;
    for (int k = q; k > 0; k--) skips[k - 1] = (int32_t)(((int64_t)skips[k] + 1) / 2);
    return q;
}

/* Alg. 2: baseblock of rank r, 0 < r < p.  Go down the skips from the largest
 * below p; a skip that is still below r is taken off r (r moves into the
 * lower copy of the pattern); the level at which r then sits on the skip is
 * the baseblock.  Level 0 always ends it: r has come down to skips[0] = 1. */
static int baseblock_alg2(const int32_t *skips, int q, int32_t r)
{
    for (int k = q - 1; k > 0; k--) {
        if (skips[k] < r) r -= skips[k];
        if (r == skips[k]) return k;
    }
    return 0;
}

int orc_baseblock(int32_t p, int32_t r)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 2 || r <= 0 || r >= p) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    return baseblock_alg2(skips, q, r);
}

/* Section 2, paragraph after Alg. 2: the linear-time list of baseblocks got
 * by replaying the first q rounds.  In round i the root hands block i to rank
 * skips[i]; every rank 1 <= r < skips[i] forwards its baseblock to
 * r + skips[i] when that is below skips[i+1].  bb[0] = -1: the root has no
 * baseblock (the tables print 0 or -1 there; it is never used). */
int orc_baseblocks_linear(int32_t p, int32_t *bb)
{
    int32_t skips[ORC_MAXQ + 2];
    int q = orc_skips(p, skips);
    if (q < 0) return q;
    bb[0] = -1;
    for (int i = 0; i < q; i++) {
        if (skips[i] < p) bb[skips[i]] = i;
        for (int32_t r = 1; r < skips[i]; r++) {
            int64_t t = (int64_t)r + skips[i];
            if (t < skips[i + 1]) bb[t] = bb[r];
        }
    }
    return q;
}

/* RangeBlocks by its definition (Section 2, paragraph before Alg. 4: the
 * baseblocks that occur among the ranks of a range): the set
 * { bb[j mod p] : a <= j <= b, j mod p != 0 } as a bit mask.  a and b are
 * plain integers and may be negative (the text after Alg. 4 writes the
 * ranges without their mod p); empty when a > b.
 * Needs the full bb[] list, so it is for small p only. */
uint32_t orc_rangeblocks_scan(int32_t p, const int32_t *bb, int64_t a, int64_t b)
{
    uint32_t m = 0;
    for (int64_t j = a; j <= b; j++) {
        int64_t jm = ((j % p) + p) % p;
        if (jm != 0) m |= (uint32_t)1 << bb[jm];
    }
    return m;
}

/* RangeBlocks for 1 <= a <= b < skips[k+1], without the bb[] list.  The
 * printed Alg. 3 is not followed (its shift index disagrees with its own
 * text and its small-k exceptions are never given).  This uses only the
 * self-similarity stated after Alg. 2: bb[skips[k]] = k, and the baseblocks
 * of skips[k]+1 .. skips[k+1]-1 repeat those of 1 .. skips[k+1]-skips[k]-1.
 *   - range entirely below skips[k]: same question one level down;
 *   - range entirely above skips[k]: shift it down by skips[k];
 *   - range containing skips[k]: block k, plus the part below, plus the part
 *     above shifted down.
 * A range that starts at rank 1 and reaches skips[k] holds skips[0..k], whose
 * baseblocks are 0..k, and nothing larger: that closes the recursion on the
 * "part above" side: a query makes O(q) calls, each with a short scan of the
 * skips. */
static uint32_t rangeblocks_rec(const int32_t *skips, int64_t a, int64_t b, int k)
{
    if (a > b) return 0;
    while (b < skips[k]) k = k - 1;
    /* now skips[k] <= b < skips[k+1] */
    if (a == 1) return ((uint32_t)2 << k) - 1;          /* {0..k} */
    if (a > skips[k])
        return rangeblocks_rec(skips, a - skips[k], b - skips[k], k - 1);
    uint32_t m = (uint32_t)1 << k;
    m |= rangeblocks_rec(skips, a, (int64_t)skips[k] - 1, k - 1);
    m |= rangeblocks_rec(skips, 1, b - skips[k], k - 1);
    return m;
}

/* RangeBlocks for integer a <= b (cyclic, rank 0 contributes nothing):
 * reduce to at most two plain ranges inside [1, p-1]. */
static uint32_t rangeblocks_fast(const int32_t *skips, int q, int64_t a, int64_t b)
{
    int64_t p = skips[q];
    if (a > b || p < 2) return 0;
    if (b - a + 1 >= p) return rangeblocks_rec(skips, 1, p - 1, q - 1);
    int64_t lo = ((a % p) + p) % p;
    int64_t hi = lo + (b - a);
    uint32_t m = 0;
    if (hi < p) {
        if (lo == 0) lo = 1;
        m = rangeblocks_rec(skips, lo, hi, q - 1);
    } else {
        if (lo == 0) lo = 1;
        m = rangeblocks_rec(skips, lo, p - 1, q - 1);
        m |= rangeblocks_rec(skips, 1, hi - p, q - 1);
    }
    return m;
}

uint32_t orc_rangeblocks(int32_t p, int64_t a, int64_t b)
{
    int32_t skips[ORC_MAXQ + 2];
    int q = orc_skips(p, skips);
    if (q < 0) return 0;
    return rangeblocks_fast(skips, q, a, b);
}

static int highest_bit(uint32_t m)
{
    int b = -1;
    while (m) { b++; m >>= 1; }
    return b;
}

/* Alg. 4: entries 0 .. min(k, q-1) of the receive schedule of rank r.
 *
 * Readings:
 *  - B starts as {baseblock(r)} for r > 0 (empty for the root): the row must
 *    hold the baseblock once and q-1 other blocks (Section 2, end), which the
 *    printed "B <- empty" cannot give.
 *  - the loop fills index i for i = 0..k; a full row is k = q-1 (or q).
 *  - ranges are over plain integers, ranks taken mod p; the root owns no
 *    baseblock and adds nothing to a range.
 *  - the upper summation index of the second range is i.
 *  - of several candidate blocks the largest is taken.
 *
 * general_only = 0: the printed special cases (i = 0 looks at rank r-1 alone;
 * i = q-1 takes the one block left).  general_only = 1: the range rule in
 * every round; tests check that both give the same row.
 *
 * bb != NULL: ranges by scanning bb[] (the definition).  bb == NULL: ranges by
 * the O(q) routine above and baseblocks by Alg. 2. */
static int recvsched_core(const int32_t *skips, int q, int32_t r, int k,
                          const int32_t *bb, int general_only, int32_t *out)
{
    int32_t p = skips[q];
    int own = -1;
    if (r > 0) own = bb ? bb[r] : baseblock_alg2(skips, q, r);
    uint32_t B = (r > 0) ? ((uint32_t)1 << own) : 0;
    uint32_t all = (q >= 32) ? 0xffffffffu : (((uint32_t)1 << q) - 1);
    int last = (k < q - 1) ? k : q - 1;
    int64_t prefix = 0;                       /* sum_{j<=i} skips[j] */
    for (int i = 0; i <= last; i++) {
        prefix += skips[i];
        if (skips[i] <= r && r < skips[i + 1]) {
            out[i] = own;
            continue;
        }
        int b;
        if (!general_only && i == 0) {
            int32_t prev = (int32_t)(((int64_t)r - 1 + p) % p);
            if (prev == 0) return ORC_ENOBLOCK;
            b = bb ? bb[prev] : baseblock_alg2(skips, q, prev);
        } else if (general_only || i < q - 1) {
            int64_t a1 = (int64_t)r - skips[i + 1] + 1, b1 = (int64_t)r - skips[i];
            uint32_t U = bb ? orc_rangeblocks_scan(p, bb, a1, b1)
                            : rangeblocks_fast(skips, q, a1, b1);
            U &= ~B;
            if (U == 0) {
                int64_t a2 = (int64_t)r - prefix, b2 = (int64_t)r - skips[i + 1];
                U = bb ? orc_rangeblocks_scan(p, bb, a2, b2)
                       : rangeblocks_fast(skips, q, a2, b2);
                U &= ~B;
            }
            if (U == 0) return ORC_ENOBLOCK;
            b = highest_bit(U);
        } else {
            uint32_t rest = all & ~B;
            if (rest == 0 || (rest & (rest - 1)) != 0) return ORC_ELAST;
            b = highest_bit(rest);
        }
        B |= (uint32_t)1 << b;
        out[i] = b - q;
    }
    return 0;
}

/* Alg. 4 through the public door.  mode bit 0: general rule in every round;
 * mode bit 1: ranges by scanning (allocates and fills bb[] first). */
int orc_recvsched(int32_t p, int32_t r, int k, int mode, int32_t *out)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1 || r < 0 || r >= p || k < 0) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    if (q == 0) return 0;
    if (mode & 2) {
        int32_t *bb = (int32_t *)malloc(sizeof(int32_t) * (size_t)p);
        if (!bb) return ORC_ENOMEM;
        orc_baseblocks_linear(p, bb);
        int rc = recvsched_core(skips, q, r, k, bb, mode & 1, out);
        free(bb);
        return rc;
    }
    return recvsched_core(skips, q, r, k, NULL, mode & 1, out);
}

/* Alg. 5: send schedule of one rank with no other rank's row at hand:
 * entry i is entry i of the first i+1 receive entries of the to-neighbour
 * (r + skips[i]) mod p. */
static int sendsched_alg5(const int32_t *skips, int q, int32_t r, int32_t *out)
{
    int32_t tmp[ORC_MAXQ + 1];
    int32_t p = skips[q];
    for (int i = 0; i < q; i++) {
        int32_t t = (int32_t)(((int64_t)r + skips[i]) % p);
        int rc = recvsched_core(skips, q, t, i, NULL, 0, tmp);
        if (rc) return rc;
        out[i] = tmp[i];
    }
    return 0;
}

int orc_sendsched(int32_t p, int32_t r, int32_t *out)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1 || r < 0 || r >= p) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    return sendsched_alg5(skips, q, r, out);
}

/* All-ranks tables, small p, everything from the definitions: baseblocks by
 * the linear recipe, ranges by scanning, Alg. 4 per rank, then the send table
 * by the neighbour look-up of Alg. 9 (its first two loops):
 * send[j][k] = recv[(j + skips[k]) mod p][k].  Rank-major, q entries a row. */
int orc_sched_definition(int32_t p, int general_only, int32_t *bb_out,
                         int32_t *recv, int32_t *send)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    int32_t *bb = (int32_t *)malloc(sizeof(int32_t) * (size_t)p);
    if (!bb) return ORC_ENOMEM;
    orc_baseblocks_linear(p, bb);
    if (bb_out) memcpy(bb_out, bb, sizeof(int32_t) * (size_t)p);
    int rc = 0;
    for (int32_t r = 0; r < p && !rc; r++)
        rc = recvsched_core(skips, q, r, q - 1, bb, general_only, recv + (size_t)r * q);
    if (!rc && send) {
        for (int32_t j = 0; j < p; j++)
            for (int k = 0; k < q; k++) {
                int32_t t = (int32_t)(((int64_t)j + skips[k]) % p);
                send[(size_t)j * q + k] = recv[(size_t)t * q + k];
            }
    }
    free(bb);
    return rc;
}

/* Rows of ranks [r0, r1) for broadcast root `root`: the row of rank r is the
 * schedule of virtual rank (r - root + p) mod p (Section 2, paragraph after
 * Alg. 2; Section 2.4).  Receive rows by Alg. 4 with the O(q) range routine.
 * Send rows: when the call covers every rank, by the look-up of Alg. 9;
 * otherwise by Alg. 5.  Output [(r - r0) * q + k]; either table may be NULL.
 * `threads` >= 1 splits the rank loop with OpenMP; results do not depend
 * on it. */
int orc_sched_range(int32_t p, int32_t root, int32_t r0, int32_t r1,
                    int32_t *recv, int32_t *send, int threads)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1 || root < 0 || root >= p || r0 < 0 || r0 > r1 || r1 > p) return ORC_EINVAL;
    if (threads < 1) threads = 1;
    int q = orc_skips(p, skips);
    if (q == 0) return 0;
    int full = (r0 == 0 && r1 == p);
    int32_t *rtab = recv;
    if (send && full && !recv) {
        rtab = (int32_t *)malloc(sizeof(int32_t) * (size_t)p * q);
        if (!rtab) return ORC_ENOMEM;
    }
    int err = 0;
    if (rtab) {
        #pragma omp parallel for schedule(static) num_threads(threads)
        for (int32_t r = r0; r < r1; r++) {
            int32_t v = (int32_t)(((int64_t)r - root + p) % p);
            int rc = recvsched_core(skips, q, v, q - 1, NULL, 0, rtab + (size_t)(r - r0) * q);
            if (rc) {
                #pragma omp critical
                err = rc;
            }
        }
    }
    if (!err && send) {
        #pragma omp parallel for schedule(static) num_threads(threads)
        for (int32_t r = r0; r < r1; r++) {
            int32_t *row = send + (size_t)(r - r0) * q;
            if (full) {
                for (int k = 0; k < q; k++) {
                    int32_t t = (int32_t)(((int64_t)r + skips[k]) % p);
                    row[k] = rtab[(size_t)t * q + k];
                }
            } else {
                int32_t v = (int32_t)(((int64_t)r - root + p) % p);
                int rc = sendsched_alg5(skips, q, v, row);
                if (rc) {
                    #pragma omp critical
                    err = rc;
                }
            }
        }
    }
    if (rtab != recv) free(rtab);
    return err;
}

/* A batch of unrelated (p, r, root) triples: each row is the schedule of
 * virtual rank (r - root + p) mod p on its own p-processor graph; send rows by
 * Alg. 5.  Rows have stride 32; entries k >= q hold INT32_MIN; q_out[i] = q. */
int orc_sched_batch(int64_t count, const int32_t *p, const int32_t *r, const int32_t *root,
                    int32_t *recv, int32_t *send, int32_t *q_out, int threads)
{
    if (count < 0) return ORC_EINVAL;
    if (threads < 1) threads = 1;
    for (int64_t i = 0; i < count; i++)
        if (p[i] < 1 || r[i] < 0 || r[i] >= p[i] || root[i] < 0 || root[i] >= p[i])
            return ORC_EINVAL;
    int err = 0;
    #pragma omp parallel for schedule(dynamic, 256) num_threads(threads)
    for (int64_t i = 0; i < count; i++) {
        int32_t skips[ORC_MAXQ + 2];
        int q = orc_skips(p[i], skips);
        int32_t v = (int32_t)(((int64_t)r[i] - root[i] + p[i]) % p[i]);
        int rc = 0;
        if (q_out) q_out[i] = q;
        if (recv) {
            int32_t *row = recv + i * ORC_BATCH_STRIDE;
            if (q > 0) rc = recvsched_core(skips, q, v, q - 1, NULL, 0, row);
            for (int k = q; k < ORC_BATCH_STRIDE; k++) row[k] = INT32_MIN;
        }
        if (!rc && send) {
            int32_t *row = send + i * ORC_BATCH_STRIDE;
            if (q > 0) rc = sendsched_alg5(skips, q, v, row);
            for (int k = q; k < ORC_BATCH_STRIDE; k++) row[k] = INT32_MIN;
        }
        if (rc) {
            #pragma omp critical
            err = rc;
        }
    }
    return err;
}

/* Alg. 6, its index arithmetic only: which block a rank receives / sends in
 * each of the n-1+q rounds.  x dummy rounds make x+n-1+q a multiple of q; the
 * schedule entries are shifted by -x (+q for the first x slots, whose first
 * use falls into the second phase); then round i = x, x+1, ... uses slot
 * k = i mod q and adds q to it afterwards.  A negative block means "nothing
 * this round" and is written as -1; a block above n-1 is block n-1 (caption
 * of Alg. 6).  One call expands one table: in[(r-r0)*q + k] ->
 * out[(r-r0)*R + j], R = n-1+q, j counts real rounds from 0.  `threads` splits
 * the row loop; rows are independent. */
int orc_expand(int32_t p, int32_t n, int64_t rows, const int32_t *in, int32_t *out, int threads)
{
    if (p < 1 || n < 1 || rows < 0) return ORC_EINVAL;
    if (threads < 1) threads = 1;
    int q = orc_q(p);
    int64_t R = (int64_t)n - 1 + q;
    if (q == 0) {
        for (int64_t i = 0; i < rows * R; i++) out[i] = -1;
        return 0;
    }
    int64_t x = (q - (n - 1 + q) % q) % q;
    #pragma omp parallel for schedule(static) num_threads(threads)
    for (int64_t row = 0; row < rows; row++) {
        int64_t sched[ORC_MAXQ + 1];
        for (int i = 0; i < q; i++) {
            if (i < x) sched[i] = (int64_t)in[row * q + i] - x + q;
            else       sched[i] = (int64_t)in[row * q + i] - x;
        }
        int64_t i = x;
        while (i < (int64_t)n + q - 1 + x) {
            int k = (int)(i % q);
            int64_t blk = sched[k];
            if (blk < 0) blk = -1;
            else if (blk > n - 1) blk = n - 1;
            out[row * R + (i - x)] = (int32_t)blk;
            sched[k] = sched[k] + q;
            i = i + 1;
        }
    }
    return 0;
}

/* Alg. 9 (irregular allgather), its index arithmetic for ONE process r: which block of buffer[j] is packed
 * for sending and which block of buffer[j] the received data is unpacked into, for every root j and every
 * round.  Steps in the paper's order: the full receive schedule (first loop), the send schedule by look-up
 * (second loop), x dummy rounds, then per round i (slot k = i mod q) and per j the virtual rank
 * r' = (r - j + p) mod p, whose send / receive entry k names the block and is then advanced by q.
 *
 * Reading: Alg. 9 as printed starts its rounds at i = x but leaves out the adjustment of the schedules that
 * Alg. 6 makes for the x dummy rounds (entries shifted by -x, slots below x advanced once); its caption speaks
 * of the same negative / too-large blocks as Alg. 6's, so the adjustment is taken from Alg. 6.  Without it the
 * allgather does not complete when x != 0 (the tests show this on a mutated copy).
 *
 * pack[(i - x) * p + j], unpack[(i - x) * p + j]: block number, -1 = nothing, clamped to n-1; R = n-1+q rows. */
int orc_allgather_tables(int32_t p, int32_t n, int32_t r, int32_t *pack, int32_t *unpack)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1 || n < 1 || r < 0 || r >= p) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    int64_t R = (int64_t)n - 1 + q;
    if (q == 0) {
        for (int64_t i = 0; i < R; i++) { pack[i] = -1; unpack[i] = -1; }
        return 0;
    }
    int64_t *recvsched = (int64_t *)malloc(sizeof(int64_t) * (size_t)p * q);
    int64_t *sendsched = (int64_t *)malloc(sizeof(int64_t) * (size_t)p * q);
    if (!recvsched || !sendsched) { free(recvsched); free(sendsched); return ORC_ENOMEM; }
    int rc = 0;
    for (int32_t j = 0; j < p && !rc; j++) {
        int32_t row[ORC_MAXQ + 1];
        rc = recvsched_core(skips, q, j, q - 1, NULL, 0, row);
        for (int k = 0; k < q; k++) recvsched[(size_t)j * q + k] = row[k];
    }
    if (rc) { free(recvsched); free(sendsched); return rc; }
    for (int32_t j = 0; j < p; j++)
        for (int k = 0; k < q; k++) {
            int32_t t = (int32_t)(((int64_t)j + skips[k]) % p);
            sendsched[(size_t)j * q + k] = recvsched[(size_t)t * q + k];
        }
    int64_t x = (q - (n - 1 + q) % q) % q;
    for (int32_t j = 0; j < p; j++)
        for (int i = 0; i < q; i++) {
            int64_t adj = (i < x) ? (q - x) : (-x);
            recvsched[(size_t)j * q + i] += adj;
            sendsched[(size_t)j * q + i] += adj;
        }
    int64_t i = x;
    while (i < (int64_t)n + q - 1 + x) {
        int k = (int)(i % q);
        for (int32_t j = 0; j < p; j++) {                         /* pack */
            int32_t rr = (int32_t)(((int64_t)r - j + p) % p);
            int64_t blk = sendsched[(size_t)rr * q + k];
            pack[(i - x) * p + j] = (int32_t)(blk < 0 ? -1 : (blk > n - 1 ? n - 1 : blk));
            sendsched[(size_t)rr * q + k] += q;
        }
        for (int32_t j = 0; j < p; j++) {                         /* unpack */
            int32_t rr = (int32_t)(((int64_t)r - j + p) % p);
            int64_t blk = recvsched[(size_t)rr * q + k];
            unpack[(i - x) * p + j] = (int32_t)(blk < 0 ? -1 : (blk > n - 1 ? n - 1 : blk));
            recvsched[(size_t)rr * q + k] += q;
        }
        i = i + 1;
    }
    free(recvsched);
    free(sendsched);
    return 0;
}

/* Block b of a buffer of m elements cut into n blocks: elements floor(b*m/n) .. floor((b+1)*m/n) - 1.
 * Reading: the paper asks for n blocks of about the same size (Section 2), each the buffer size over n
 * (Section 2.4), and gives no rule for remainders; this balanced cut covers the buffer exactly with block sizes
 * that differ by at most one.  m < 2^31 and b <= n < 2^31 keep the product inside 64 bits. */
static int64_t block_begin(int64_t m, int64_t n, int64_t b) { return (b * m) / n; }

/* Alg. 9, "Pack" loop of one round: for every root j in order, block idx[j] of buffer[j] (nothing when idx[j] < 0)
 * is appended to the message.  Buffers lie in `data` at element offsets displs[j] .. displs[j+1].
 * offsets[j] = where root j's block starts in the message, offsets[p] = message length.  Returns that length
 * (or a negative code); copies nothing beyond `capacity` elements. */
int64_t orc_pack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, const int32_t *data,
                       int32_t *packed, int64_t capacity, int64_t *offsets)
{
    if (p < 1 || n < 1) return ORC_EINVAL;
    int64_t off = 0;
    for (int32_t j = 0; j < p; j++) {
        offsets[j] = off;
        if (idx[j] < 0) continue;
        int64_t b = idx[j] > n - 1 ? n - 1 : idx[j];      /* caption of Alg. 9: beyond n-1 means n-1 */
        int64_t m = displs[j + 1] - displs[j];
        int64_t lo = block_begin(m, n, b), hi = block_begin(m, n, b + 1);
        for (int64_t e = lo; e < hi; e++)
            if (off + (e - lo) < capacity) packed[off + (e - lo)] = data[displs[j] + e];
        off += hi - lo;
    }
    offsets[p] = off;
    return off;
}

/* Alg. 9, "Unpack" loop of one round: the message is cut in the same way and each piece stored as block idx[j]
 * of buffer[j]. */
int64_t orc_unpack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, int32_t *data,
                         const int32_t *packed, int64_t length, int64_t *offsets)
{
    if (p < 1 || n < 1) return ORC_EINVAL;
    int64_t off = 0;
    for (int32_t j = 0; j < p; j++) {
        offsets[j] = off;
        if (idx[j] < 0) continue;
        int64_t b = idx[j] > n - 1 ? n - 1 : idx[j];
        int64_t m = displs[j + 1] - displs[j];
        int64_t lo = block_begin(m, n, b), hi = block_begin(m, n, b + 1);
        if (off + (hi - lo) > length) return ORC_EINVAL;
        for (int64_t e = lo; e < hi; e++) data[displs[j] + e] = packed[off + (e - lo)];
        off += hi - lo;
    }
    offsets[p] = off;
    return off;
}

/* Alg. 7 (regular allgather on the circulant graph), the plan of process r: in round k it sends the first
 * skips[k+1]-skips[k] blocks of its buffer to (r - skips[k] + p) mod p and receives as many from
 * (r + skips[k]) mod p into buffer[skips[k] ..]; buffer[i] then holds the block of process (r + i) mod p.
 * Arrays of q entries. */
int orc_allgather_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *count, int32_t *recv_first)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1 || r < 0 || r >= p) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    for (int k = 0; k < q; k++) {
        to[k] = (int32_t)(((int64_t)r - skips[k] + p) % p);
        from[k] = (int32_t)(((int64_t)r + skips[k]) % p);
        count[k] = skips[k + 1] - skips[k];
        recv_first[k] = skips[k];
    }
    return q;
}

/* Alg. 8 (census / allreduce), the plan of process r.  Round k: when skips[k] + skips[k] > skips[k+1] the partner
 * is one rank closer on both sides and only the partial sum S is sent; otherwise the own value is folded in
 * (own[k] = 1).  Reading: the condition is printed with index i where the loop variable is k. */
int orc_census_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *own)
{
    int32_t skips[ORC_MAXQ + 2];
    if (p < 1 || r < 0 || r >= p) return ORC_EINVAL;
    int q = orc_skips(p, skips);
    for (int k = 0; k < q; k++) {
        if ((int64_t)skips[k] + skips[k] > skips[k + 1]) {
            to[k] = (int32_t)(((int64_t)r - skips[k] + 1 + p) % p);
            from[k] = (int32_t)(((int64_t)r + skips[k] - 1) % p);
            own[k] = 0;
        } else {
            to[k] = (int32_t)(((int64_t)r - skips[k] + p) % p);
            from[k] = (int32_t)(((int64_t)r + skips[k]) % p);
            own[k] = 1;
        }
    }
    return q;
}

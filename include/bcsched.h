/*
 * bcsched.h -- C ABI of libbcsched: round-optimal n-block broadcast schedules
 * on a p-processor circulant graph, constructed on one AMD MI355X (gfx950).
 *
 * Method: J. L. Traff, "(Poly)Logarithmic Time Construction of Round-optimal
 * n-Block Broadcast Schedules for Broadcast and irregular Allgather in MPI"
 * (arXiv 2205.10072), Section 2.  Citations below name that paper's sections,
 * algorithms and tables.
 *
 * Vocabulary (Section 2): p ranks 0..p-1; q = ceil(log2 p); skips[0..q] with
 * skips[q] = p and skips[k-1] = ceil(skips[k]/2) (Alg. 1); in slot k a rank r
 * sends to (r + skips[k]) mod p and receives from (r - skips[k] + p) mod p.
 * A rank's receive schedule recvsched[0..q-1] (Alg. 4) and send schedule
 * sendsched[0..q-1] (Alg. 5) hold block numbers relative to the current phase
 * of q rounds: one non-negative entry (the baseblock, Alg. 2) and negative
 * entries b - q for blocks of the previous phase.
 *
 * Conventions of every call
 *   - "device" pointers are HIP device memory on the current device, owned by
 *     the caller, at least 4-byte aligned; "host" pointers are plain memory.
 *   - All tables are int32, row-major, one row per rank.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it.  No call waits for the device, with one
 *     exception: a plain (not *_ws) call that finds the library's per-device
 *     scratch too small synchronises the device, frees it and allocates a
 *     larger one (so such a call cannot be part of a stream capture).
 *   - Return value: BCS_OK (0) or a negative BCS_E* code.  On an error nothing
 *     has been enqueued and no output is touched.  No call throws.
 *   - No call allocates or frees its outputs.  bcs_sched* with a send table
 *     over the full rank range, or over a large part of it, need scratch
 *     memory (bcs_sched_workspace_bytes says how much): the *_ws variants take it
 *     from the caller, the plain variants keep one allocation per device that
 *     grows on demand and is released by bcs_release().  Plain calls on one
 *     device share that allocation: the library orders them itself (a plain
 *     call on another stream than the plain call before it is made to wait,
 *     on the device, for that stream's work), so they never overlap; callers
 *     that want overlap use the *_ws variants with a workspace per stream.
 *     A stream handed to a plain call should stay alive until the next plain
 *     call on the device (else that call synchronises the device instead).
 *   - The first call on a device that builds schedules (bcs_sched*,
 *     bcs_sched_batch, bcs_allgather_tables*) also enqueues, ahead of its own
 *     work, a short kernel that fills a 544 KiB table kept in the library's
 *     code object (baseblock sets of the seven lowest levels of the circulant
 *     graph).  Until that kernel has finished, calls on other streams are made
 *     to wait for it on the device; no call waits on the host.
 *   - Calls that allocate nothing (the *_ws entry points, bcs_expand,
 *     bcs_sched_batch) may be recorded into a HIP graph, once one schedule-
 *     building call has been made on the device outside the capture (that first
 *     call also queries an event).  They enqueue kernels only.
 */
#ifndef BCSCHED_H
#define BCSCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BCS_OK        0
#define BCS_EINVAL  (-1)  /* an argument is outside its domain (see each call)        */
#define BCS_EHIP    (-2)  /* a HIP call failed; bcs_last_hip_error() has its code      */
#define BCS_ENOMEM  (-3)  /* scratch allocation failed, or the given workspace is small */
#define BCS_ETOOBIG (-4)  /* bcs_sched_rooted_static: needs more than its fixed scratch  */

#define BCS_MAX_Q         31           /* p <= 2^31 - 1                                */
#define BCS_BATCH_STRIDE  32           /* ints per row of the batch tables             */
#define BCS_BATCH_PAD     INT32_MIN    /* fills batch row entries k >= q               */
#define BCS_NO_BLOCK      (-1)         /* expanded tables: nothing moves in this round */
#define BCS_MAX_N         (INT32_MAX - 64) /* bcs_expand: rounds and blocks stay in int32 */

/* q = ceil(log2 p) (Section 2, first paragraph).  p = 1 gives 0.
 * Returns BCS_EINVAL for p < 1. */
int bcs_q(int32_t p);

/* Alg. 1.  Writes skips[0..q] (q+1 values) to host memory `skips_host` and
 * returns q.  BCS_EINVAL for p < 1 or a NULL pointer. */
int bcs_skips(int32_t p, int32_t *skips_host);

/* Number of rounds of the n-block broadcast, n - 1 + q (Section 1; Alg. 6).
 * Returns BCS_EINVAL (as int64) for p < 1 or n < 1. */
int64_t bcs_rounds(int32_t p, int32_t n);

/* Receive and send schedules (Alg. 4; Alg. 5 / first loops of Alg. 9) of the
 * ranks r0 <= r < r1 for a broadcast rooted at rank 0.
 *   recv_out, send_out: device, (r1-r0) x q int32, entry [(r-r0)*q + k].
 *   Either may be NULL (that table is not produced); both NULL is an error.
 * When the call covers all ranks (r0 = 0, r1 = p) send rows are read off the
 * receive rows of the to-neighbours (Alg. 9, second loop); otherwise each send
 * entry is recomputed from the neighbour's receive schedule (Alg. 5).  Both
 * give the same values.
 * p = 1: q = 0, rows are empty, nothing is enqueued, BCS_OK.
 * BCS_EINVAL: p < 1, r0 < 0, r0 > r1, r1 > p, both outputs NULL. */
int bcs_sched(int32_t p, int32_t r0, int32_t r1,
              int32_t *recv_out, int32_t *send_out, void *stream);

/* As bcs_sched for an arbitrary root: the row of rank r is the schedule of
 * the virtual rank (r - root + p) mod p (Section 2, paragraph after Alg. 2;
 * Section 2.4 uses this for every root at once).  Neighbours are unchanged:
 * rank r still sends to (r + skips[k]) mod p.
 * Also BCS_EINVAL for root outside [0, p). */
int bcs_sched_rooted(int32_t p, int32_t root, int32_t r0, int32_t r1,
                     int32_t *recv_out, int32_t *send_out, void *stream);

/* Scratch bytes bcs_sched_rooted_ws needs for these arguments (0 when none).
 * Negative: BCS_EINVAL.  A call over all ranks that also wants send rows keeps
 * there the receive entries slot by slot (one byte each) and the greedy skip
 * sums of all ranks (the walk of Alg. 2 kept as a mask, one word a rank,
 * rounded up to 256 bytes): every end point of a
 * window of Alg. 4 is some rank, so the receive rows read these instead of
 * walking q + 2 times each.  A call for a part of the ranks with send rows
 * (Alg. 5) asks for the same table when filling it costs less than the walks
 * it saves: (r1 - r0) q^2 >= 8 p. */
int64_t bcs_sched_workspace_bytes(int32_t p, int32_t r0, int32_t r1, int want_send);

/* bcs_sched_rooted with caller-provided scratch.  `workspace` is device
 * memory, 256-byte aligned, of at least bcs_sched_workspace_bytes(...) bytes;
 * its contents are undefined afterwards.  BCS_ENOMEM if it is too small or
 * NULL while scratch is needed, BCS_EINVAL if it is needed and not 256-byte
 * aligned.  Performs no allocation.  A call over all
 * ranks for receive rows alone needs none; given 4 p bytes (rounded up to 256)
 * it uses them for the table of skip sums. */
int bcs_sched_rooted_ws(int32_t p, int32_t root, int32_t r0, int32_t r1,
                        int32_t *recv_out, int32_t *send_out,
                        void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc):
 * bcs_sched_rooted with its scratch in a fixed array of
 * BCS_STATIC_SCRATCH_BYTES that lives in the library's code object, one copy
 * on every GPU the library runs on, held until the process ends.  Arguments,
 * results and errors are those of bcs_sched_rooted, bit for bit.  The call
 * allocates and frees nothing; the first call on a device looks the array's
 * address up (and, as every schedule-building call, may enqueue the fill of the
 * low-level table), later calls enqueue kernels only.
 * Limit: bcs_sched_workspace_bytes(p, r0, r1, send_out != NULL) must not
 * exceed BCS_STATIC_SCRATCH_BYTES, else BCS_ETOOBIG and nothing is enqueued
 * (all ranks with send rows: p up to 1 342 016).  Every call on a
 * GPU shares that GPU's array: calls that overlap on one GPU (two streams, or
 * two threads) race and must be ordered by the caller.  Nothing in the array
 * has to start at zero: each call overwrites what it reads, so the contents
 * the last call left behind do no harm. */
#define BCS_STATIC_SCRATCH_BYTES (32u << 20)
int bcs_sched_rooted_static(int32_t p, int32_t root, int32_t r0, int32_t r1,
                            int32_t *recv_out, int32_t *send_out, void *stream);

/* `count` unrelated problems: problem i is rank r[i] of a p[i]-rank graph with
 * broadcast root root[i].  p, r, root: device arrays of `count` int32.
 *   recv_out, send_out: device, count x BCS_BATCH_STRIDE int32; row i holds
 *   q_i = ceil(log2 p[i]) entries, the rest BCS_BATCH_PAD.  Either may be NULL.
 *   q_out: device, count int32, may be NULL.
 * Send rows need no other rank of that graph: an entry is taken from the rank's
 * own greedy digits where that gives Alg. 5's value, and recomputed per Alg. 5
 * (the to-neighbour's rounds up to it) otherwise; the results are Alg. 5's.
 * Triples are validated on the device: a row with p < 1 or r, root outside
 * [0, p) gets q_out = -1 and all-PAD rows; host-side errors are BCS_EINVAL for
 * count < 0, a NULL input array, or all outputs NULL. */
int bcs_sched_batch(int64_t count, const int32_t *p, const int32_t *r, const int32_t *root,
                    int32_t *recv_out, int32_t *send_out, int32_t *q_out, void *stream);

/* The (rank, round) -> block tables of the n-block broadcast (index arithmetic
 * of Alg. 6: x = (q - (n-1+q) mod q) mod q dummy rounds, entries shifted by -x,
 * slot k = (x+j) mod q in real round j, +q per phase; caption of Alg. 6: a
 * negative block means nothing is sent / received, a block above n-1 is n-1).
 *   recv, send: device, (r1-r0) x q, as produced by bcs_sched*; either may be
 *   NULL together with its output.
 *   recv_blocks, send_blocks: device, (r1-r0) x R int32, R = n-1+q, entry
 *   [(r-r0)*R + j] = block moved in round j, or BCS_NO_BLOCK.
 * p = 1: q = 0, the input tables have empty rows and are ignored (may be
 * NULL); each output given gets R = n-1 columns, all BCS_NO_BLOCK.
 * Outputs that are 16-byte aligned are written with 16-byte stores.
 * BCS_EINVAL: p < 1, n < 1, n > BCS_MAX_N, bad range, a table given without
 * its output (or the reverse), nothing to do. */
int bcs_expand(int32_t p, int32_t n, int32_t r0, int32_t r1,
               const int32_t *recv, const int32_t *send,
               int32_t *recv_blocks, int32_t *send_blocks, void *stream);

/* bcs_expand (index arithmetic of Alg. 6 and its caption) with scratch memory
 * from the caller.  This is the fast path for long rows: measured on MI355X
 * at p = 65 537, n = 4096 it writes 0.87-0.89 of the HBM peak where bcs_expand,
 * which may not use scratch memory, reaches 0.82-0.83.  For rows of 256 rounds or more
 * the schedule rows are first rewritten as bytes into `workspace` (about a
 * million rows at a time, so that it stays in cache) and the tables are
 * expanded from there; results are those of bcs_expand, bit for bit.
 *   workspace: device, 16-byte aligned, bcs_expand_workspace_bytes(p, n, r0, r1)
 *   bytes (0 when the detour does not pay; negative: BCS_EINVAL); its contents
 *   are undefined afterwards.  With less, or with outputs that are not 16-byte
 *   aligned, the call is bcs_expand.  Performs no allocation.
 * Errors as bcs_expand. */
int64_t bcs_expand_workspace_bytes(int32_t p, int32_t n, int32_t r0, int32_t r1);
int bcs_expand_ws(int32_t p, int32_t n, int32_t r0, int32_t r1,
                  const int32_t *recv, const int32_t *send,
                  int32_t *recv_blocks, int32_t *send_blocks,
                  void *workspace, size_t workspace_bytes, void *stream);

/* Schedules of all p ranks and both of their (rank, round) -> block tables in
 * one call: the same results as bcs_sched_rooted_ws(p, root, 0, p, ...) followed
 * by bcs_expand(p, n, 0, p, ...) (Alg. 4, Alg. 9's send look-up, index arithmetic
 * of Alg. 6), bit for bit.  For many ranks and moderate n the rows are expanded
 * by the workgroup that built them, straight from on-chip memory; other sizes
 * run the two calls above one after the other.
 *   recv_out, send_out: device, p x q int32 (required when q > 0).
 *   recv_blocks, send_blocks: device, p x R int32, R = n-1+q (required when
 *   R > 0; p = 1 with n = 1 has nothing to write and returns BCS_OK).
 * For longer rows the schedule kernels also leave the rows as bytes in scratch
 * memory, which the expansion then reads from cache instead of re-reading the
 * int32 tables.
 * Scratch: bcs_sched_expand_workspace_bytes(p, n) bytes (negative: BCS_EINVAL);
 * the plain call uses the per-device allocation, the _ws call takes it from the
 * caller (256-byte aligned) and allocates nothing.  With less than that but at
 * least bcs_sched_workspace_bytes(p, 0, p, 1) bytes the _ws call still works
 * (without the byte rows).  p = 1: both block tables get n-1 columns of
 * BCS_NO_BLOCK.
 * BCS_EINVAL: p < 1, root outside [0, p), n < 1, n > BCS_MAX_N, a required
 * table NULL, a workspace that is not 256-byte aligned.  BCS_ENOMEM: workspace
 * NULL or too small. */
int64_t bcs_sched_expand_workspace_bytes(int32_t p, int32_t n);
int bcs_sched_expand(int32_t p, int32_t root, int32_t n,
                     int32_t *recv_out, int32_t *send_out,
                     int32_t *recv_blocks, int32_t *send_blocks, void *stream);
int bcs_sched_expand_ws(int32_t p, int32_t root, int32_t n,
                        int32_t *recv_out, int32_t *send_out,
                        int32_t *recv_blocks, int32_t *send_blocks,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Index tables of the irregular allgather for ONE process r (Alg. 9, its pack
 * and unpack loops; Section 2.4): in real round j the process packs, for every
 * root `root`, block pack_idx[j*p + root] of buffer[root] for its to-neighbour
 * and unpacks what it receives into block unpack_idx[j*p + root] of
 * buffer[root].  Towards root `root` the process acts as virtual rank
 * (r - root + p) mod p of a broadcast rooted at 0, with the dummy-round shift and
 * clamping of Alg. 6 (Alg. 9 prints only x; the adjustment of the schedules is
 * taken from Alg. 6).
 *   pack_idx, unpack_idx: device, R x p int32, R = n-1+q, round-major;
 *   BCS_NO_BLOCK where nothing moves.  Either may be NULL.
 * Scratch: bcs_allgather_workspace_bytes(p) bytes (the slot-major receive table
 * of all ranks); the plain call uses the per-device allocation of bcs_sched*,
 * the _ws call takes it from the caller (256-byte aligned) and allocates
 * nothing.  p = 1: R = n-1 entries of BCS_NO_BLOCK.
 * BCS_EINVAL: p < 1, n < 1, n > BCS_MAX_N, r outside [0, p), both outputs NULL,
 * a workspace that is not 256-byte aligned.  BCS_ENOMEM: workspace NULL or too
 * small. */
int64_t bcs_allgather_workspace_bytes(int32_t p);
int bcs_allgather_tables(int32_t p, int32_t n, int32_t r,
                         int32_t *pack_idx, int32_t *unpack_idx, void *stream);
int bcs_allgather_tables_ws(int32_t p, int32_t n, int32_t r,
                            int32_t *pack_idx, int32_t *unpack_idx,
                            void *workspace, size_t workspace_bytes, void *stream);

/* One round of packing / unpacking for the irregular allgather (Alg. 9, its
 * "Pack" and "Unpack" loops).  A process keeps the p buffers in one device
 * array `data` of int32 elements, buffer j at elements displs[j] ..
 * displs[j+1]-1 (displs: device, p+1 int64, non-decreasing; a buffer has fewer
 * than 2^31 elements).  A buffer of m elements is cut into n blocks, block b
 * being elements floor(b*m/n) .. floor((b+1)*m/n)-1 (the paper asks for blocks of
 * about the same size and gives no rule for remainders).
 *   idx: device, p int32: the block of each buffer that moves in this round
 *   (a row of the tables of bcs_allgather_tables); negative = none; values
 *   above n-1 are read as n-1.
 * bcs_pack_round appends, root by root, block idx[j] of buffer j to the
 * message `packed` (device, `capacity` elements; what does not fit is not
 * written).  bcs_unpack_round cuts the message `packed` of `length` elements
 * the same way and stores the pieces as block idx[j] of buffer j.
 *   offsets: device, p+1 int64, output of both: where root j's piece starts in
 *   the message; offsets[p] = length of the whole message (compare it with
 *   `capacity` / `length` after synchronising).
 *   workspace: device, 8-byte aligned, bcs_pack_workspace_bytes(p) bytes.
 * Both calls enqueue four kernels and allocate nothing.
 * BCS_EINVAL: p < 1, n < 1, a NULL array (`packed` may be NULL when capacity /
 * length is 0: then only `offsets` is produced), negative capacity / length.
 * BCS_ENOMEM: workspace NULL, misaligned or too small. */
int64_t bcs_pack_workspace_bytes(int32_t p);
int bcs_pack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs,
                   const int32_t *data, int32_t *packed, int64_t capacity,
                   int64_t *offsets, void *workspace, size_t workspace_bytes, void *stream);
int bcs_unpack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs,
                     int32_t *data, const int32_t *packed, int64_t length,
                     int64_t *offsets, void *workspace, size_t workspace_bytes, void *stream);

/* The same with the plans of ALL rounds made ahead, in one launch (Alg. 9 runs its pack and unpack loops once
 * per round; at the paper's sizes -- p = 1152, a few hundred KB per round -- a round is bound by launch latency,
 * so the per-round work is cut to one kernel per direction).
 * bcs_pack_plan_rounds: row j of idx_table (device, rounds x p int32: a table of bcs_allgather_tables, or any
 * rows of block numbers) is planned into row j of
 *   offsets_all: device, rounds x (p+1) int64: what bcs_pack_round writes to `offsets` for that round;
 *   src_all: device, rounds x p int64: where each root's block starts in `data` (elements).
 * bcs_pack_round_planned / bcs_unpack_round_planned: the payload of one round from its two plan rows
 * (offsets: p+1 entries, src: p entries); arguments otherwise as bcs_pack_round / bcs_unpack_round.
 * All three enqueue one kernel and allocate nothing.
 * BCS_EINVAL: p < 1, n < 1, rounds < 0, a NULL array, plan arrays not 8-byte aligned, negative capacity / length. */
int bcs_pack_plan_rounds(int32_t p, int32_t n, int64_t rounds, const int32_t *idx_table, const int64_t *displs,
                         int64_t *offsets_all, int64_t *src_all, void *stream);
int bcs_pack_round_planned(int32_t p, const int64_t *offsets, const int64_t *src, const int32_t *data,
                           int32_t *packed, int64_t capacity, void *stream);
int bcs_unpack_round_planned(int32_t p, const int64_t *offsets, const int64_t *src, int32_t *data,
                             const int32_t *packed, int64_t length, void *stream);

/* Plans of the two other collectives the paper runs on the same circulant
 * graph; host-side, O(q), all arrays are host memory with room for q entries,
 * the return value is q (or BCS_EINVAL for p < 1, r outside [0, p), NULL).
 * bcs_allgather_plan (Alg. 7, regular allgather): in round k process r sends
 * the first count[k] = skips[k+1]-skips[k] blocks of its buffer to to[k] =
 * (r - skips[k] + p) mod p and receives count[k] blocks from from[k] =
 * (r + skips[k]) mod p into buffer[recv_first[k] ..], recv_first[k] = skips[k];
 * buffer[i] ends up holding the block of process (r + i) mod p.
 * bcs_census_plan (Alg. 8, census / allreduce): in round k process r sends to
 * to[k] and receives from from[k]; own[k] = 1: it sends x_r + S (partner at
 * distance skips[k]); own[k] = 0: it sends its partial sum S alone (partner at
 * distance skips[k] - 1; this is the case skips[k] + skips[k] > skips[k+1]).
 * After the q rounds S + x_r is the sum over all processes. */
int bcs_allgather_plan(int32_t p, int32_t r, int32_t *to, int32_t *from,
                       int32_t *count, int32_t *recv_first);
int bcs_census_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *own);

/* The partner tables of the same two collectives for the processes [r0, r1) at
 * once, written by one kernel (HBM-bound, pure stores): what a launcher or a
 * simulator of the whole machine needs, and the device-side form of the two
 * plans above.  to and from are device arrays of (r1 - r0) * q int32, entry
 * [(r - r0) * q + k]; either may be NULL.
 * bcs_allgather_partners (Alg. 7): to = (r - skips[k] + p) mod p, from =
 * (r + skips[k]) mod p.  bcs_census_partners (Alg. 8): the same with the
 * distance skips[k] - 1 in the rounds where 2 skips[k] > skips[k+1].  The
 * per-round quantities that do not depend on the process (count, recv_first,
 * own) come from the host plans of any one process.
 * Asynchronous on `stream`, no allocation.  BCS_EINVAL: p < 1, a range outside
 * 0 <= r0 <= r1 <= p, both arrays NULL with entries to write (p = 1 and
 * r0 = r1 have none). */
int bcs_allgather_partners(int32_t p, int32_t r0, int32_t r1, int32_t *to, int32_t *from, void *stream);
int bcs_census_partners(int32_t p, int32_t r0, int32_t r1, int32_t *to, int32_t *from, void *stream);

/* Frees the per-device scratch kept by the plain bcs_sched* calls on the
 * current device (after synchronising that device).  Safe to call anytime. */
int bcs_release(void);

/* Device-side duration of each kernel, for measurements.  Between
 * bcs_timing_begin() and bcs_timing_end() every kernel this library launches
 * (from the calling process, any stream) carries its own start/stop event
 * pair from a pool of BCS_TIMING_MAX_LAUNCHES; later launches run untimed.
 * bcs_timing_end waits for the timed launches and writes, per kernel id
 * 0..BCS_KERNEL_COUNT-1, the summed duration in milliseconds and the number
 * of timed launches into host arrays of BCS_KERNEL_COUNT entries.  Not
 * thread-safe; meant for one measuring thread. */
#define BCS_KERNEL_COUNT         16
#define BCS_TIMING_MAX_LAUNCHES  4096
int bcs_timing_begin(void);
int bcs_timing_end(double *ms_sum_host, int64_t *launches_host);
/* bcs_timing_end that also gives the shortest and the longest timed launch of
 * each kernel (arrays of BCS_KERNEL_COUNT doubles; either may be NULL). */
int bcs_timing_stats(double *ms_sum_host, int64_t *launches_host, double *ms_min_host, double *ms_max_host);
/* Name of kernel `id` as a profiler shows it (without template arguments). */
const char *bcs_kernel_name(int id);

/* Measurement aid, not part of the method: launches a kernel of `blocks`
 * workgroups of 256 lanes in which every lane executes
 * iters * BCS_VALU_PEAK_OPS_PER_ITER independent
 * full-rate 32-bit integer vector operations (add, xor, min, subtract) and then
 * stores one word to sink[blocks * 256] (device).  Timed with
 * bcs_timing_begin/end (kernel "k_valu_peak") it gives the integer-ALU rate
 * this GPU reaches in practice.  BCS_EINVAL for a zero count or NULL sink. */
#define BCS_VALU_PEAK_OPS_PER_ITER 32
int bcs_valu_peak_launch(uint32_t blocks, uint32_t iters, uint32_t *sink, void *stream);

/* Text for a BCS_* code; never NULL. */
const char *bcs_strerror(int code);

/* hipError_t (as int) of the last failed HIP call made by this library in the
 * calling thread; 0 if none. */
int bcs_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BCSCHED_H */

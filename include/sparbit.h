/*
 * sparbit.h -- C ABI of the Sparbit Allgather hot path for one MI355X (gfx950).
 *
 * The library executes Allgather exchange schedules for p *virtual* ranks
 * whose send and receive buffers all live in one GPU's HBM.  A point-to-point
 * message of the paper (one Isend matched with one Irecv of one block) becomes
 * one block_bytes-sized device copy; the per-step Waitall becomes a kernel
 * boundary or a device-wide barrier inside one persistent kernel.
 *
 * Buffer layout (all pointers are DEVICE pointers, owned by the caller, never
 * retained or freed by the library):
 *   sendbufs  p blocks; rank r's block at byte offset r * block_bytes.
 *   recvbufs  p * p blocks; rank r's receive buffer at byte r * p * block_bytes,
 *             its slot k at + k * block_bytes.  On return (after the stream has
 *             drained) slot k of every rank holds rank k's block: the
 *             MPI_Allgather post-condition of Section II of the paper.
 *   Blocks are opaque bytes; the MPI (count, datatype) pair collapses into
 *   block_bytes.  Any block_bytes and any base alignment is accepted.  What
 *   a Sparbit call needs to run as one launch at any size is that p *
 *   block_bytes, the distance between two ranks' receive buffers, is a
 *   multiple of 128: blocks of 512 bytes and more then move in 16-byte vectors
 *   that cover whole 128-byte lines wherever the blocks start and end (single
 *   bytes at their two ends).  With other row lengths such blocks still move
 *   in 16-byte vectors, on calls of several GiB at about 60 % of that rate
 *   (one launch per step); blocks shorter than 512 bytes move with 16-, 4- or
 *   single-byte accesses as their alignment allows.  The highest rate (about
 *   a fifth more on calls of 0.4 GiB and more) is that of blocks whose length
 *   is a multiple of 64 KiB, better of 128 KiB, in a receive buffer that
 *   starts on such a boundary (see "tree_gang" below); other bases on the
 *   128-byte grid keep 0-8 % of it.  Long blocks of other lengths come to
 *   within 10 % of it where p * block_bytes (Allgatherv: row_bytes) is a
 *   multiple of 64 KiB.
 *
 * Every entry point returns SPARBIT_OK (0) or a negative SPARBIT_ERR_* code and
 * never throws.  Work is enqueued on the caller's stream; the call returns
 * without synchronising, with these exceptions, all of them first uses:
 *   - the first call for a (schedule, p) on a device builds and uploads its
 *     tables with blocking copies (the TREE form has no tables);
 *   - the first PERSISTENT or DATAFLOW launch on a stream (AUTO may choose them
 *     for schedules other than Sparbit) allocates that stream's barrier / flag
 *     state and synchronises the device once; a later call that needs more ready
 *     flags than any before it on that stream synchronises the stream, frees the
 *     flag array and allocates a larger one (device synchronisation again);
 *   - Bruck's working buffer grows the same way (device synchronisation), is
 *     one per device and is shared by all streams: Bruck calls on different
 *     streams must not overlap;
 *   - Allgatherv: a geometry not among the last 8 used on the device is built
 *     and uploaded, and evicting the oldest one synchronises the device.
 *
 * Recording into a HIP graph (stream capture).  A call on a capturing stream
 * records kernel launches and nothing else: one for Sparbit in the tree form
 * (no table, no state, no earlier call needed; Allgatherv with unequal blocks
 * reads the geometry's device copy, see below), one per step for everything
 * else.  The graph is replayed with the pointers it was recorded with.  A
 * capturing call cannot allocate or upload, so where tables are used the same
 * call (same schedule and p; for Allgatherv the same counts, displs and
 * row_bytes; for Bruck a call at least as large) must have run once outside
 * the capture -- otherwise SPARBIT_ERR_UNSUPPORTED, with nothing recorded.
 * SPARBIT_MODE_AUTO records the tree or the per-step form; the PERSISTENT and
 * DATAFLOW modes keep per-stream state on the device that replays would share
 * and are refused with SPARBIT_ERR_UNSUPPORTED.  A graph of table-driven
 * launches refers to the library's cached tables: destroy it before
 * sparbit_finalize, and (Allgatherv) before more than 7 other geometries have
 * been used on the device.
 */
#ifndef SPARBIT_H
#define SPARBIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- return codes ------------------------------------------------------- */
#define SPARBIT_OK 0
#define SPARBIT_ERR_ARG (-1)         /* p < 1, p > SPARBIT_MAX_P, NULL recvbufs, size overflow, bad step range, bad enum */
#define SPARBIT_ERR_ALIAS (-2)       /* sendbufs range overlaps recvbufs range (MPI forbids it; use NULL for in-place) */
#define SPARBIT_ERR_UNSUPPORTED (-3) /* Recursive Doubling with p not a power of two; Bruck in place; a call on a
                                        capturing stream that would have to allocate or wait on itself */
#define SPARBIT_ERR_HIP (-4)         /* a HIP call failed; see sparbit_last_hip_error() */
#define SPARBIT_ERR_NOMEM (-5)       /* host allocation failed */
#define SPARBIT_ERR_TIMEOUT (-6)     /* an earlier PERSISTENT or DATAFLOW launch on this stream gave up a bounded wait: what
                                        it wrote is incomplete.  Reported once, by the next call on that stream, which
                                        enqueues nothing */

#define SPARBIT_ERR_TOO_LARGE (-7)   /* sparbit_allgather_static: p beyond SPARBIT_STATIC_MAX_P */

#define SPARBIT_MAX_P 4096 /* the tables hold p * (p - 1) entries of 8 bytes */
#define SPARBIT_STATIC_MAX_P 512 /* most ranks sparbit_allgather_static accepts: its fixed 2 MiB table holds p * p entries */

/* ---- schedules (Section II-A and Section III of the paper) --------------- */
#define SPARBIT_ALGO_SPARBIT 0            /* Algorithm 1: distance halves, data doubles */
#define SPARBIT_ALGO_RING 1               /* p - 1 steps of one block to rank + 1 */
#define SPARBIT_ALGO_RECURSIVE_DOUBLING 2 /* log2 p pairwise steps, p a power of two */
#define SPARBIT_ALGO_BRUCK 3              /* distance doubles, rotated working buffer + final shift */
#define SPARBIT_ALGO_DIRECT 4             /* no schedule: every slot copied straight from its owner (context only) */

/* ---- how the steps of one call are issued -------------------------------- */
#define SPARBIT_MODE_AUTO 0       /* library picks.  Sparbit, Recursive Doubling and Ring: TREE, except for blocks of
                                     512 bytes and more that are off the 128-byte grid in rows (p * block_bytes)
                                     that are off it too, when the call is larger than 512 MiB (and, below 64 KiB
                                     per block, off the 16-byte grid).  Everything else: DATAFLOW for
                                     calls of at most 256 work items (block copies x 16 KiB pieces) or at most 512
                                     with pieces of up to 64 KiB, PERSISTENT (one workgroup) for other calls of at most
                                     4 KiB, else PER_STEP with the leading small steps (at most 512 work items)
                                     merged into one DATAFLOW launch */
#define SPARBIT_MODE_PER_STEP 1   /* one kernel launch per step (Waitall = kernel boundary) */
#define SPARBIT_MODE_PERSISTENT 2 /* one launch; device-wide barrier between steps */
#define SPARBIT_MODE_DATAFLOW 3   /* one launch; no barrier: a copy starts when the chunk it forwards has landed
                                     (ready flag per chunk of a receive slot).
                                     PERSISTENT and DATAFLOW grids wait on themselves.  A persistent grid of more
                                     than one workgroup is a cooperative launch: the runtime makes the whole grid
                                     resident or the call fails with SPARBIT_ERR_UNSUPPORTED.  A dataflow grid has
                                     one workgroup per work item (block copy x piece) and needs no residency: an
                                     item only waits for items of lower-numbered workgroups, which the GPU starts
                                     first; a call with more than 2^24 - 1 items is refused (SPARBIT_ERR_UNSUPPORTED).
                                     Their waits are bounded all the same (see sparbit_barrier_timeouts).
                                     PER_STEP never waits on the device; in TREE only the wavefronts of one
                                     workgroup wait for each other (small calls, bounded), which needs nothing
                                     resident but that workgroup. */
#define SPARBIT_MODE_TREE 4       /* Sparbit, Recursive Doubling and Ring, whole calls only: one launch in which every
                                     wavefront (in small calls: every team of 4 or 8 wavefronts of one workgroup)
                                     carries one piece of one block through that block's binomial tree
                                     (Section III-B: the p trees are independent; Recursive Doubling's messages,
                                     seen by block, form such trees too, with rank xor origin as the relative rank
                                     (the same tree as Sparbit's once the bits of that relative rank are reversed);
                                     Ring's form a chain per block).  Same messages as Algorithm 1, each read from the
                                     forwarder's receive buffer; a forwarder's reads of one slot for different steps
                                     are merged, and the order is any order in which a rank forwards after it
                                     received.  No table, no barrier and no state in device memory.
                                     Blocks of 512 bytes and more that do not start and end on 128-byte lines are
                                     cut into pieces relative to the lines of the owner's receive buffer (the
                                     same block offsets at every rank): 16-byte chunks, and single bytes at a
                                     block's two ends. */

/*
 * MPI_Allgather over p virtual ranks with the Sparbit schedule (Algorithm 1 of
 * the paper: ceil(log2 p) dependent steps; in the step with distance d rank r
 * forwards the blocks in slots (r - 2 j d) mod p, j < data - ignore, to rank
 * (r + d) mod p, where they land in the same slots).
 *   sendbufs    device, p * block_bytes bytes; NULL = in place (as MPI_IN_PLACE:
 *               recvbufs slot r of rank r already holds rank r's block).
 *   recvbufs    device, p * p * block_bytes bytes.
 *   stream      a hipStream_t of the current device (NULL = the null stream).
 * p = 1 is legal (no steps, the own block is placed).  block_bytes = 0 is legal
 * and does nothing (MPI allows a zero count).
 */
int sparbit_allgather(const void *sendbufs, void *recvbufs, int p, size_t block_bytes,
                      void *stream);

/* Same call with the schedule chosen by `algo` (Section II-A schedules run
 * through the same kernels, for comparison). */
int sparbit_allgather_algo(const void *sendbufs, void *recvbufs, int p, size_t block_bytes,
                           int algo, void *stream);

/* Same call with the schedule and the issue mode chosen explicitly. */
int sparbit_allgather_mode(const void *sendbufs, void *recvbufs, int p, size_t block_bytes,
                           int algo, int mode, void *stream);

/*
 * Run only steps first_step .. last_step (inclusive) of a schedule, one launch
 * per step: the state after each Waitall of Algorithm 1 can be inspected.
 * first_step = -1 also places the own blocks (ignored when sendbufs is NULL);
 * steps are numbered 0 .. num_steps - 1; last_step = -1 with first_step = -1
 * places the own blocks only.  Bruck keeps its rotated working buffer inside
 * the library, so for Bruck only the full range (-1 .. num_steps - 1) is
 * accepted.  DIRECT has no steps: only the range -1 .. -1.
 */
int sparbit_allgather_steps(const void *sendbufs, void *recvbufs, int p, size_t block_bytes,
                            int algo, int first_step, int last_step, void *stream);

/*
 * For callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): sparbit_allgather_steps over the
 * whole range (-1 .. num_steps - 1) of the Sparbit schedule -- own-block
 * placement and one launch per step -- with the copy table in a fixed 2 MiB
 * array inside the library's device image instead of allocated memory.  The
 * call allocates and frees nothing, on the device or through any library, and
 * caches nothing: a small kernel at its head rebuilds the table on the device.
 *   p > SPARBIT_STATIC_MAX_P returns SPARBIT_ERR_TOO_LARGE; every block_bytes
 *   and alignment the other entry points take is accepted.
 *   Each GPU has ONE such array, shared by every call on it and kept until the
 *   process ends: calls to this entry point that overlap in time on one GPU
 *   (different streams, or replays of graphs that recorded it) race on the
 *   table and give wrong results; calls in stream order are fine.
 *   The first call on a device looks up the array's address and is best made
 *   outside a capture.
 * Arguments and result as sparbit_allgather.
 */
int sparbit_allgather_static(const void *sendbufs, void *recvbufs, int p, size_t block_bytes,
                             void *stream);

/*
 * MPI_Allgatherv over the same schedules -- the extension to blocks of
 * different sizes that the paper's conclusion (Section VII) names as future
 * work; the schedule is unchanged, every message just has its slot's length.
 *   counts, displs  HOST arrays of p entries, read during the call and not kept:
 *               rank k contributes counts[k] bytes (0 allowed), which land at
 *               byte displs[k] of every rank's receive buffer.  Blocks must lie
 *               inside row_bytes and must not overlap each other;
 *               p * row_bytes must stay below 2^40.
 *   recvbufs    device; rank r's receive buffer starts at byte r * row_bytes.
 *               Bytes that belong to no block are left untouched.
 *   sendbufs    device, laid out like ONE receive buffer (rank r's block at
 *               displs[r], row_bytes in all); NULL = in place.
 *   algo        SPARBIT, RING, RECURSIVE_DOUBLING (p a power of two) or DIRECT;
 *               BRUCK returns SPARBIT_ERR_UNSUPPORTED (its rotated working
 *               buffer is defined for equal blocks).
 * Equal counts packed back to back (displs[k] = k * counts[0], row_bytes =
 * p * counts[0]) are the layout of sparbit_allgather and are handed to it.
 * Sparbit, Recursive Doubling and Ring go out as ONE launch of the tree form
 * (SPARBIT_MODE_TREE), which
 * reads each block's length and offset from the geometry's device copy, under
 * the same rules as equal blocks: counts and displs of any granularity run as
 * one launch when row_bytes is a multiple of 128 (round the rows up where
 * the layout is yours to choose, best to a multiple of 64 KiB: long
 * blocks of any size then move in gangs as aligned ones do, 7-10 % faster
 * on 16 GiB; a multiple of 1024 is worth 1-4 %); with other row lengths the tree form serves
 * calls of up to 512 MiB, and larger ones only when everything is on the
 * 128-byte grid (or, for blocks below 64 KiB, on the 16-byte grid).
 * Equal blocks at their packed offsets in rows that are longer than p blocks
 * (displs[k] = k * counts[0], row_bytes > p * counts[0]: padded rows, e.g. to
 * take a power-of-two row off the channel interleave) need no geometry at all:
 * they run through the equal-block tree kernel with row_bytes as the row
 * stride, at the cost of the packed call.
 * Otherwise, as for equal blocks of the other schedules, a call of at most 256
 * work items is one dataflow launch and the leading small steps of a larger one
 * share one; the rest goes out as one launch per step, or, where the block
 * lengths of a step are very uneven, one per size class (lengths within a
 * factor of two).  The copy lists of the last few (algo, p, counts, displs,
 * row_bytes) geometries are cached per device; a new geometry costs O(p^2) host
 * work and one upload.
 */
int sparbit_allgatherv(const void *sendbufs, void *recvbufs, int p, const size_t *counts,
                       const size_t *displs, size_t row_bytes, int algo, void *stream);

/* ---- schedule builder (host only; no GPU needed) -------------------------- */
typedef struct sparbit_plan sparbit_plan_t;

typedef struct {
    int distance;             /* d of Algorithm 1; 1 for Ring; 2^s for Recursive Doubling and Bruck */
    int nblocks;              /* blocks every rank sends (and receives) in this step: data - ignore */
    int ignore;               /* 1 if Algorithm 1 drops its last stripe on this step, else 0 */
    const int32_t *dst;       /* [p] rank that r sends to */
    const int32_t *src;       /* [p] rank that r receives from */
    const int32_t *send_slot; /* [p * nblocks], row r: slots of r's buffer it sends, in posting order j */
    const int32_t *recv_slot; /* [p * nblocks], row r: slot of r's buffer where the j-th block from src[r] lands */
} sparbit_step_t;

/* Build the tables of `algo` for p ranks.  *out is owned by the caller until
 * sparbit_plan_destroy.  For Bruck the slots are those of the rotated working
 * buffer (working slot i of rank r holds block (r + i) mod p). */
int sparbit_plan_create(int p, int algo, sparbit_plan_t **out);
/* ceil(log2 p) for Sparbit (the loop bound of Algorithm 1 and the latency term
 * of its cost formula, Section III-B) and Bruck, p - 1 for Ring, log2 p for
 * Recursive Doubling (Section II-A), 0 for DIRECT; negative error code for a
 * NULL plan. */
int sparbit_plan_num_steps(const sparbit_plan_t *plan);
/* Fill *out with pointers into the plan (valid until the plan is destroyed). */
int sparbit_plan_step(const sparbit_plan_t *plan, int step, sparbit_step_t *out);
void sparbit_plan_destroy(sparbit_plan_t *plan);

/* ---- housekeeping --------------------------------------------------------- */
/* Frees the per-device table caches and Bruck's working buffer.  The caller
 * must have synchronised every stream that still runs library work. */
void sparbit_finalize(void);
const char *sparbit_strerror(int code);
/* hipError_t value of the last failed HIP call on this thread (0 if none). */
int sparbit_last_hip_error(void);
/*
 * What the last successful call of this thread enqueued: the number of kernel
 * launches in *launches and the name of the kernel that moved the most bytes,
 * spelled as a profiler prints it (template arguments included), in
 * kernel[0 .. cap) (NUL-terminated, truncated if cap is too small).  Either
 * pointer may be NULL.  For reports and benchmarks: the library, not its
 * caller, knows which variant its selection rules picked.
 */
int sparbit_last_launch_info(char *kernel, size_t cap, int *launches);
/*
 * The waits of the persistent kernel (barrier) and of the dataflow kernel (ready
 * flags) are bounded, so that a launch that cannot make progress ends instead
 * of hanging.  Neither can happen in normal operation: a persistent grid of
 * more than one workgroup is launched cooperatively (the runtime co-schedules
 * the whole grid or the call returns SPARBIT_ERR_UNSUPPORTED), and a dataflow
 * grid has one workgroup per work item, each of which only waits for items of
 * lower-numbered workgroups, which the GPU starts first.  Should a wait expire
 * all the same (or be made to, with the "spin_limit_ms" knob), the launch
 * leaves incomplete results, the next call on that stream returns
 * SPARBIT_ERR_TIMEOUT without enqueuing anything, and a per-stream counter is
 * bumped.  This call synchronises `stream` and stores that counter in *count
 * (0 = every launch completed).
 */
int sparbit_barrier_timeouts(void *stream, uint64_t *count);
/*
 * Tuning knobs for experiments (process-wide; unknown keys or out-of-range
 * values return SPARBIT_ERR_ARG):
 *   "wg_threads"           most lanes per workgroup of the per-step kernel: 64, 128, 256, 512, 1024, or 0 (default):
 *                          64 for 16-byte-aligned blocks of 8 KiB .. 4 MiB, else 256
 *   "unroll"               vectors each lane of that kernel moves: 1, 2 or 4 (2 and 4 only with 256 lanes)
 *   "interleave_log2"      log2 of the block copies dealt round-robin to consecutive workgroups (3 = one per XCD)
 *   "dataflow_max_items"   AUTO uses the dataflow kernel when the call has at most this many work items
 *                          (block copies x chunks per block)
 *   "persistent_max_bytes" else AUTO uses the persistent kernel when p*p*block_bytes is at most this;
 *                          otherwise one launch per step
 *   "hybrid_max_items"     ... where the leading steps that together have at most this many work items (0..1024;
 *                          one workgroup each) share one dataflow launch; 0 = every step its own launch
 *   "flow_chunk_bytes"     unit of work and of readiness of the dataflow kernel (multiple of 16): a block is cut into
 *                          round(block_bytes / this) equal pieces; AUTO may use 2x or 4x this to fit more steps
 *   "nontemporal"          0/1: loads and stores carry the non-temporal hint
 *   "wgs_per_cu"           workgroups per compute unit of the persistent kernel (1..16, capped by occupancy)
 *   "var_idle_max"         Allgatherv: a step whose block lengths differ by more than a factor of four still goes out
 *                          as one launch if that starts at most this many workgroups past the end of shorter blocks
 *   "realign_min_bytes"    blocks at least this long that are off the 16-byte grid use the realigning kernel (>= 16)
 *   "line_align_min_bytes" so do blocks at least this long that are on the 16-byte grid but off the 128-byte one (>= 16)
 *   "spin_limit_ms"        bound of one wait of the persistent and dataflow kernels
 *   "tree_auto"            0/1: AUTO runs whole Sparbit calls as the tree kernel (default 1)
 *   "tree_auto_doubling"   0/1: ... and whole Recursive Doubling calls too (default 1; needs tree_auto)
 *   "tree_auto_ring"       0/1: ... and whole Ring calls (default 1; needs tree_auto)
 *   "tree_team_log2"       small calls (at most tree_small_bytes): 2^this wavefronts per workgroup share the walk of a
 *                          tree's piece (0..4; -1, the default: 4 wavefronts from 33 ranks on, 8 from 65 on)
 *   "tree_run_log2"        the tree kernel walks a tree in runs of 2^this relative ranks (0..12; -1, the default: 5, 4,
 *                          3, 2 or 3 as the grid has fewer than 1024, 2048, 4096, 8192, or more wavefronts; 2 instead
 *                          of the last 3 up to 32 ranks)
 *   "tree_small_bytes"     calls of at most this many receive bytes walk it in step order instead (default 96 MiB)
 *   "tree_unroll"          16-byte vectors per lane of the tree kernel: 1 or 2
 *   "tree_store"           its stores: 0 plain, 2 write-through (default), 3 plain to ranks that are read again soon
 *                          and write-through to the others; 1 and 4 (Sparbit and Recursive Doubling, 16-byte
 *                          vectors; elsewhere they run as 0 and 2): runs of 8 with every forwarder read back right
 *                          after it was stored, all stores plain (1) or only those that are read back (4).  Left at
 *                          2, AUTO and MODE_TREE take 1 by the tree_hot rule and, in calls of more than 336 MiB, 4
 *                          (see tree_hot)
 *   "tree_hot"             Sparbit and Recursive Doubling, 16-byte vectors (aligned blocks or the any-alignment
 *                          form): plain stores, runs of 8, every forwarder read back right after it was stored (-1,
 *                          the default: in calls of 48 MiB (from 65 ranks on: 96 MiB) .. 336 MiB; the any-alignment
 *                          form in rows that are not a multiple of 128 bytes in calls of 48 MiB .. 768 MiB up to 64
 *                          ranks, above 48 MiB below 32 ranks, 96 .. 384 MiB beyond 64 ranks; 0 never; 1 always).
 *                          Left at -1, with the other tree keys untouched, larger calls take store form 4 on a capped
 *                          grid (see tree_store; the any-alignment form only in rows on the lines, blocks of 10 KiB
 *                          and more, below 8 GiB)
 *   "tree_gang"            store forms 1 and 4 on 16-byte vectors, and Ring: workgroups of 4 wavefronts whose pieces lie 32
 *                          KiB apart and that meet at barriers (-1, the default: by size and block length, and one
 *                          workgroup of 8 per compute unit, pieces 16 KiB apart, from 48 ranks on where the blocks
 *                          are a multiple of 128 KiB; 0 never; 1 or 4 wherever the form allows; 8: workgroups of 8
 *                          for equal blocks of whole vectors in store form 4 and for Ring, of 4 elsewhere);
 *                          tree_lds_bytes then counts per wavefront all the same, up to the 64 KiB a workgroup of 4
 *                          may reserve (16384 per wavefront: 2 gangs per unit) and the 160 KiB a workgroup of 8 may
 *   "tree_gang_apart_log2" ... 2^this KiB apart instead (0..10; -1, the default: by the call)
 *   "tree_prefetch"        0/1: it loads the first rank of the next run while it serves the current one
 *   "tree_any_align"       0/1: blocks of realign_min_bytes and more that are off the 128-byte grid run through the
 *                          tree kernel's any-alignment form (default 1; 0: one launch per step, realigning kernel)
 *   "tree_part_line_max_bytes"  ... in rows that are not a multiple of 128 bytes apart only for calls of at most
 *                          this many receive bytes (default 512 MiB)
 *   "tree_lds_bytes"       LDS each of its wavefronts reserves without using it, which caps the wavefronts per
 *                          compute unit (0..65536; 160 KiB per unit, handed out in granules of 1280 bytes; -1, the
 *                          default: by form, size and rank count 0, 10240 (16 wavefronts per unit) or 14336 (10 per
 *                          unit), the latter for grids of 8192 and more wavefronts on more than 32 ranks)
 */
int sparbit_tune(const char *key, long long value);

#ifdef __cplusplus
}
#endif
#endif /* SPARBIT_H */

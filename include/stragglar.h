/*
 * stragglar.h - C ABI of the MI355X (gfx950) StragglAR AllReduce hot path.
 *
 * StragglAR (arXiv 2505.23523) is a straggler-aware AllReduce: while one rank
 * (the straggler) is late, the other n-1 ranks run a ReduceScatter among
 * themselves (the "precondition" of Sec. 3.1); once the straggler arrives, the
 * schedule of Alg. 1 completes the AllReduce in n + log2(n) - 2 rounds (Thm. 1).
 *
 * This library runs that data path on ONE GPU: the n ranks are n separate
 * buffers in the device's HBM, so every transfer of a round becomes an
 * on-device chunk copy and every reduction an on-device chunk add.  All of a
 * round's ops are fused into one kernel launch.
 *
 * Conventions common to every entry point
 *   - Every function returns a sar_status (0 = success) unless stated; nothing
 *     throws or aborts across this boundary.
 *   - "host" / "device" says where a pointer must point.
 *   - Rank ids are physical ranks 0..n-1 (index into rank_bufs).
 *   - Chunking (Sec. 3.1: n-1 equal chunks; App. E: n chunks for ring): with
 *     P parts, chunk_elems = ceil(count / P) rounded up to a multiple of
 *     16 bytes; chunk k covers elements [k*chunk_elems, min((k+1)*chunk_elems,
 *     count)).  The last chunk may be shorter.  A count so small that a chunk
 *     would be empty is rejected with SAR_EINVAL.
 *   - Arithmetic per reducing op (one rounding per op, as on a real wire):
 *       SAR_I32   two's-complement wrap-around add
 *       SAR_F32   one IEEE-754 round-to-nearest-even add, denormals kept
 *       SAR_BF16  widen both to fp32, add, round to nearest even to bf16
 */
#ifndef STRAGGLAR_H
#define STRAGGLAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SAR_OK = 0,
    SAR_EINVAL = 1,        /* bad argument: n < 2, rank out of range, count too small,
                              null / misaligned / overlapping pointers, unknown enum */
    SAR_EUNSUPPORTED = 2,  /* rank count outside what the paper's generators cover: odd n
                              (undefined, Sec. 4 "Limitations"), n above 256, or recursive
                              halving asked for a non-power of two */
    SAR_ENOMEM = 3,        /* host allocation failed */
    SAR_EDEVICE = 4        /* a HIP call failed (no device, launch error) */
} sar_status;

typedef enum { SAR_I32 = 0, SAR_F32 = 1, SAR_BF16 = 2 } sar_dtype;

/* Ops of a round (Sec. 3.1: a round is a set of matchings, each moving one
 * chunk per direction).  SAR_COPY: dst[chunk] = src[chunk].  SAR_REDUCE:
 * dst[chunk] = rnd(dst[chunk] + src[chunk]).  SAR_REDUCE_EXCHANGE: `src` is the
 * on-time rank and `dst` the straggler; t = rnd(src[chunk] + dst[chunk]) is
 * stored to BOTH (Alg. 1, straggler pairing step). */
typedef enum { SAR_COPY = 0, SAR_REDUCE = 1, SAR_REDUCE_EXCHANGE = 2 } sar_opkind;

/* The schedules a plan holds: StragglAR's two phases and the baselines of App. E. */
typedef enum {
    SAR_SCHED_PRECONDITION = 0, /* ring ReduceScatter among the n-1 on-time ranks, n-2 rounds */
    SAR_SCHED_COMPLETION = 1,   /* Alg. 1, n + log2(n) - 2 rounds (App. D's generator for other even n) */
    SAR_SCHED_RING = 2,         /* classic ring AllReduce over all n ranks, 2(n-1) rounds */
    SAR_SCHED_RHD = 3,          /* recursive halving / doubling over all n ranks, 2 log2(n) rounds */
    SAR_SCHED_BCAST_PRECONDITION = 4, /* Broadcast baseline: ring AllReduce among the n-1 on-time
                                         ranks, 2(n-2) rounds */
    SAR_SCHED_BCAST_COMPLETION = 5,   /* Broadcast baseline: whole-buffer exchange with the
                                         straggler, then doubling; log2(n) rounds of s bytes */
    SAR_SCHED_ALLREDUCE = 6     /* the precondition's rounds followed by the completion's: StragglAR
                                   with no delay to wait for (what stragglar_allreduce runs when it
                                   is given no arrival event) */
} sar_schedule;
#define SAR_NUM_SCHEDULES 7

typedef struct { int32_t src, dst, chunk, op; } sar_op;

typedef struct sar_plan sar_plan; /* opaque, owned by the library, host memory only */

#define SAR_MAX_RANKS 256

/*
 * Host-side schedule planner (Sec. 3.1, Alg. 1; generated once, offline, Sec. 4
 * "Schedule generator").  Builds, for n ranks with `straggler_rank` late and
 * buffers of `count` elements of `dtype`:
 *   - the precondition: a ring ReduceScatter over the n-1 on-time ranks, after
 *     which on-time rank g (in ascending physical order, g = 0..n-2) holds in
 *     chunk g the sum over all on-time ranks;
 *   - the completion rounds of Alg. 1, relabelled so that the on-time ranks in
 *     ascending order are the paper's ranks 0..n-2 and the straggler is n-1;
 *   - the baselines of App. E: ring AllReduce; recursive halving/doubling (both
 *     on n chunks, straggler-oblivious); and the straggler-aware Broadcast, whose
 *     precondition is a ring AllReduce among the on-time ranks and whose
 *     completion swaps the straggler's whole buffer with the first on-time rank
 *     and then doubles the set of holders every round.
 * n must be even, 2 <= n <= SAR_MAX_RANKS.  For an n that is not a power of two
 * the completion comes from App. D's generator instead of Alg. 1: each round is a
 * maximum-weight matching (weight 2 if both ranks hold a reduced chunk the other
 * lacks, 1 if one does); no bound is proven, the schedules built here take about
 * n + log2(n) rounds (the paper reports about n + 2 log2(n) - 2); planning takes
 * up to ~10 s at n = 254.  Recursive halving/doubling has no rounds then and
 * rhd_allreduce returns SAR_EUNSUPPORTED.
 * *out receives a plan to be released with stragglar_plan_destroy.  Touches no GPU.
 */
int stragglar_plan(int n, int straggler_rank, size_t count, int dtype, sar_plan** out);
/* Releases a plan (host memory only; the schedule is generated once and reused, Sec. 4
 * "Schedule generator").  NULL is accepted.  No call using the plan may be in progress. */
void stragglar_plan_destroy(sar_plan* plan);

/* Introspection (host): the schedule exactly as the execution calls run it, so that a
 * checker can replay it.  `which` is a sar_schedule.
 *   num_rounds: number of rounds of the schedule - the length of Alg. 1's `schedule` list
 *               for the completion (n + log2(n) - 2, Thm. 1), Table 1 / App. E's round
 *               counts for the baselines - or -1 on a bad argument.
 *   num_chunks: number of chunks of that schedule's chunking (Sec. 3.1: n-1; App. E: n
 *               for ring and recursive halving/doubling), or -1.
 *   round:      the set of matchings of one round (Sec. 3.1; Alg. 1 appends one such set
 *               per round) as ops: *ops points at plan-owned storage valid until destroy,
 *               *nops is its length.  SAR_EINVAL on a bad argument.
 *   chunk:      element offset and length of chunk `chunk` (the c_k of Sec. 3.1) under the
 *               chunking rule at the top of this file.  SAR_EINVAL on a bad argument. */
int stragglar_plan_num_rounds(const sar_plan* plan, int which);
int stragglar_plan_num_chunks(const sar_plan* plan, int which);
int stragglar_plan_round(const sar_plan* plan, int which, int round, const sar_op** ops, int* nops);
int stragglar_plan_chunk(const sar_plan* plan, int which, int chunk, size_t* elem_offset, size_t* elem_len);

/* How an execution call on schedule `which` would run with the settings in force now (the
 * plan's launch options, else the process-wide tunables), and what it moves.  Host only;
 * touches no GPU.  The byte counts are the HBM traffic the form has to cause when nothing is
 * cached: every load and store of a chunk counted with that chunk's true length.  For one
 * launch per round they are the per-op costs of the schedule as the paper states it (a chunk
 * sent is read once and written once; a reducing receiver also reads its own copy; Sec. 3.2
 * counts the same chunks per rank and link): 2ns for the completion, up to chunk rounding.
 *   form = 0  one launch per round, every op reads its own source
 *   form = 1  one launch per round, a round's copies of the same value read it once
 *             (SAR_TUNE_MERGE_COPIES)
 *   form = 2  all rounds in one launch per group of chunk indices (SAR_TUNE_FUSE_ROUNDS)
 *   form = 3  as 2 for the ops that produce each chunk's final value, then a launch that
 *             copies it to the ranks still lacking it (SAR_TUNE_FUSED_SPLIT) - the two in turn
 *             for one group of chunk indices after the other when the rank buffers are large;
 *             the copying launch fetches each value once (its workgroups re-read it from L2,
 *             not counted)
 * Returns SAR_EINVAL on a bad argument. */
typedef struct {
    int form;
    int launches;               /* kernel launches the call enqueues */
    unsigned long long bytes_loaded, bytes_stored;
} sar_launch_form;
int stragglar_plan_launch_form(const sar_plan* plan, int which, sar_launch_form* out);

/*
 * Execution.  `rank_bufs` is a HOST array of n DEVICE pointers; rank_bufs[i] is
 * physical rank i's flat buffer of `count` elements, 16-byte aligned, no two
 * overlapping, reduced in place.  The caller owns buffers and stream.
 * `hip_stream` is a hipStream_t (NULL = the default stream).  Each call
 * enqueues its kernels (one per round, or one for all rounds, see
 * SAR_TUNE_FUSE_ROUNDS) on that stream and returns without synchronising; rank_bufs is read before the call returns.  Argument errors
 * are detected before anything is enqueued.
 *
 * stragglar_phase1_reducescatter - the precondition (Sec. 3.1), meant to run
 *   while the straggler is late.  Afterwards the g-th on-time rank holds the
 *   partial sum of the on-time ranks in its chunk g; its other chunks are
 *   unspecified (intermediate sums with one launch per round, possibly still
 *   the input with a single launch); the straggler's buffer is untouched.
 * stragglar_phase2_complete - the n + log2(n) - 2 completion rounds (Alg. 1):
 *   the straggler's critical path.  Requires the state phase 1 leaves (not
 *   checked).  Afterwards all n buffers hold the full sum (Sec. 3.1
 *   postcondition).
 * ring_allreduce - the ring baseline of App. E on the same kernels; needs no
 *   phase 1.  Afterwards all n buffers hold the full sum.
 * rhd_allreduce - recursive halving/doubling (App. E), likewise.
 * broadcast_phase1_allreduce / broadcast_phase2_complete - the Broadcast baseline
 *   (App. E): phase 1 leaves every on-time rank with the sum over the on-time ranks
 *   and the straggler untouched; phase 2 requires that state and leaves all n
 *   buffers with the full sum (bit-identical to StragglAR's result: the additions
 *   are the same, in the same order).
 */
/*
 * stragglar_allreduce - both phases as one call, the packaging Sec. 4 ("Runtime")
 *   describes: the precondition is enqueued at once; the completion is enqueued
 *   behind `straggler_ready`, a hipEvent_t the caller records (on any stream) when
 *   the straggler's buffer is final, or directly behind the precondition if it is
 *   NULL.  Same arguments, results and errors as the two calls below; if an error
 *   is returned after the precondition was enqueued, the buffers hold its result.
 *   With no event and SAR_TUNE_FUSE_ROUNDS allowing it, both phases run as ONE
 *   launch (SAR_SCHED_ALLREDUCE): the partial sums then go from the precondition
 *   to the completion in registers.  (Where the completion alone would take its
 *   split form, see SAR_TUNE_FUSED_SPLIT, the two phases stay two calls: faster.)
 */
int stragglar_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream, void* straggler_ready);
int stragglar_phase1_reducescatter(const sar_plan* plan, void* const* rank_bufs, void* hip_stream);
int stragglar_phase2_complete(const sar_plan* plan, void* const* rank_bufs, void* hip_stream);
int ring_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream);
int rhd_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream);
int broadcast_phase1_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream);
int broadcast_phase2_complete(const sar_plan* plan, void* const* rank_bufs, void* hip_stream);

/*
 * Straggler emulation (Sec. 4.1: the late rank is idled for a set time while the
 * others start the precondition).  Enqueues on `hip_stream` a one-wavefront kernel
 * that idles for about `nanoseconds` of wall-clock time (at most 1e9, else
 * SAR_EINVAL) and exits; work queued behind it on that stream, or on streams that
 * wait on an event recorded after it, plays the part of the late rank.  The wait
 * is bounded by an iteration limit as well, so the kernel always terminates.
 */
int stragglar_delay(unsigned long long nanoseconds, void* hip_stream);

/* Launch-shape knobs (host).  stragglar_tune_set / _get act on the process-wide
 * defaults; stragglar_plan_option_set / _get on ONE plan, whose setting then wins
 * for every call made with that plan, so that callers sharing a process cannot
 * disturb each other (SAR_OPTION_INHERIT, the initial state, hands the key back
 * to the process-wide value; _get returns the value in force for the plan).
 * Setting an option while a call with the same plan is in progress on another
 * thread is a race on which shape that call takes, never on its result.  Values
 * outside the documented range return SAR_EINVAL and change nothing.  These are
 * properties of this implementation, not of the paper's method: every setting
 * computes the same bits.
 *   SAR_TUNE_BLOCKS_PER_CU  upper bound on workgroups per compute unit and round
 *                           (1..65536); 0 (default) = no bound: one workgroup per
 *                           4 KiB x UNROLL tile, which is fastest at every size; a
 *                           bounded grid strides over the tiles
 *   SAR_TUNE_UNROLL         16-byte vectors in flight per thread: 1, 2 or 4,
 *                           -1 (default) = automatic (by schedule and buffer size)
 *   SAR_TUNE_NONTEMPORAL    non-temporal (streaming) cache hints on accesses whose data
 *                           is not needed again soon: 0 = never, 1 = always,
 *                           -1 (default) = when the n buffers together exceed 256 MiB
 *   SAR_TUNE_FUSE_ROUNDS    0 = one kernel launch per round (the schedule executed round by
 *                           round, as the paper's runtime does); 1 = run all
 *                           rounds of a call in one launch (a few for many ranks: a launch
 *                           carries the ops of as many chunk indices as fit its arguments;
 *                           each workgroup takes its own 4 KiB tile of a chunk through every
 *                           round; same resulting bits, fewer launches, less HBM traffic:
 *                           values stay in registers from one round to the next, and a store
 *                           that a later round overwrites before anything reads it is dropped);
 *                           a schedule whose per-chunk op list exceeds one launch and that
 *                           has no kernel of its own (SAR_TUNE_FUSED_DIRECT) runs as 0;
 *                           -1 (default) = automatic: 1 up to 32
 *                           ranks, where it is faster at every size; above, the completion still
 *                           takes it (in its split form, see SAR_TUNE_FUSED_SPLIT) and the other
 *                           schedules whichever form a small cost model (launch count, chain
 *                           length, bytes) predicts faster
 *   SAR_TUNE_FUSED_UNROLL   16-byte vectors per thread in the single-launch kernel: 1, 2, 4,
 *                           -1 (default) = automatic
 *   SAR_TUNE_FUSED_WGS_PER_CU  cap on workgroups resident per compute unit in the single-launch
 *                           kernel: 0 = none, 2..6, -1 (default) = automatic
 *   SAR_TUNE_FUSED_SPLIT    single-launch mode, for schedules in which every chunk ends with copies
 *                           that only hand its final value on (Alg. 1: after its straggler pairing a
 *                           chunk is only ever copied): 1 = run those copies as a launch of their
 *                           own, ordered so that few ranks' buffers are written at any moment,
 *                           0 = keep them in the one launch, -1 (default) = automatic (for the
 *                           completion: split with more than 16 ranks when the buffers together
 *                           reach 512 MiB and each is at most 256 MiB, and always above 32 ranks)
 *   SAR_TUNE_FUSED_DIRECT   single-launch mode, schedules of a shape a kernel of its own exists
 *                           for: 1 = that kernel, 0 = the general op-list kernel, -1 (default) =
 *                           automatic.  The shapes: every chunk one exchange followed by copies
 *                           of the sum to all other ranks (the completion of Alg. 1; up to 32
 *                           ranks; automatic: up to 256 MiB per rank), and every chunk a reduce
 *                           chain around one ring of ranks (the ring ReduceScatter of the
 *                           precondition, Sec. 3.1, and of the ring AllReduce, App. E; any rank
 *                           count; automatic: above 32 ranks, where op lists no longer fit one
 *                           launch, for a ring AllReduce of 4-byte elements among 16 to 28
 *                           ranks and for a bf16 precondition on buffers above 256 MiB per rank)
 *   SAR_TUNE_MERGE_COPIES   with one launch per round (up to 32 ranks): 1 = a round's copies of
 *                           the same value - in a steady round of Alg. 1 every holder of the
 *                           oldest active chunk sends it, and all hold identical bits - read it
 *                           from one holder and store it to all their destinations; 0 (default)
 *                           = every op reads its own source, the schedule as written
 */
typedef enum {
    SAR_TUNE_BLOCKS_PER_CU = 0,
    SAR_TUNE_UNROLL = 1,
    SAR_TUNE_NONTEMPORAL = 2,
    SAR_TUNE_FUSE_ROUNDS = 3,
    SAR_TUNE_FUSED_UNROLL = 4,
    SAR_TUNE_FUSED_WGS_PER_CU = 5,
    SAR_TUNE_MERGE_COPIES = 6,
    SAR_TUNE_FUSED_SPLIT = 7,
    SAR_TUNE_FUSED_DIRECT = 8
} sar_tunable;
#define SAR_NUM_TUNABLES 9
#define SAR_OPTION_INHERIT (-1000L)
int stragglar_tune_set(int key, long value);
long stragglar_tune_get(int key); /* current value; -1 also for an unknown key */
int stragglar_plan_option_set(sar_plan* plan, int key, long value);
long stragglar_plan_option_get(const sar_plan* plan, int key); /* value in force; -1 also on a bad argument */

/* Text for a sar_status (static string, never NULL). */
const char* stragglar_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* STRAGGLAR_H */

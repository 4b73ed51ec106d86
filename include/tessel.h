/*
 * tessel.h -- C ABI of the MI355X (gfx950) repetend-candidate evaluator.
 *
 * The library scores candidate repetends of the Tessel schedule search (arXiv 2311.15269):
 * every candidate is one per-device ordering of the blocks of N_R consecutive micro-batches
 * plus a micro-batch index assignment; scoring means its steady-state period and its
 * per-device peak memory against a cap; the best (period, index) is kept.  All arithmetic
 * is integer (Sec. III-A).  Everything below runs on ONE GPU; the "devices" of a problem
 * are simulated entities of the schedule, not GPUs.
 *
 * Pointer conventions: `*_dev` arguments are DEVICE pointers, every other pointer is a HOST
 * pointer.  Host arrays handed to tessel_problem_create() are read during the call only.
 * The library allocates no device memory: the caller owns the workspace and the stream.
 * A workspace serves ONE problem handle at a time (the kernels keep the problem's tables, the running
 * best and their queues in it): handing it to another handle ends the first handle's search; that
 * handle's result calls then return TESSEL_E_WORKSPACE and its next scoring call starts a new search.
 * Every function returns TESSEL_OK (0) or a negative TESSEL_E_* code; nothing aborts or
 * throws across this boundary.  One problem handle must not be used from two host threads
 * at once; the only state shared between handles is the table of which handle a workspace belongs to.
 */
#ifndef TESSEL_H
#define TESSEL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- limits of this implementation -------------------------------------------------- */
#define TESSEL_MAX_DEVICES        32   /* simulated devices D (more than 8, or more than 32
                                          block types: scored by the general kernel alone;
                                          no searched completion)                            */
#define TESSEL_MAX_TYPES_PER_DEV  8    /* block types that occupy one device (more than 4:
                                          sampled spaces only; as for more than 8 devices);
                                          at most 32 blocks per device and window             */
#define TESSEL_MAX_NR             16   /* micro-batches per repetend window, N_R (more than 8:
                                          sampled spaces only; as for more than 8 devices)    */
#define TESSEL_MAX_TYPES          64   /* K (more than 32: as for more than 8 devices)      */
#define TESSEL_NUM_STATUS         6

/* ---- error codes --------------------------------------------------------------------- */
enum {
    TESSEL_OK                 = 0,
    TESSEL_E_INVALID_ARG      = -1,
    TESSEL_E_BAD_DEP          = -2,   /* the micro-batch dependency graph has a cycle            */
    TESSEL_E_UNBALANCED_MEMORY= -3,   /* sum of m over the blocks of a device != 0: no steady state */
    TESSEL_E_TOOBIG           = -4,   /* a count or a time bound exceeds what the kernels hold   */
    TESSEL_E_WORKSPACE        = -5,   /* workspace missing, misaligned or too small              */
    TESSEL_E_HIP              = -6,   /* a HIP runtime call failed (see tessel_last_hip_error)   */
    TESSEL_E_NO_FEASIBLE      = -7,   /* nothing scored so far is feasible                       */
    TESSEL_E_RANGE            = -8,   /* candidate range outside the space / too few micro-batches */
    TESSEL_E_UNSUPPORTED      = -9,   /* valid problem outside the limits above                  */
    TESSEL_E_NO_SCHEDULE      = -10   /* completion cannot order warm-up/cool-down under the cap */
};

/* ---- candidate spaces (how a 64-bit candidate index is turned into a candidate) --------
 * A candidate = a lead vector (the micro-batch index n_i of Eq. 3 for every block type,
 * 0 <= n_i < N_R) + for every device the order of its n_d = (#types on d) * N_R blocks.
 * By Property 1 (Sec. IV-B) blocks of one type run in increasing micro-batch order, so an
 * order is a sequence of type ids; the q-th occurrence of type i in window k handles
 * micro-batch n_i + q + N_R*k.
 *
 * FACTORIAL       factorial number system per device over labelled blocks
 *                 (type ascending, label 0..N_R-1): index = sum_d r_d * prod_{d'<d} n_d'!,
 *                 r_d = lexicographic permutation rank.  The first label of a type is its
 *                 lead; labels that do not continue cyclically name a Property-1 duplicate.
 * CANONICAL       index = r_0 + C_0*(r_1 + ... + C_{D-1}*lead_rank): r_d = lexicographic rank
 *                 of the device's type sequence, lead_rank = rank among the lead vectors that
 *                 satisfy Property 2 and have minimum 0, in lexicographic order.
 * SAMPLED_STRICT  index = ordinal of a counter-based pseudo-random stream keyed by `seed`
 *                 that draws leads and uniformly random type sequences; an order that can
 *                 never execute is rejected (DEADLOCK).
 * SAMPLED_REPAIR  the same draws, then a deterministic head-of-line repair that turns the
 *                 drawn priority lists into the nearest executable orders.                 */
enum {
    TESSEL_SPACE_FACTORIAL      = 0,
    TESSEL_SPACE_CANONICAL      = 1,
    TESSEL_SPACE_SAMPLED_STRICT = 2,
    TESSEL_SPACE_SAMPLED_REPAIR = 3
};

/* ---- per-candidate status; every candidate gets exactly one --------------------------- */
enum {
    TESSEL_STATUS_OK          = 0,   /* executable and within the cap: has a period             */
    TESSEL_STATUS_DUP         = 1,   /* FACTORIAL only: Property-1 duplicate of another index   */
    TESSEL_STATUS_TP_MISMATCH = 2,   /* FACTORIAL only: a multi-device block has two leads      */
    TESSEL_STATUS_PROP2       = 3,   /* a producer's lead is below its consumer's (Property 2)  */
    TESSEL_STATUS_DEADLOCK    = 4,   /* the per-device orders can never execute                 */
    TESSEL_STATUS_MEM         = 5    /* a device's peak memory exceeds the cap (Eq. 1 [2])      */
};

/* ---- problem statement (Table I, Sec. III-A) ----------------------------------------- */
typedef struct {
    int32_t  num_devices;       /* D                                                            */
    int32_t  num_block_types;   /* K blocks per micro-batch                                     */
    int32_t  nr;                /* N_R, micro-batches per repetend window (Eq. 3)               */
    int32_t  mem_cap;           /* M, the same on every device                                  */
    const int32_t  *time;       /* [K] t_B >= 1                                                 */
    const int32_t  *mem;        /* [K] m_B, negative = releases memory                          */
    const uint32_t *dev_mask;   /* [K] bit d set <=> the block occupies device d (d_B)          */
    int32_t  num_deps;          /* dependencies inside one micro-batch, B_src -> B_dst: any acyclic graph;
                                   disjoint chains score fastest, other graphs (at most 128 dependencies)
                                   on a slower general path                                       */
    const int32_t  *dep_src;    /* [num_deps]                                                   */
    const int32_t  *dep_dst;    /* [num_deps]                                                   */
    int32_t  space;             /* TESSEL_SPACE_*                                               */
    const int32_t  *fixed_leads;/* [K] or NULL; not allowed with TESSEL_SPACE_FACTORIAL         */
    uint64_t seed;              /* sampled spaces                                               */
    uint32_t lead_step_q16;     /* sampled spaces: P(lead grows by one across a dependency
                                   between different device sets) * 65536                       */
} tessel_problem_desc;

typedef struct tessel_problem tessel_problem;   /* opaque, host memory only */

/* ---- results -------------------------------------------------------------------------- */
typedef struct {
    int32_t  period;                          /* best T* (repetend time t_R, Eq. 4)            */
    uint64_t index;                           /* lowest candidate index attaining it (Alg. 1
                                                 replaces the incumbent on strict < only)      */
    int32_t  peak_mem[TESSEL_MAX_DEVICES];    /* per-device peak of the best candidate         */
    int32_t  peak_max;
    int32_t  lower_bound;                     /* N_R * max_d sum of t on d (Alg. 1 GetLowerBound) */
    uint64_t n_evaluated;
    uint64_t n_feasible;
    uint64_t n_reject[TESSEL_NUM_STATUS];     /* indexed by TESSEL_STATUS_*; [0] unused        */
    uint64_t n_window_sweeps;                 /* sweeps of the window spent on period computations
                                                 (0 when the general kernel did the scoring)    */
    uint64_t n_blocks_placed;                 /* blocks the builds placed in executable order: a candidate that
                                                 is over the cap early is not built to the end by
                                                 tessel_eval_candidates (exact in the REPAIR space, an upper
                                                 bound elsewhere; 0 when the general kernel did the scoring) */
} tessel_result;

/* A complete schedule of N micro-batches: warm-up, R copies of the best window, cool-down
 * (Sec. IV-C, Eq. 5-6).  All arrays are caller-allocated host memory. */
typedef struct {
    int32_t  num_microbatches;   /* in:  N                                                     */
    int32_t  capacity;           /* in:  elements available in start[] and in each row of
                                         dev_order[]; needs K*N                                 */
    int32_t *start;              /* out: [K*N] start time of block (type, mu) at type*N + mu    */
    int32_t *dev_order;          /* out: [D][capacity] blocks (type*N+mu) in execution order    */
    int32_t *dev_len;            /* out: [D]                                                    */
    int32_t  makespan;           /* out: max end time (objective of Eq. 1)                      */
    int32_t  period;             /* out: T* of the window that was repeated                     */
    int32_t  num_windows;        /* out: R                                                      */
} tessel_schedule;

/* Validates the problem statement (Sec. III-A) and builds the host-side tables.
 * Errors: INVALID_ARG, BAD_DEP, UNBALANCED_MEMORY, UNSUPPORTED, TOOBIG. */
int  tessel_problem_create(const tessel_problem_desc *desc, tessel_problem **out);
void tessel_problem_destroy(tessel_problem *p);

/* Number of candidates of the problem's space; UINT64_MAX for the sampled spaces (any
 * ordinal is a candidate). */
int  tessel_candidate_count(const tessel_problem *p, uint64_t *count);

/* Bytes of device workspace tessel_eval_candidates / tessel_score_candidates need: the running best, the list of
 * candidates left to the general kernel (8 MiB) and, for problems the fast kernel takes, three queues per resident
 * wave between the phases of the kernel (3 x 27 KB per wave for 256 blocks a window; a few hundred MB in all).  Sized for the current
 * device (for 512 compute units where there is none to ask); a workspace too small for the device a call runs on is
 * refused there with TESSEL_E_WORKSPACE. */
int  tessel_workspace_bytes(const tessel_problem *p, size_t *bytes);

/* Scores candidates first .. first+count-1 (Alg. 1, the loop over repetends: decode,
 * validity, period, memory) and merges into the running best of `p` under the total order
 * (period, index).  Asynchronous on `hip_stream` (a hipStream_t, NULL = default stream).
 * May be called again with any other range, in any order; the running best and the
 * counters live in `workspace_dev`, which must be the same 256-byte aligned buffer for all
 * calls of one search.  tessel_reset() starts a new search. */
int  tessel_eval_candidates(tessel_problem *p, uint64_t first, uint64_t count,
                            void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): tessel_eval_candidates without a workspace argument.  The running best,
 * the problem's tables and the kernels' queues live in a buffer that is part of the library's code object
 * (TESSEL_NOALLOC_SCRATCH_BYTES of device memory on every GPU the library runs on, held until the process
 * ends); the grid shrinks to the workgroups whose queues fit it (about a hundred of the 4096 the chip holds
 * for windows of 256 blocks, all of them for small windows), so this call can be much slower than the one above.  No hipMalloc, hipFree or other allocating call
 * is made.  Every call on a GPU shares that GPU's buffer: it serves one handle at a time like any workspace
 * (another handle's call ends this handle's search), and calls that overlap on one GPU, from different
 * streams or threads, race.  tessel_best, tessel_reset, tessel_best_candidate, tessel_complete_schedule and
 * the completion search apply as after tessel_eval_candidates.
 * Errors: RANGE, TOOBIG (count above TESSEL_NOALLOC_MAX_CANDIDATES per call), HIP. */
#define TESSEL_NOALLOC_SCRATCH_BYTES   (24u << 20)
#define TESSEL_NOALLOC_MAX_CANDIDATES  (1ull << 26)
int  tessel_eval_candidates_noalloc(tessel_problem *p, uint64_t first, uint64_t count, void *hip_stream);

/* Per-candidate records for tests and analysis: code_dev[k] = T* of candidate first+k when
 * it is feasible, else -(TESSEL_STATUS_*); peak_dev[k] (may be NULL) = its largest
 * per-device peak when the status is OK or MEM, else 0.  Does not touch the running best. */
int  tessel_score_candidates(tessel_problem *p, uint64_t first, uint64_t count,
                             int32_t *code_dev, int32_t *peak_dev,
                             void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* Waits for the stream of the last call, then returns the running best.  NO_FEASIBLE when
 * nothing feasible has been scored (counters in *out are still valid).  If a launch left more
 * candidates to the general kernel than its list holds (2^20 of a range of up to 2^26: possible only
 * when most periods need more than the fast kernel's ten sweeps), every range scored since the last
 * reset is scored again here in smaller pieces before the result is returned.  WORKSPACE: the buffer
 * was bound to another handle in the meantime. */
int  tessel_best(tessel_problem *p, tessel_result *out);

/* Decoded form of the best candidate as the GPU decoded it: leads[K], order_len[D] and
 * orders[D][32] (block type ids in device order, after repair in the REPAIR space), and
 * its least start times at T*: starts[K*N_R] at type*N_R + occurrence. Any pointer may be NULL. */
int  tessel_best_candidate(tessel_problem *p, int32_t *leads, int32_t *order_len, int32_t *orders,
                           int32_t *starts);

/* Forgets the running best and the counters. */
int  tessel_reset(tessel_problem *p);

/* Extends the best window to N micro-batches (Sec. IV-C): warm-up and cool-down block sets
 * of Eq. 5-6, ordered by a deterministic greedy list schedule (instead of the paper's
 * time-optimal solver), R = floor((N - max lead)/N_R) windows in between; start times are
 * the earliest ones for that per-device order.  Errors: NO_FEASIBLE, RANGE (R < 1 or
 * capacity too small), NO_SCHEDULE. */
int  tessel_complete_schedule(tessel_problem *p, tessel_schedule *out);

/* ---- searched completion (Sec. IV-C; the paper orders warm-up and cool-down with a time-optimal solver) ---
 * Completion candidate `ordinal` is a perturbed greedy list schedule of the two outer phases around the R
 * copies of the best window: per phase every block type offers its lowest unscheduled micro-batch
 * (Property 1); an offered block is eligible when its producers' blocks of the same micro-batch are scheduled
 * and its memory delta fits on all its devices; the eligible block with the smallest (earliest start +
 * jitter, micro-batch, type id) is appended at its earliest start.  jitter(type, mu) = (draw * (J + 1)) >> 16
 * with the 16-bit draw number type*N + mu of the counter-based stream keyed by (seed + 0x632BE59BD9B4E019,
 * ordinal); ordinal 0 has no jitter and is the schedule of tessel_complete_schedule.
 *
 * tessel_search_completions scores candidates first .. first+count-1 on the GPU (one per lane: warm-up and
 * cool-down block by block, the R windows between them as the one linear map in the (max, +) algebra that
 * they are for every candidate) and merges into the running best (makespan, lowest ordinal).  The first call
 * for a best window waits for it (as tessel_best does); the scoring itself is asynchronous on the stream of the
 * last tessel_eval_candidates call, in the workspace bound there.  A new best window, N or J restarts the
 * running best.  Errors: NO_FEASIBLE, RANGE (fewer than one window fits), INVALID_ARG,
 * TOOBIG (state of N micro-batches does not fit the LDS, N * sum of t exceeds 16 bits, N > 1023 or J > 63),
 * UNSUPPORTED (|m| > 127; more than 8 devices, 32 block types, 4 types on a device or 8 micro-batches per
 * window), HIP. */
int  tessel_search_completions(tessel_problem *p, int32_t num_microbatches, int32_t jitter, uint64_t first,
                               uint64_t count);
/* makespan_dev[k] (device, int32) = makespan of completion candidate first+k, INT32_MAX where the greedy rule
 * gets stuck under the memory cap.  Does not touch the running best. */
int  tessel_score_completions(tessel_problem *p, int32_t num_microbatches, int32_t jitter, uint64_t first,
                              uint64_t count, int32_t *makespan_dev);
/* Waits, then writes the complete schedule of the best completion candidate scored so far (out as for
 * tessel_complete_schedule, num_microbatches as searched) and its ordinal.  Errors: NO_FEASIBLE (nothing
 * searched), NO_SCHEDULE (no candidate had a schedule), INVALID_ARG, RANGE, HIP. */
int  tessel_best_completion(tessel_problem *p, tessel_schedule *out, uint64_t *ordinal);

/* ---- runtime instantiation (Sec. IV-D): the global operation sequence of a complete schedule --------
 * Blocks in ascending start time; blocks that start together are consecutive, ordered by their lowest
 * device (a device's own blocks keep its execution order).  A tensor that a consumer needs on a device
 * where its producer did not run is one send/receive pair, a single operation placed right after the
 * time slot (group of equal start times) of the producer; the sender is the producer's lowest device;
 * pairs of one slot follow their producers' order, then the dependency's position in the problem
 * statement, then the receiving device.  Every device executes, in this order, the operations it takes
 * part in; the common order rules out mismatched send/receive pairs. */
enum { TESSEL_OP_BLOCK = 0, TESSEL_OP_SENDRECV = 1 };
typedef struct {
    int32_t kind;    /* TESSEL_OP_*                                                           */
    int32_t block;   /* type*N + mu; for a pair: the producer                                 */
    int32_t src;     /* block: device mask;  pair: sending device                             */
    int32_t dst;     /* block: start time;   pair: receiving device                           */
    int32_t aux;     /* block: 0;            pair: the consumer block                         */
} tessel_op;

/* Writes the sequence of `sched` (as filled in by tessel_complete_schedule: num_microbatches and start[]
 * are read) to ops[0 .. *num_ops-1] (host memory, `capacity` elements).  Host work only.
 * Errors: INVALID_ARG (null pointer, a block without start time), RANGE (capacity too small; *num_ops
 * then holds the number needed). */
int  tessel_instantiate(const tessel_problem *p, const tessel_schedule *sched, tessel_op *ops, int32_t capacity,
                        int32_t *num_ops);

/* ---- the whole search of Alg. 1 (Sec. IV-C): all window sizes ---------------------------
 * In: which window sizes and how many candidates of each; out: the incumbent and what each
 * window size gave.  Repetend times of different window sizes compare per micro-batch:
 * T_a/N_a < T_b/N_b  <=>  T_a*N_b < T_b*N_a. */
typedef struct {
    int32_t  max_nr;              /* in:  largest N_R tried, 1..TESSEL_MAX_NR                            */
    int32_t  use_inflight_bound;  /* in:  non-zero: stop at N_R = CalMaxInflight as Alg. 1 does           */
    uint64_t max_candidates;      /* in:  per window size, indices 0 .. min(space size, this) - 1 are scored */
    uint64_t launch_candidates;   /* in:  candidates per kernel launch; the early exit is tested between
                                          launches; 0 = 2^24                                              */
    int32_t  inflights;           /* out: CalMaxInflight: min over devices of floor(M / hold_d), hold_d =
                                          what one micro-batch alone holds on d at most (blocks in
                                          topological order, smallest type id first); max_nr if
                                          nothing holds memory                                            */
    int32_t  lower_bound;         /* out: GetLowerBound: max_d sum of t on d, per micro-batch             */
    int32_t  nr_tried;            /* out: window sizes entered                                            */
    int32_t  best_nr;             /* out: window size of the incumbent, 0 = nothing feasible              */
    int32_t  best_period;         /* out: its T* (per micro-batch: best_period / best_nr), -1 = none      */
    int32_t  early_exit;          /* out: 1 = the lower bound was reached and the search stopped there    */
    uint64_t best_index;          /* out: its candidate index in the space of window size best_nr         */
    int32_t  period_nr[TESSEL_MAX_NR + 1];      /* out: best T* of window size n at [n], -1 = none        */
    uint64_t index_nr[TESSEL_MAX_NR + 1];       /* out: lowest index attaining it                         */
    uint64_t evaluated_nr[TESSEL_MAX_NR + 1];   /* out: candidates scored (whole launches)                */
} tessel_search;

/* Device workspace tessel_search_run needs for the window sizes that `in` (its max_nr and
 * use_inflight_bound are read) selects for `desc` (desc->nr is ignored).  Errors: as
 * tessel_problem_create. */
int  tessel_search_workspace_bytes(const tessel_problem_desc *desc, const tessel_search *in, size_t *bytes);

/* Alg. 1: for N_R = 1 .. min(max_nr, inflights) score the candidates of that window size in
 * ascending index order, launch by launch, keep the incumbent under strict <, and stop as soon
 * as a window reaches N_R * lower_bound.  The incumbent starts empty (the paper starts it at the
 * serial time, which would leave a problem that cannot beat serial execution without any
 * schedule).  desc->nr and desc->fixed_leads are ignored.  Synchronises `hip_stream` between
 * launches.  On success *best_out (if not NULL) is a new problem handle of window size
 * best_nr, bound to `workspace_dev`, whose running best is the incumbent: tessel_best,
 * tessel_best_candidate and tessel_complete_schedule apply; the caller destroys it.
 * Errors: those of tessel_problem_create for any window size, WORKSPACE, HIP, and NO_FEASIBLE
 * (the fields of *io are still filled in; no handle is returned). */
int  tessel_search_run(const tessel_problem_desc *desc, tessel_search *io, void *workspace_dev,
                       size_t workspace_bytes, void *hip_stream, tessel_problem **best_out);

/* Measurement aid, not part of the method: launches a kernel of `blocks` x 256 threads in which
 * every lane runs `rounds` rounds of 32 independent full-rate 32-bit integer VALU operations
 * (add, unsigned max), asynchronously on `hip_stream`.  *lane_ops (host, may be NULL) receives the
 * number of lane operations of the launch; divided by the launch's duration it is the integer
 * VALU rate the chip sustains in practice, the second denominator beside the published peak.
 * out_dev: device buffer of blocks*256 uint32 (overwritten).  Errors: INVALID_ARG, WORKSPACE
 * (out_bytes too small), HIP. */
int  tessel_alu_probe(int blocks, int rounds, uint32_t *out_dev, size_t out_bytes, void *hip_stream,
                      uint64_t *lane_ops);

const char *tessel_strerror(int code);
int  tessel_last_hip_error(const tessel_problem *p);   /* hipError_t of the last failure, 0 if none */

#ifdef __cplusplus
}
#endif
#endif /* TESSEL_H */

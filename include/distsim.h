/*
 * distsim.h -- C ABI of the batched DistSim strategy evaluator for AMD MI355X (gfx950).
 *
 * The library evaluates many candidate hybrid-parallel training strategies at once,
 * following DistSim (arXiv 2306.08423): profiled per-layer event times are composed into
 * per-stage events (Sec. 4.3, model-parallel modelling), the pipeline schedule is replayed
 * with the dependency rule of Algorithm 1 (pipeline modelling), the data-parallel gradient
 * all-reduce is appended (data-parallel modelling), and the resulting timeline is reduced
 * to the iteration ("batch") time and per-device activity (Sec. 3.2, Sec. 5); the grid
 * search of Sec. 6 picks the best candidate.
 *
 * Conventions that hold for every call
 *  - Every call makes the context's device current for its own duration and restores the
 *    caller's current device before it returns.
 *  - "device pointer" = memory of the HIP device the context was created on, owned by the
 *    caller (e.g. a PyTorch tensor).  The library never frees or reallocates caller memory
 *    and allocates no device memory itself; everything it needs beyond the inputs and
 *    outputs lives in distsim_events.workspace, which the caller sizes with
 *    distsim_workspace_bytes().
 *  - Work is enqueued on the hipStream_t passed as `hip_stream` (NULL = the default
 *    stream); no call synchronises.  Results are valid once that stream has reached them.
 *  - All times are int64 nanoseconds, all sizes int64 bytes.
 *  - Return value: DISTSIM_OK, or a negative code; text via distsim_last_error().
 *    A *candidate* that is not a valid strategy is not a call error: see `status`.
 *  - Preconditions on table entries (device memory, not checked): 0 <= time < 2^40 ns,
 *    0 <= bytes < 2^40.  The cluster description (host memory) is checked: 0 <= alpha < 2^40,
 *    1 <= beta < 2^32, num_devices <= 2^22, bucket bytes < 2^53, else DISTSIM_ERANGE.  Together
 *    they keep every product in the collective formulas below within 63 bits.
 */
#ifndef DISTSIM_H
#define DISTSIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DISTSIM_OK       0
#define DISTSIM_EINVAL  (-1)   /* null pointer, negative size, inconsistent arguments        */
#define DISTSIM_ERANGE  (-2)   /* a cost or bound of the cluster description would let the
                                  collective formulas leave their integer range: alpha >= 2^40,
                                  beta >= 2^32, bucket bytes >= 2^53 or more than 2^22 devices
                                  (table entries live in device memory and are not inspected by
                                  the host; times that would pass 2^53 are caught per candidate,
                                  see DISTSIM_ST_RANGE)                                        */
#define DISTSIM_EHIP    (-3)   /* HIP runtime error                                          */
#define DISTSIM_ELIMIT  (-4)   /* a size is beyond a documented limit of this library (C, L, V,
                                  n, K)                                                        */

#define DISTSIM_MAX_PP   64    /* pipeline stages per candidate (one 64-lane wavefront)      */
#define DISTSIM_MAX_L    255   /* layers (partition boundaries are bytes)                    */
#define DISTSIM_MAX_V    16    /* tensor-parallel variants in a cost table                   */

#define DISTSIM_GPIPE    0     /* all forwards, then all backwards (Sec. 2.1.3)              */
#define DISTSIM_1F1B     1     /* Dapple early backward: at most pp - s micro-batches alive  */
#define DISTSIM_INTERLEAVED 3  /* interleaved one-forward-one-backward (Narayanan et al., SC 2021;
                                  an extension in the sense of the paper's Sec. 7: a new pipeline
                                  algorithm enters through its schedule).  Every device holds
                                  chunks[c] model chunks; virtual stage k = chunk * pp + device
                                  owns the k-th of pp * chunks parts of the layers (part_pool
                                  then holds pp * chunks + 1 boundaries).  Needs m % pp == 0,
                                  pp * chunks <= L (more than 64 virtual stages is
                                  DISTSIM_ST_UNSUPPORTED).  Forward slot i
                                  of a device: chunk (i mod (pp chunks)) / pp, micro-batch
                                  (i / (pp chunks)) pp + i mod pp; backward slot i: the mirrored
                                  chunk.  Device d runs 2 (pp-d-1) + (chunks-1) pp forwards,
                                  then forward / backward in turn, then the backwards left.
                                  One trailing gradient all-reduce per device; with a bucket
                                  size the device fills its buckets across its chunks (a chunk's
                                  gradients are complete in its backward of micro-batch m - 1,
                                  last layer first).  Per-stage outputs are per device; no
                                  stage table.                                                  */
#define DISTSIM_EXPLICIT 4     /* the schedule S of Algorithm 1 given by the caller (Sec. 4.3: which device
                                  runs which stage-task of which micro-batch, in which order; Sec. 7: a
                                  new pipeline algorithm enters through its schedule).  chunks[c] names
                                  one of the schedules in distsim_candidates.schedule_words, a block of
                                  32-bit words:
                                    [0] pp  [1] S virtual stages (<= 64)  [2] m  [3] nparts: parts of the
                                    layer partition the stages refer to (<= min(64, L); part_pool then
                                    holds nparts + 1 boundaries)  [4] replicas >= 1: a device's gradient
                                    all-reduce spans dp * replicas ranks
                                    [5 .. 5+pp] first task of each device's list, then the task total
                                    S triples: device of the stage, its part, the stage before it in
                                    its pipeline (-1: none; at most one stage after any stage)
                                    the tasks, device after device: kind << 31 | stage << 16 |
                                    micro-batch, kind 0 = forward; each at most once, on the device of
                                    its stage.
                                  F(k, j) needs F(prev k, j) and its p2p event (the activation leaving
                                  prev k's part; link class by the nodes of the two devices); B(k, j)
                                  needs B(next k, j) and its p2p event, or on a stage without successor
                                  its own F(k, j).  A device runs its list in order.  One gradient
                                  all-reduce per device after its list, over the bytes of the parts of
                                  all its stages; with a bucket size the device fills its buckets across
                                  its stages (a stage's gradients are complete in its last backward task
                                  on the list, last layer first; a stage without a backward task adds
                                  nothing).  pp and m must equal the candidate's.  A schedule that
                                  cannot be run to its end is invalid, as is a malformed block; one with
                                  S > 64, nparts > 64 or S * m > DISTSIM_MAX_SLOTS is
                                  DISTSIM_ST_UNSUPPORTED.  Per-stage outputs are per device; no stage
                                  table.  distsim_build_events turns every schedule into a program
                                  once (the order of the tasks does not depend on the durations) and
                                  distsim_simulate runs the candidates from it; the schedules after the
                                  first 4096, those whose blocks reach beyond the first 2^17 words of
                                  schedule_words and those in which more than min(16, 128 / S) ends of
                                  one stage wait for their consumers at a time take a slower path with
                                  the same results.                                                */
#define DISTSIM_MAX_SLOTS 2048 /* (virtual stage, micro-batch) pairs of an explicit schedule       */
#define DISTSIM_1F1B_ASYNC 2   /* asynchronous pipeline (Sec. 7, discussion of new algorithms):
                                  the Dapple order without the global synchronisation event, i.e.
                                  no gradient all-reduce event is appended to the device lists   */

/* per-candidate status written by distsim_build_events */
#define DISTSIM_ST_OK       0
#define DISTSIM_MAX_M    65536 /* micro-batches per candidate                                 */
#define DISTSIM_ST_INVALID  1  /* "unreachable" strategy (Sec. 6): dp*tp*pp != devices, pp > L,
                                  pp > DISTSIM_MAX_PP, m < 1, no table variant for tp, unknown
                                  schedule, or a partition that is not 0 = b0 < b1 < ... < bpp = L */
#define DISTSIM_ST_RANGE    2  /* m * (sum of all stage-task and p2p durations) >= 2^53        */
#define DISTSIM_ST_NOROOM   3  /* valid, but its stages do not fit stage_cap                    */
#define DISTSIM_ST_UNSUPPORTED 4 /* passes every check that takes O(1) per candidate, but lies beyond
                                  what the kernels of this library simulate: m > DISTSIM_MAX_M; an
                                  interleaved candidate with pp * chunks > 64; an explicit schedule
                                  with S > 64, nparts > 64 or S * m > DISTSIM_MAX_SLOTS.  Not a statement
                                  about the strategy: the method itself has no such bounds.  Treated
                                  like an invalid candidate by every call (batch_ns = INT64_MAX).  */

typedef struct distsim_ctx distsim_ctx;   /* opaque; host-side state only (device id, error text, timers) */

/* Create / destroy a context bound to HIP device `hip_device`: host memory, one HIP stream of
 * default priority and two events (for long lists distsim_build_events and distsim_simulate run
 * some kernels on that stream next to those on the caller's, forked from and joined to the
 * caller's stream inside the call; that is safe under stream capture).
 * A context serves one host thread at a time.
 * One tuning knob is read from the environment here: DISTSIM_SPLIT_MIN_ITEMS, the list length
 * from which the two calls use the second stream and distsim_simulate gives the GPipe
 * candidates a launch of their own (default 262144 candidates; 0 = always).  Results do not depend on it. */
int         distsim_create(distsim_ctx **out, int hip_device);
void        distsim_destroy(distsim_ctx *ctx);
/* Text of the last error on this context; valid until the next call on it. */
const char *distsim_last_error(const distsim_ctx *ctx);

/*
 * Profiled per-layer event times (the output of the event profiler, Sec. 4.2), one row per
 * tensor-parallel variant: arrays are device pointers of V*L entries, entry [v*L + l].
 * A layer of variant v is mapped to the composed event {computation, all-reduce} when
 * variant_tp[v] > 1 and to the single computation event when it is 1 (Sec. 4.3); a layer
 * with a2a_bytes > 0 additionally runs one all-to-all over the dp group per pass.
 */
typedef struct {
    int32_t L, V;                    /* 1 <= L <= DISTSIM_MAX_L, 1 <= V <= DISTSIM_MAX_V          */
    const int32_t *variant_tp;       /* [V] device: tensor-parallel size the row was profiled for */
    const int64_t *fwd_comp_ns;      /* forward computation event                                 */
    const int64_t *bwd_comp_ns;      /* backward computation event                                */
    const int64_t *fwd_comm_ns;      /* in-layer blocking all-reduce event(s), forward            */
    const int64_t *bwd_comm_ns;      /* same, backward                                            */
    const int64_t *act_bytes;        /* activation sent if a stage ends after this layer          */
    const int64_t *grad_bytes;       /* gradient bytes this layer contributes to the DP all-reduce */
    const int64_t *a2a_bytes;        /* all-to-all payload (0 = none); may be NULL                */
} distsim_costs;

/*
 * Simulated cluster, passed by value in host memory.  Collective events are evaluated as
 *   p2p(P, k)       = alpha[k] + P / beta[k]
 *   allreduce(n, P) = alpha[k] + (2 (n-1) P) / (n beta[k])     ring volume 2(N-1)P/N, Sec. 4.2
 *   alltoall(n, P)  = alpha[k] + ((n-1) P) / (n beta[k])
 * with truncating integer division in exactly this order; n = 1 or P = 0 means no event.
 * Link class k: 0 = intra-node, 1 = inter-node (the communication events' attribute of
 * Sec. 4.1).  A collective over n ranks is intra-node iff n <= gpus_per_node; the boundary
 * between stages s and s+1 is intra-node iff floor(s tp dp / g) == floor((s+1) tp dp / g)
 * (ranks ordered tp fastest, then dp, then pp).
 */
typedef struct {
    int32_t num_devices;             /* dp*tp*pp of every valid candidate                         */
    int32_t gpus_per_node;
    int64_t alpha_ns[2];
    int64_t beta_bytes_per_ns[2];    /* 1 GB/s == 1 byte/ns                                       */
    int64_t dp_bucket_bytes;         /* 0: one all-reduce after the last backward (Sec. 4.3);
                                        > 0: gradient buckets of this size, each issued as soon
                                        as the last micro-batch's backward has produced it       */
    int32_t p2p_blocking;            /* 0: the p2p event is latency on the edge to the neighbouring
                                        stage, the sender goes on with its next task (default);
                                        1: the sender's device is occupied for the p2p event, which
                                        then counts as the tail of the stage-task, and the
                                        neighbour may start when it ends;
                                        2: the sender goes on, but sends queue on their link: each
                                        boundary carries one transfer per direction at a time, a
                                        send starts when its task has ended and the previous send
                                        over that link has arrived (slower kernel; an extension,
                                        the paper models no contention).  A link is an ordered pair
                                        (sending device, receiving device): with several virtual
                                        stages per device (interleaved, explicit schedules) all
                                        transfers between the same two devices share its queue    */
} distsim_cluster;

/* Candidate strategies "xM xP xD" (Sec. 5.1) x micro-batches x schedule x partition.
 * Struct of arrays, device pointers, C entries each. */
typedef struct {
    const int32_t *dp, *tp, *pp, *m;
    const uint8_t *schedule;         /* DISTSIM_GPIPE / _1F1B / _1F1B_ASYNC / _INTERLEAVED / _EXPLICIT */
    const int64_t *part_off;         /* -1: uniform split, stage s owns layers [s L / pp, (s+1) L / pp);
                                        else offset into part_pool of b0..bpp                    */
    const uint8_t *part_pool;        /* concatenated boundaries; may be NULL if never referenced  */
    int64_t part_pool_len;           /* entries in part_pool (offsets beyond it => invalid)       */
    const int32_t *chunks;           /* model chunks per device of DISTSIM_INTERLEAVED candidates,
                                        index of its schedule for DISTSIM_EXPLICIT ones (ignored for
                                        the other schedules); NULL = the list has no such
                                        candidate (one that is there anyway is invalid)            */
    int64_t n_schedules;             /* explicit schedules (see DISTSIM_EXPLICIT); 0 = none        */
    const int64_t *schedule_off;     /* [n_schedules + 1] device: first word of each schedule      */
    const int32_t *schedule_words;   /* device                                                     */
    int64_t schedule_words_len;      /* words in schedule_words (a schedule beyond it => invalid)  */
} distsim_candidates;

/* Columns of distsim_events.stage_tab: per pipeline stage of a candidate */
enum {
    DISTSIM_COL_FC = 0,   /* forward computation time of the stage's layers                       */
    DISTSIM_COL_FA = 1,   /* forward communication time inside the stage (all-reduce, all-to-all) */
    DISTSIM_COL_BC = 2,   /* backward computation                                                 */
    DISTSIM_COL_BA = 3,   /* backward communication inside the stage                              */
    DISTSIM_COL_PF = 4,   /* p2p event to stage s+1 after a forward (0 on the last stage)         */
    DISTSIM_COL_PB = 5,   /* p2p event to stage s-1 after a backward (0 on the first stage)       */
    DISTSIM_COL_G  = 6,   /* gradient bytes of the stage                                          */
    DISTSIM_COL_AR = 7,   /* duration of the single trailing gradient all-reduce (0 = no event)   */
    DISTSIM_NCOLS  = 8
};

/*
 * The event flow of all candidates: output of distsim_build_events, input of
 * distsim_simulate.  All pointers are caller-allocated device memory.
 *
 * Per-stage arrays (stage_tab, stage_layers and the per-stage outputs of distsim_simulate)
 * are laid out in the order in which the library visits candidates, not in the caller's
 * order: candidate c with status[c] == DISTSIM_ST_OK owns the entries
 * stage_pos[c] .. stage_pos[c] + pp - 1.  A candidate occupies pp rounded up to a power of
 * two entries and candidates of equal rounded size are packed 64 entries to a wavefront, so
 *   stage_cap >= distsim_stage_entries(C)   (= 64 C + 448, always enough), or any tighter
 *   bound >= U = 64 * sum over k of ceil(n_k 2^k / 64) with n_k = candidates whose rounded pp is 2^k;
 * candidates that do not fit get DISTSIM_ST_NOROOM.  Of the first min(U, stage_cap rounded down
 * to a multiple of 64) entries, those not owned by any candidate are written as zero; entries
 * from there on are not touched.
 *
 * The stage table is an optional product: the events proper are the shared layer-event tables
 * kept in the workspace (every candidate that generates an event reuses its time, Sec. 3.2),
 * and distsim_simulate composes them per stage itself, with the same arithmetic.  With
 * stage_tab == NULL nothing per-stage is written by distsim_build_events; status then only
 * reflects the checks that need no per-stage work (everything but the partition and the 2^53
 * guard) and num_events is not yet written -- distsim_simulate completes both.
 */
typedef struct {
    int64_t  stage_cap;      /* entries available in every per-stage array                        */
    int32_t  L, V;           /* table shape; filled in by distsim_build_events                    */
    int32_t *status;         /* [C]                                                               */
    int64_t *stage_pos;      /* [C] first per-stage entry of the candidate, -1 if it has none     */
    int64_t *stage_tab;      /* [DISTSIM_NCOLS][stage_cap], or NULL: do not write the table       */
    int32_t *stage_layers;   /* [stage_cap] first layer | (one past last layer) << 8; NULL iff
                                stage_tab is NULL                                                 */
    int64_t *num_events;     /* [C] events on the pp distinct device timelines: 2 m pp stage-tasks
                                + 2 m (pp-1) p2p + gradient all-reduce events; 0 if not OK       */
    void    *workspace;      /* distsim_workspace_bytes() bytes, 256-byte aligned; opaque         */
    size_t   workspace_bytes;
    int64_t  num_candidates; /* C of the call that produced the events; filled in by
                                distsim_build_events, checked by distsim_simulate / _timeline     */
} distsim_events;
/* The struct holds nothing of the caller's inputs: the calls that follow distsim_build_events take
 * the candidate arrays again as an argument and find everything they need of the cost table in
 * the workspace, so the cost table may be released once distsim_build_events has run. */

/* A stage_cap that is always enough for C candidates. */
int64_t distsim_stage_entries(int64_t C);

/* Bytes of distsim_events.workspace needed for tables of (L, V) and C candidates; 0 if a size is
 * outside its limit. */
size_t distsim_workspace_bytes(int32_t L, int32_t V, int64_t C);

/*
 * One allocation for all arrays of a distsim_events.  distsim_events_bytes: device bytes needed for
 * status, stage_pos, num_events and the workspace of C candidates of a cost table of shape
 * (costs->L, costs->V; its pointers are not read), plus stage_tab and stage_layers of stage_cap
 * entries when with_stage_table != 0; every array starts on a 256-byte boundary.  0 if a size is
 * outside its limit.  distsim_events_bind: fills *ev (every field) with pointers into `memory`
 * (device, 256-byte aligned, at least distsim_events_bytes() bytes) laid out that way; host-side
 * pointer arithmetic only.  Errors: EINVAL, ELIMIT.
 */
size_t distsim_events_bytes(const distsim_costs *costs, int64_t C, int64_t stage_cap, int with_stage_table);
int    distsim_events_bind(distsim_events *ev, void *memory, size_t memory_bytes, const distsim_costs *costs,
                           int64_t C, int64_t stage_cap, int with_stage_table);

/*
 * Event-flow generation (Sec. 4.1 events -> Sec. 4.3 composed events).  For every candidate:
 * validate, map layers to composed events, evaluate collective events, reduce the layer
 * events of each stage (segmented sums over the layer axis) and write the stage table.
 * Also prepares, inside the workspace, the order in which distsim_simulate visits candidates.
 * Errors: EINVAL (null pointers, workspace too small, stage_cap < 0), ERANGE (cluster), ELIMIT
 * (C, L or V outside their limits), EHIP.  C == 0 is valid.
 */
int distsim_build_events(distsim_ctx *ctx, const distsim_costs *costs, const distsim_cluster *cluster,
                         const distsim_candidates *cand, int64_t C, distsim_events *out,
                         void *hip_stream);

/*
 * Timeline simulation.  Replays every candidate's schedule with the rule of Algorithm 1:
 * a stage-task starts at max(end of the previous task on the same device, end of the
 * producing task on the neighbouring stage + its p2p event), runs for the stage's composed
 * duration, then the gradient all-reduce event(s) follow the device's last backward.
 * Outputs (device): batch_ns[C] = time of the last event (INT64_MAX unless status OK);
 * comp_busy_ns / comm_busy_ns [stage_cap] = sum of the durations of the computation /
 * communication events on each stage's device (index stage_pos[c] + s); util (may be NULL)
 * = comp_busy / batch as fp64; of the entries that the library lays candidates out in (the first
 * min(U, stage_cap) of distsim_build_events' description), those not owned by an OK candidate are
 * written as zero; entries from there on are not touched.
 * Also writes num_events[c], and the status of candidates whose partition is invalid or
 * whose times would leave the 2^53 range (final values; distsim_build_events has already
 * written the same ones if it was asked for the stage table).  `events` must come from
 * distsim_build_events with the same cluster, candidates and C.  Errors: EINVAL, ERANGE, ELIMIT, EHIP.
 */
int distsim_simulate(distsim_ctx *ctx, const distsim_cluster *cluster, const distsim_candidates *cand,
                     const distsim_events *events, int64_t C, int64_t *batch_ns, int64_t *comp_busy_ns,
                     int64_t *comm_busy_ns, double *util, void *hip_stream);

/*
 * Strategy search (Sec. 6): best[0] = index of the best candidate, best[1] = its batch_ns
 * (device, 2 x int64).  objective 0: smallest batch_ns.  objective 1: smallest
 * batch_ns / weight (weight[C] device, e.g. samples per iteration), compared exactly as
 * batch_a * w_b < batch_b * w_a in 128 bits.  Ties go to the lowest index.  Candidates with
 * batch_ns == INT64_MAX (or weight <= 0 under objective 1) never win; if none is left,
 * best = {-1, INT64_MAX}.  `scratch` is device memory of distsim_search_scratch_bytes(C)
 * bytes.  Errors: EINVAL, EHIP.
 */
size_t distsim_search_scratch_bytes(int64_t C);
int distsim_search(distsim_ctx *ctx, const int64_t *batch_ns, const int64_t *weight, int64_t C,
                   int objective, int64_t *best, void *scratch, void *hip_stream);

/*
 * distsim_search for callers that cannot allocate device memory or hand any over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as distsim_search, minus `scratch`: the per-workgroup partial results live in a device
 * array inside the library, DISTSIM_SEARCH_STATIC_SCRATCH_BYTES (48 KiB) on every GPU the library
 * is used on, held until the process ends; its address was taken when the context was created.
 * The call allocates nothing (no device memory, no events, no host-side growth) and never
 * synchronises; it is not timed by distsim_timing_enable.  At most DISTSIM_SEARCH_STATIC_MAX_C
 * candidates, else ELIMIT.  All calls on one GPU share the array: two that may overlap in time
 * (different streams, threads or contexts of that GPU) race; calls on one stream are ordered
 * and every call overwrites what it reads, so nothing has to be cleared in between.
 */
#define DISTSIM_SEARCH_STATIC_SCRATCH_BYTES (2048 * 24)
#define DISTSIM_SEARCH_STATIC_MAX_C 2147483647LL
int distsim_search_static(distsim_ctx *ctx, const int64_t *batch_ns, const int64_t *weight, int64_t C,
                          int objective, int64_t *best, void *hip_stream);

/*
 * Timeline dump for selected candidates: the per-device event lists that Algorithm 1 builds,
 * reduced to their stage-tasks (Sec. 3.2: the timeline says when which device computes and
 * communicates; Sec. 5.3 / 5.4 compare exactly these start and end timestamps).
 *   sel[n]       device: candidate indices (status must be OK after distsim_simulate, or after
 *                distsim_build_events with a stage table; other candidates, and indices outside
 *                [0, C), get no task entries and no all-reduce windows)
 *   task_off[n]  device: first entry of the candidate's block in start_ns / end_ns; the block
 *                holds 2*pp*m entries laid out [kind][stage][micro-batch], kind 0 = forward,
 *                1 = backward.  With p2p_blocking the end includes the send.  A candidate with
 *                the interleaved schedule has 2*pp*chunks*m entries, [kind][virtual stage]
 *                [micro-batch], virtual stage k on device k mod pp; one with an explicit schedule
 *                2*S*m entries in the same layout, -1 for tasks that its lists do not hold.
 *   ar_start_ns / ar_end_ns [n][DISTSIM_MAX_PP]: start of the first and end of the last gradient
 *                all-reduce event on each stage's device (interleaved: each device), -1 where
 *                there is none.
 * p2p events follow from the table: the one after task (kind, s, j) starts at that task's end
 * (its compute end) and lasts stage_tab[PF or PB].  `cand`: the candidates of the
 * distsim_build_events call.  Errors: EINVAL, ERANGE, ELIMIT, EHIP.
 */
int distsim_timeline(distsim_ctx *ctx, const distsim_cluster *cluster, const distsim_candidates *cand,
                     const distsim_events *events, int64_t n, const int64_t *sel, const int64_t *task_off,
                     int64_t *start_ns, int64_t *end_ns, int64_t *ar_start_ns, int64_t *ar_end_ns,
                     void *hip_stream);

/*
 * Bubble analysis of a timeline dumped by distsim_timeline (Sec. 3.2 names pipeline bubble
 * analysis as a use of the timeline; Sec. 5: the per-stage, per-micro-batch timestamps locate the
 * bubbles).  For the same sel / task_off and the start_ns / end_ns that distsim_timeline wrote,
 * idle_before_ns gets, in the same [kind][stage][micro-batch] layout, the time the stage's device
 * was idle in front of each stage-task: its start minus the end of the task the device ran before
 * it in the schedule's order (minus 0 for the device's first task).  Candidates that got no
 * timeline get nothing, nor do tasks that an explicit schedule does not list.  Errors: EINVAL, ELIMIT, EHIP.
 */
int distsim_bubbles(distsim_ctx *ctx, const distsim_candidates *cand, const distsim_events *events, int64_t n,
                    const int64_t *sel, const int64_t *task_off, const int64_t *start_ns, const int64_t *end_ns,
                    int64_t *idle_before_ns, void *hip_stream);

/*
 * Event generator (Sec. 4.1): operators that agree in name, parameters and input shape (and,
 * for communication, in the intra-/inter-node attribute) are one event and are profiled once.
 *   records[n][K]  device: one operator per row, K int64 words that identify it (how names and
 *                  shapes are encoded in words is the caller's business); 1 <= K <= 16
 *   event_id[n]    device out: the operator's event; events are numbered 0, 1, ... in the order
 *                  of their first operator
 *   rep[n]         device out: rep[e] = index of the first operator of event e, for
 *                  e < *num_events (the rest is left untouched)
 *   num_events     device out, one int64
 *   workspace      device memory of distsim_dedup_workspace_bytes(n) bytes
 * n <= 2^28.  Errors: EINVAL, ELIMIT, EHIP.
 */
size_t distsim_dedup_workspace_bytes(int64_t n);
int distsim_dedup_events(distsim_ctx *ctx, const int64_t *records, int64_t n, int32_t K,
                         int32_t *event_id, int32_t *rep, int64_t *num_events,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Elapsed time of communication events from their profiles (Sec. 4.2), all arrays device, [n]:
 *   kind 0  point-to-point: elapsed = min(t_a, t_b), the profiled durations of the SEND and of
 *           the RECV call (the transmission starts when the second of them is called)
 *   kind 1  all-reduce over ranks[i] devices: t_a is the profile on min(ranks, 8) devices;
 *           elapsed = t_a for up to 8 devices, else floor(t_a * 8 (N-1) / (7 N)), the ratio of
 *           the ring volumes 2(N-1)P/N at N and at 8 devices; t_b is ignored
 * A record of another kind, with ranks < 1 or with a negative time gets elapsed = -1.
 * Times below 2^62.  Errors: EINVAL, EHIP.
 */
int distsim_comm_event_times(distsim_ctx *ctx, int64_t n, const int32_t *kind, const int32_t *ranks,
                             const int64_t *t_a, const int64_t *t_b, int64_t *elapsed_ns,
                             void *hip_stream);

/*
 * Optional kernel timing with HIP events recorded on the caller's stream around each kernel
 * launch.  distsim_timing_read blocks until the recorded launches have finished and returns
 * the accumulated time and launch count of one kernel, then clears that kernel's record.
 * DISTSIM_K_SIMULATE spans the whole sweep of distsim_simulate, i.e. also the kernel that runs
 * beside it on the context's stream (DISTSIM_K_SIMULATE_GPIPE, timed there on its own);
 * DISTSIM_K_TIMELINE spans the packing of the selection and both dump kernels of the built-in
 * schedules (DISTSIM_K_TIMELINE_GPIPE is the second of them, timed on its own as well).
 */
enum {
    DISTSIM_K_LAYER_TABLES = 0, DISTSIM_K_DECODE, DISTSIM_K_BINS, DISTSIM_K_SCATTER,
    DISTSIM_K_STAGE_EVENTS, DISTSIM_K_SIM_INIT, DISTSIM_K_SIMULATE, DISTSIM_K_SEARCH, DISTSIM_K_TIMELINE,
    DISTSIM_K_DEDUP, DISTSIM_K_COMM_TIMES, DISTSIM_K_BUBBLES, DISTSIM_K_SIMULATE_VIRTUAL,
    DISTSIM_K_TIMELINE_VIRTUAL, DISTSIM_K_SIMULATE_GPIPE, DISTSIM_K_SIMULATE_EXPLICIT,
    DISTSIM_K_TIMELINE_EXPLICIT, DISTSIM_K_COMPILE_SCHEDULES, DISTSIM_K_TIMELINE_GPIPE, DISTSIM_K_COUNT
};
int distsim_timing_enable(distsim_ctx *ctx, int on);
int distsim_timing_read(distsim_ctx *ctx, int kernel, double *total_ms, int64_t *launches);
const char *distsim_kernel_name(int kernel);

#ifdef __cplusplus
}
#endif
#endif /* DISTSIM_H */

/*
 * ccld.h - C ABI of the MI355X decision-analyzer hot path of CCL-D.
 *
 * The library analyses per-rank collective-communication trace records on one
 * GPU: it groups them by Trace ID (communicator id, operation counter), computes
 * cross-rank statistics per collective, flags slow ranks, evaluates the paper's
 * slow-detection and slow-location rules, raises hang alerts, locates a hang's
 * root rank from Send/Recv progress counters, and accumulates per-rank blame.
 *
 * Conventions
 *  - "device" pointers are HIP device memory owned by the caller (for example a
 *    PyTorch tensor's data_ptr()); "host" pointers are ordinary host memory.
 *  - The library allocates no device memory: everything it needs lives in the
 *    caller's workspace (ccld_query_workspace / ccld_create).  It never frees or
 *    keeps caller memory other than that workspace.
 *  - All work is enqueued on the HIP stream given to ccld_create.  Calls that
 *    return counts (analyze, locate, blame) synchronise that stream before they
 *    return; ccld_ingest does not.
 *  - Every function returns a ccld_status: 0 = CCLD_OK, negative = error,
 *    positive = warning.  Nothing throws, aborts or prints.
 *  - Output tables are column-major int64 matrices: column c of a table with
 *    capacity CAP starts at table + c*CAP.  Unsigned fields (seq, bytes) are
 *    stored bit-for-bit.  When a table is too small its list is truncated, its
 *    count is still exact, and the status is CCLD_W_TRUNCATED.
 *  - All arithmetic is 64-bit integer; products are compared in 128 bits.
 */
#ifndef CCLD_H
#define CCLD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ccld_ctx ccld_ctx;
typedef int32_t ccld_status;

enum {
  CCLD_OK = 0,
  CCLD_E_UNKNOWN_COMM = -1,     /* a record names a communicator that is not in the topology        */
  CCLD_E_RANK_NOT_MEMBER = -2,  /* a record's rank is not a member of its communicator              */
  CCLD_E_RANGE = -3,            /* op >= 16, t_enter < 0 or == CCLD_T_INFLIGHT, t_exit < t_enter    */
  CCLD_E_DUPLICATE_KEY = -4,    /* two records (or snapshot rows) with the same key                 */
  CCLD_E_SNAPSHOT_GAP = -5,     /* a (snapshot, rank, communicator, channel) row is missing         */
  CCLD_E_BAD_ARG = -6,          /* parameter out of range                                           */
  CCLD_E_NULL = -7,             /* required pointer is NULL                                         */
  CCLD_E_CAPACITY = -8,         /* batch or window larger than the capacity given at create         */
  CCLD_E_KEY_WIDTH = -9,        /* communicator + sequence + rank bits do not fit in 64 bits        */
  CCLD_E_BAD_TOPOLOGY = -10,    /* malformed communicator table                                     */
  CCLD_E_HIP = -11,             /* a HIP runtime call failed                                        */
  CCLD_E_WORKSPACE = -12,       /* workspace too small or misaligned                                */
  CCLD_W_TRUNCATED = 1          /* an output list did not fit its table                             */
};

#define CCLD_T_INFLIGHT INT64_MAX     /* t_exit of an operation that has not completed              */
#define CCLD_NO_RANK 0xFFFFFFFFll
#define CCLD_OP_MAX 16                /* operation codes are 0..15                                  */

/* operation codes (Operation Type Set, Section 4.1.2); only ALLREDUCE has a meaning to the
 * analyzer (barrier filter), the others are labels */
enum { CCLD_OP_ALLREDUCE = 0, CCLD_OP_ALLGATHER = 1, CCLD_OP_REDUCESCATTER = 2, CCLD_OP_ALLTOALL = 3,
       CCLD_OP_SENDRECV = 4, CCLD_OP_BROADCAST = 5 };
enum { CCLD_ALGO_RING = 0, CCLD_ALGO_TREE = 1 };   /* Section 4.2.1: ring vs tree comparison groups */

/* Analyzer parameters; all integer, ratios as numerator/denominator.  Defaults in brackets. */
typedef struct {
  int64_t hang_threshold_ns;   /* [300e9] an operation in flight longer than this raises a hang alert (Sec. 4.2.1, 6.1) */
  int64_t tbase_init_ns;       /* [INT64_MAX/4] administrator-set initial baseline T_base^(init) (Eq. 1)    */
  uint32_t tbase_rounds;       /* [100] cap of m, the rounds averaged into the baseline (Eq. 1)             */
  uint32_t repeat_threshold;   /* [2] slow detections needed before location is triggered (Sec. 4.2.1)      */
  int64_t tbase_warmup_ns;     /* [120e9] rounds later than this after the first one end the warm-up (Eq. 1) */
  uint32_t theta_num, theta_den;          /* [3,1] slowdown threshold theta_slow (Eq. 3)                    */
  uint32_t alpha_num, beta_num, ab_den;   /* [4,6,10] boundaries alpha, beta of P (Eq. 4)                   */
  uint32_t barrier_bytes;      /* [4] an ALLREDUCE smaller than this is a barrier and is ignored (Sec. 4.2.1) */
  uint32_t kmad_num, kmad_den; /* [9,2] a rank is late when its lag exceeds kmad * MAD ...                  */
  int64_t lag_floor_ns;        /* [300000] ... and this floor (must exceed twice the clock skew)            */
  uint32_t stall_snapshots;    /* [30] a counter unchanged over this many snapshots is stalled              */
  uint32_t fifo_depth;         /* [8] ring back-pressure depth used by the wait-for edges                   */
  uint32_t window_batches;     /* [1] the window holds the last this-many ingested batches                  */
  uint32_t placement;          /* [CCLD_PLACEMENT_SORT] how ccld_analyze_window brings a collective's records together */
} ccld_params;

/* ccld_params.placement.  SORT: the window is sorted by (communicator, operation counter, rank).  DENSE: a
 * window of one batch is first analysed without sorting: every rank of a communicator bumps the same
 * operation counter (Section 5.1), so the Trace ID and the member slot fix a record's cell in a dense
 * (communicator, counter, member) grid, and one partition pass brings the records of a cell range together.
 * A window of several batches, a window with a round in which no member has a record or with counters
 * that are far apart, and a topology with a communicator of more than 2,048 members are sorted as under
 * SORT.  Both give the same tables; ccld_window_result.path tells which one ran. */
enum { CCLD_PLACEMENT_SORT = 0, CCLD_PLACEMENT_DENSE = 1 };

/* Communicator table (host pointers, copied by ccld_create). */
typedef struct {
  uint32_t n_ranks, n_comms;
  const uint8_t *algo;          /* [n_comms] CCLD_ALGO_*                                          */
  const uint32_t *size;         /* [n_comms] members per communicator                             */
  const uint32_t *member_off;   /* [n_comms] first slot of each communicator in members[]         */
  const uint32_t *members;      /* ranks; ring order (successor = next slot, cyclic) or BFS order */
  const int32_t *tree_parent;   /* per slot: parent's slot index inside the communicator, -1 = root; may be NULL */
} ccld_topology;

/* One batch of trace records, SoA (Section 5.1: Trace ID = communicator id + operation counter;
 * Section 4.1.2: Operation Type Set = op, bytes; Duration Time = t_exit - t_enter). */
typedef struct {
  const uint32_t *rank, *comm;
  const uint64_t *seq;
  const uint8_t *op;
  const uint64_t *bytes;
  const int64_t *t_enter, *t_exit;   /* ns; t_exit == CCLD_T_INFLIGHT while the operation runs   */
  int32_t on_device;                 /* 1: device pointers, 0: host pointers (copied synchronously) */
} ccld_records;

/* Progress-counter snapshots (Section 4.1.2 SendCount/RecvCount, per channel), SoA. */
typedef struct {
  const uint32_t *snap, *rank, *comm, *channel;
  const uint64_t *seq_posted;        /* operation counter of the operation the counters describe  */
  const uint32_t *chunks_sent, *chunks_recv;
  int32_t on_device;
  uint32_t n_snapshots;              /* snapshots are numbered 0 .. n_snapshots-1                   */
  uint32_t n_channels;               /* channels are numbered 0 .. n_channels-1                     */
} ccld_snapshots;

/* ---- table layouts ------------------------------------------------------------------------- */
/* segment table: one row per collective (communicator, operation counter), ordered by (comm, seq) */
enum { CCLD_SEG_COMM, CCLD_SEG_SEQ, CCLD_SEG_N, CCLD_SEG_INFLIGHT, CCLD_SEG_STATE, CCLD_SEG_OP, CCLD_SEG_BYTES,
       CCLD_SEG_ENTER_MIN, CCLD_SEG_ENTER_MED, CCLD_SEG_ENTER_MAX, CCLD_SEG_ENTER_MAD,
       CCLD_SEG_EXIT_MIN, CCLD_SEG_EXIT_MED, CCLD_SEG_EXIT_MAX, CCLD_SEG_EXIT_MAD,
       CCLD_SEG_DUR_MIN, CCLD_SEG_DUR_MAX, CCLD_SEG_ARGMIN_RANK, CCLD_SEG_ARGMAX_RANK,
       CCLD_SEG_INFLIGHT_ENTER_MIN, CCLD_SEG_FIRST, CCLD_SEG_NCOL };
/* CCLD_SEG_STATE bits */
enum { CCLD_SEG_COMPLETE = 1,    /* every member has a record and none is in flight              */
       CCLD_SEG_CONSISTENT = 2,  /* all records carry the same op and bytes                      */
       CCLD_SEG_BARRIER = 4,     /* ALLREDUCE of fewer than barrier_bytes bytes                  */
       CCLD_SEG_USABLE = 8 };    /* complete, consistent and not a barrier                       */
/* flag list: one row per late record, ordered by (comm, seq, rank) */
enum { CCLD_FLG_COMM, CCLD_FLG_SEQ, CCLD_FLG_RANK, CCLD_FLG_KIND, CCLD_FLG_LAG_ENTER, CCLD_FLG_LAG_EXIT,
       CCLD_FLG_NCOL };
enum { CCLD_FLAG_LATE_ENTER = 1, CCLD_FLAG_LATE_EXIT = 2 };
/* detection groups (communicator, op, floor(log2 bytes)), ordered by that triple */
enum { CCLD_GRP_COMM, CCLD_GRP_OP, CCLD_GRP_CLS, CCLD_GRP_N_USABLE, CCLD_GRP_RSTAR_SEQ, CCLD_GRP_TMAX,
       CCLD_GRP_TMIN, CCLD_GRP_TBASE, CCLD_GRP_STATIC, CCLD_GRP_FROZEN, CCLD_GRP_M, CCLD_GRP_SLOW,
       CCLD_GRP_CLASS, CCLD_GRP_ROOT_S1, CCLD_GRP_ROOT_S2, CCLD_GRP_REPEATS, CCLD_GRP_LOCATE, CCLD_GRP_NCOL };
enum { CCLD_SLOW_NONE = 0, CCLD_SLOW_S1_COMPUTATION = 1, CCLD_SLOW_S2_COMMUNICATION = 2, CCLD_SLOW_S3_MIXED = 3 };
/* hang alerts, ordered by (comm, seq); candidates of alert a are cand[off .. off+n) */
enum { CCLD_ALR_COMM, CCLD_ALR_SEQ, CCLD_ALR_AGE, CCLD_ALR_CLASS, CCLD_ALR_NCAND, CCLD_ALR_CAND_OFF,
       CCLD_ALR_NCOL };
enum { CCLD_HANG_H1_NOT_ENTERED = 1, CCLD_HANG_H2_INCONSISTENT = 2, CCLD_HANG_H3_HARDWARE = 3 };
/* per-rank blame */
enum { CCLD_BLM_N_LATE_ENTER, CCLD_BLM_N_LATE_EXIT, CCLD_BLM_SUM_LAG_ENTER, CCLD_BLM_SUM_LAG_EXIT,
       CCLD_BLM_N_RECORDS, CCLD_BLM_NCOL };

/* Result of ccld_analyze_window.  The caller fills capacities and device pointers; the
 * library fills the tables and, on return, the host-side counts and status. */
typedef struct {
  uint64_t seg_cap, flag_cap, group_cap, alert_cap, cand_cap;   /* in: rows                     */
  int64_t *seg;        /* device [CCLD_SEG_NCOL][seg_cap]                                        */
  int64_t *flag;       /* device [CCLD_FLG_NCOL][flag_cap]                                       */
  int64_t *group;      /* device [CCLD_GRP_NCOL][group_cap]                                      */
  int64_t *alert;      /* device [CCLD_ALR_NCOL][alert_cap]                                      */
  int64_t *cand;       /* device [cand_cap]                                                      */
  int64_t *lag_enter;  /* device [n_records] or NULL: t_enter - median, in sorted order, 0 on unusable rounds */
  int64_t *lag_exit;   /* device [n_records] or NULL                                             */
  uint8_t *rec_flag;   /* device [n_records] or NULL: CCLD_FLAG_* bits, in sorted order          */
  uint32_t *perm;      /* device [n_records] or NULL: window index of the j-th record in (comm, seq, rank) order */
  uint64_t n_records, n_seg, n_flag, n_group, n_alert, n_cand;  /* out (host)                   */
  ccld_status status;  /* out (host): CCLD_OK, a data error (counts are zero; table contents undefined), or CCLD_W_TRUNCATED */
  int32_t path;        /* out (host): 0 the window was sorted, 1 it was analysed by dense placement     */
} ccld_window_result;

/* Root cause and secondary effects among the late entries (ccld_flag_chains).
 * chain table: one row per row of the flag table, in the same order */
enum { CCLD_CHN_PARENT,     /* row of the flag that caused this late entry, -1: none (a root flag, or a late exit) */
       CCLD_CHN_ROOT,       /* first flag of the chain (the row itself for a root flag)                           */
       CCLD_CHN_ROOT_RANK,  /* rank of that flag                                                                  */
       CCLD_CHN_DEPTH,      /* links between the row and its root                                                 */
       CCLD_CHN_NCOL };
/* per rank: its late entries without / with a parent, and the late entries (of any rank) whose chain starts at
 * one of its root flags */
enum { CCLD_CHR_ROOT_ENTRIES, CCLD_CHR_SECONDARY_ENTRIES, CCLD_CHR_CAUSED, CCLD_CHR_NCOL };

typedef struct {
  uint64_t chain_cap;  /* in: rows                                                                   */
  int64_t *chain;      /* device [CCLD_CHN_NCOL][chain_cap]                                           */
  int64_t *per_rank;   /* device [CCLD_CHR_NCOL][n_ranks] or NULL                                     */
  uint64_t n_chain;    /* out (host): rows the full table has = flags of the analysis                */
  ccld_status status;  /* out (host)                                                                  */
  int32_t reserved;
} ccld_chain_result;

/* hang location tables */
/* roots, ordered by (rank, communicator) */
enum { CCLD_HROOT_RANK, CCLD_HROOT_COMM, CCLD_HROOT_CLASS, CCLD_HROOT_NCOL };
/* one row per member slot of every communicator, in the order of the topology's members[] */
enum { CCLD_HPAIR_RANK, CCLD_HPAIR_COMM, CCLD_HPAIR_STALLED, CCLD_HPAIR_ENTERED, CCLD_HPAIR_SEQ, CCLD_HPAIR_SENT,
       CCLD_HPAIR_RECV, CCLD_HPAIR_WAITS_ON, CCLD_HPAIR_HOPS, CCLD_HPAIR_ONSET, CCLD_HPAIR_NCOL };
/* one row per communicator */
enum { CCLD_HCOMM_COMM, CCLD_HCOMM_HUNG, CCLD_HCOMM_CLASS, CCLD_HCOMM_SEQ_MAX, CCLD_HCOMM_ROOT_BY_COUNT,
       CCLD_HCOMM_NCAND, CCLD_HCOMM_NCOL };

typedef struct {
  uint64_t root_cap, pair_cap, comm_cap;   /* in: rows                                             */
  int64_t *root;       /* device [CCLD_HROOT_NCOL][root_cap]                                        */
  int64_t *pair;       /* device [CCLD_HPAIR_NCOL][pair_cap] or NULL                                */
  int64_t *comm;       /* device [CCLD_HCOMM_NCOL][comm_cap] or NULL                                */
  uint64_t n_root, n_pair, n_hung_comm;    /* out (host)                                           */
  ccld_status status;  /* out (host)                                                                */
  int32_t reserved;
} ccld_hang_result;

/* progress-rate tables */
/* one row per member slot of every communicator, in the order of the topology's members[]:
 * operations observed and count changes observed, for SendCount and for RecvCount */
enum { CCLD_RATE_RANK, CCLD_RATE_COMM, CCLD_RATE_OPS_SEND, CCLD_RATE_CHANGES_SEND, CCLD_RATE_OPS_RECV,
       CCLD_RATE_CHANGES_RECV, CCLD_RATE_NCOL };
/* one row per communicator: the member of minimal SendRate, of minimal RecvRate, and of the minimal
 * of both kinds (CCLD_NO_RANK when no member has a rate) */
enum { CCLD_RCOMM_COMM, CCLD_RCOMM_ROOT_SEND, CCLD_RCOMM_ROOT_RECV, CCLD_RCOMM_ROOT, CCLD_RCOMM_NCOL };

typedef struct {
  uint64_t pair_cap, comm_cap;  /* in: rows                                                          */
  int64_t *pair;       /* device [CCLD_RATE_NCOL][pair_cap] or NULL                                   */
  int64_t *comm;       /* device [CCLD_RCOMM_NCOL][comm_cap] or NULL                                  */
  uint64_t n_pair, n_comm;      /* out (host): rows the full tables have                              */
  ccld_status status;  /* out (host)                                                                  */
  int32_t reserved;
} ccld_rate_result;

/* Probing Frames (Section 5.1): one 1184-byte frame per rank = 32-byte header + 8 blocks of 144
 * bytes; a block = one 16-byte Trace ID + 8 channels x {SendCount, RecvCount}.  Byte layout
 * (little-endian; the paper lists the fields, the widths are this library's):
 *   header: u64 kernel counter | u32 mode (bit 0: measurement on) | u32 kernelIndex | u32 channels | 12 reserved
 *   block : u32 communicator id | u32 extension (bit 0: block written) | u64 operation counter
 *           | 8 x { u64 SendCount, u64 RecvCount } */
enum { CCLD_FRAME_BYTES = 1184, CCLD_FRAME_HEADER_BYTES = 32, CCLD_FRAME_BLOCKS = 8, CCLD_FRAME_BLOCK_BYTES = 144,
       CCLD_FRAME_CHANNELS = 8 };

typedef struct {
  const uint8_t *frames;       /* [n_frames][CCLD_FRAME_BYTES], 16-byte aligned; host or device per on_device */
  const uint32_t *frame_rank;  /* [n_frames] rank each frame belongs to (same memory space as frames)        */
  uint64_t n_frames;
  int32_t on_device;
  uint32_t n_channels;         /* channels of the snapshot rows to write, 1 .. CCLD_FRAME_CHANNELS           */
  uint32_t snapshot;           /* snapshot number the rows get                                               */
  uint32_t reserved;
} ccld_frames;

/* snapshot rows written by ccld_decode_frames: device arrays of `capacity` entries each */
typedef struct {
  uint32_t *snap, *rank, *comm, *channel;
  uint64_t *seq_posted;
  uint32_t *chunks_sent, *chunks_recv;
  uint64_t capacity;
} ccld_snapshot_rows;

/* ---- entry points ---------------------------------------------------------------------------- */

/* Fills *params with the defaults listed above. */
ccld_status ccld_default_params(ccld_params *params);

/* Bytes of device workspace needed for windows of up to max_window_records records, batches of
 * up to max_batch_records and hang analyses of up to max_snapshot_rows rows. */
ccld_status ccld_query_workspace(const ccld_params *params, const ccld_topology *topo,
                                 uint64_t max_window_records, uint64_t max_batch_records,
                                 uint64_t max_snapshot_rows, uint64_t *bytes);

/* Creates an analyzer.  workspace: device memory of at least the queried size, 256-byte aligned,
 * owned by the caller and reserved for this context until ccld_destroy.  hip_stream: a hipStream_t
 * (NULL = the default stream).  The topology is copied. */
ccld_status ccld_create(const ccld_params *params, const ccld_topology *topo,
                        uint64_t max_window_records, uint64_t max_batch_records, uint64_t max_snapshot_rows,
                        void *workspace, uint64_t workspace_bytes, void *hip_stream, ccld_ctx **out);
ccld_status ccld_destroy(ccld_ctx *ctx);

/* Appends one batch of n records to the window (the analyzer works through the ranks' metrics
 * period by period, Section 3); when the window already holds window_batches batches the oldest
 * batch is dropped first.  The records are validated, keyed by Trace ID (communicator id, operation
 * counter; Section 5.1) plus the rank's position among the communicator's members, and stored on
 * the device.  Asynchronous for device input; data errors found on the device are reported by the
 * next ccld_analyze_window. */
ccld_status ccld_ingest(ccld_ctx *ctx, const ccld_records *batch, uint64_t n);

/* Drops every batch from the window; the per-group detection state (Eq. 1 baseline, repetition
 * counters) is kept. */
ccld_status ccld_reset_window(ccld_ctx *ctx);

/* Analyses the resident window (Sections 4.2.1 and 4.2.2): sorts the records by (communicator,
 * operation counter, rank); per collective computes earliest / lower-median / latest arrival and
 * completion, their median absolute deviations, T_min / T_max of the per-rank Duration Time with
 * the ranks attaining them, consistency of the Operation Type Set; flags late ranks; per detection
 * group applies Eq. 1 (baseline), Eq. 2 (round of largest range), Eq. 3 (slowdown ratio against
 * theta), Eq. 4 (P against alpha/beta, root = rank of minimal communication time) and the
 * repetition counter; raises hang alerts for operations in flight longer than the hang threshold
 * (barriers excepted) with the not-entered / inconsistent / hardware branch of the hang decision
 * tree.  now_ns is the analyzer's clock.  Per-rank blame of this window is kept for
 * ccld_rank_blame.  Returns out->status. */
ccld_status ccld_analyze_window(ccld_ctx *ctx, int64_t now_ns, ccld_window_result *out);

/* Separates root cause from secondary effects among the late-entry flags of the most recent
 * ccld_analyze_window (Section 4.2.2: in a large cluster an anomaly propagates across ranks, and the
 * location step has to tell the rank that triggered it from the ranks that pass it on).  `analysed` is
 * the result of that analysis (its collective table must hold every collective: n_seg <= seg_cap) and no
 * other call on the context may lie in between (else CCLD_E_BAD_ARG).  Per late entry F of rank r: the
 * operation r ran just before = r's completed record with the largest t_exit <= t_enter(F), on r's own
 * clock (ties: larger t_enter, then larger communicator); among that operation's late entries the one
 * with the largest lag (ties: smallest rank) ended it late and is F's parent, also when it is r's own;
 * without a late entry there F is a root flag: r is late of its own.  Late exits have no parent.  Parents
 * are followed to the chain's first flag.  A delay that a whole communicator carries in step for several
 * operations leaves no late entry there, so a chain can end before it reaches the rank that injected the
 * delay: the chains separate the direct consequences, not every later echo. */
ccld_status ccld_flag_chains(ccld_ctx *ctx, const ccld_window_result *analysed, ccld_chain_result *out);

/* Locates the root of a hang from progress-counter snapshots (Section 4.2.2, hang decision tree;
 * Section 4.1.2, SendCount / RecvCount; Section 4.2.1, ring vs tree comparison groups).  The n_rows
 * rows must fill the grid snapshots x (communicator, member) x channels exactly once, in any order
 * (otherwise CCLD_E_SNAPSHOT_GAP / CCLD_E_DUPLICATE_KEY; the grid must fit max_snapshot_rows).
 * Per (rank, communicator): stalled iff every channel's (operation counter, sent, received) is the
 * same at the last snapshot and stall_snapshots earlier; entered iff its operation counter equals
 * the communicator's largest.  A communicator is hung iff a member is stalled and it is not idle
 * (all entered with identical totals across the ring, or inside each layer of the tree).  Per hung
 * communicator the paper's tree is applied: members that have not entered are the root
 * (Not-Entered-Hang); else members that are not stalled (Inconsistent-Hang); else (Hardware-Fault)
 * the ring's wait-for edges are walked (a rank that consumed all its predecessor sent waits on the
 * predecessor, a rank whose successor holds fifo_depth unconsumed chunks waits on the successor)
 * and the ranks that wait on nobody are the root, or in a tree the ranks furthest behind their
 * layer; with no such rank, the rank with the fewest SendCount + RecvCount.  A not-entered rank
 * that has entered another hung communicator is a victim and is dropped. */
ccld_status ccld_locate_hang(ccld_ctx *ctx, const ccld_snapshots *snapshots, uint64_t n_rows,
                             ccld_hang_result *out);

/* For callers that cannot allocate device memory (code under HIP graph capture set-up, tight serving
 * loops, harnesses that forbid hipMalloc) and whose context was created with max_snapshot_rows = 0:
 * ccld_locate_hang with every buffer of the pass (the snapshot grid, the per-member and
 * per-communicator tables, the root list's sort buffers, staging for host-resident rows) taken from a
 * static device array of CCLD_STATIC_SCRATCH_BYTES bytes that the library holds on every GPU it runs
 * on until the process ends, instead of from the context's workspace.  Inputs, outputs, results and
 * error behaviour are those of ccld_locate_hang, except that the capacity limit is the array: a grid
 * (member slots x channels x snapshots, 16 bytes per cell, plus about 200 bytes per member slot and
 * 32 bytes per host-resident row) that does not fit returns CCLD_E_CAPACITY.  The call allocates and
 * frees nothing.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (from several contexts, streams or threads) race; everything the pass needs cleared is cleared by
 * the call itself.  The context's window state is left alone (its sort buffers are not borrowed). */
#define CCLD_STATIC_SCRATCH_BYTES (32u << 20)
ccld_status ccld_locate_hang_static(ccld_ctx *ctx, const ccld_snapshots *snapshots, uint64_t n_rows,
                                    ccld_hang_result *out);

/* SendRate / RecvRate of every (communicator, member) from a series of SendCount / RecvCount
 * snapshots (Section 4.1.2, slow diagnostic metrics): the rate is the reciprocal of the number of
 * times the count changes from one sample to the next while an operation runs, so a rank whose
 * transfers are slow shows more changes for the same operation.  Rows, validation and capacity as
 * for ccld_locate_hang.  Per (member, channel) the series is cut into runs of equal operation
 * counter; the last run is still open and is left out; inside a run a sample is compared with the
 * previous one, the run's first sample with zero; a run with at least one change counts as one
 * observed operation.  Per member the operations and changes are summed over channels: its rate is
 * ops / changes (undefined without a change; rates are compared by cross-multiplication, ties go
 * to the smaller rank).  The communicators' minimal-rate members (CCLD_RCOMM_ROOT) stay in the
 * context: from then on ccld_analyze_window reports them as CCLD_GRP_ROOT_S2 of communication-slow
 * and mixed groups (Section 4.2.1, Eq. 4: the rank of minimal SendRate / RecvRate is the root of a
 * communication slowdown).  Before the first call that column holds CCLD_NO_RANK. */
ccld_status ccld_progress_rates(ccld_ctx *ctx, const ccld_snapshots *snapshots, uint64_t n_rows,
                                ccld_rate_result *out);

/* Decodes one Probing Frame per rank into the rows of one snapshot (the input of ccld_locate_hang
 * and ccld_progress_rates).  Per frame and communicator the written block with the largest
 * operation counter (then the largest block index) is the rank's latest kernel there; it replaces
 * what the context remembers for (rank, communicator) unless that is newer.  Communicators that are
 * absent from a frame (a frame only holds the rank's latest 8 kernels) keep their remembered state.
 * Then one row per member slot (in the order of the topology's members[]) and channel
 * 0 .. n_channels-1 is written: *n_rows = member slots x n_channels rows, which must fit
 * rows->capacity (else CCLD_E_CAPACITY).  Channels beyond a frame's own channel count read zero.
 * Checked, in this order of precedence: unknown communicator, rank not a member (or no such rank),
 * range (a header with more than 8 channels, a count above 2^32 - 1), two frames of one rank
 * (CCLD_E_DUPLICATE_KEY).  On an error nothing is remembered and no row is written.
 * ccld_reset_frames forgets every remembered state. */
ccld_status ccld_decode_frames(ccld_ctx *ctx, const ccld_frames *frames, const ccld_snapshot_rows *rows,
                               uint64_t *n_rows);
ccld_status ccld_reset_frames(ccld_ctx *ctx);

/* Per-rank blame of the most recent ccld_analyze_window: blame = device [CCLD_BLM_NCOL][n_ranks]
 * (late-entry and late-exit counts, their summed lags, records seen); order = device [n_ranks]
 * ranks sorted by (number of flags descending, summed lag descending, rank ascending).  Either
 * pointer may be NULL.  The first entries of order[] name the faulty rank(s): locating the faulty
 * GPU rank is the analyzer's stated purpose (Section 1). */
ccld_status ccld_rank_blame(ccld_ctx *ctx, int64_t *blame, uint32_t *order);

/* Optional timing of the library's kernels with HIP events recorded on the context's stream, by
 * kernel class.  ccld_profile_enable(ctx, 1) clears the accumulators and starts timing every class
 * in the following calls; ccld_profile_enable(ctx, 2 + class) times that one class only (every
 * event record costs several microseconds on the stream); 0 stops.  ccld_profile_read copies the
 * accumulated milliseconds and launch counts (host arrays of CCLD_PROF_NCLASS entries). */
enum { CCLD_PROF_INGEST, CCLD_PROF_SORT_HIST, CCLD_PROF_SORT_SCAN, CCLD_PROF_SORT_SCATTER, CCLD_PROF_SEGMENTS,
       CCLD_PROF_FLAGS, CCLD_PROF_BLAME, CCLD_PROF_GROUPS, CCLD_PROF_ALERTS, CCLD_PROF_HANG,
       CCLD_PROF_SEG_HEADS, CCLD_PROF_DENSE_PARTITION, CCLD_PROF_HANG_PLACE, CCLD_PROF_FRAMES,
       CCLD_PROF_NCLASS = 16 };
ccld_status ccld_profile_enable(ccld_ctx *ctx, int32_t on);
ccld_status ccld_profile_read(ccld_ctx *ctx, double *ms, uint64_t *launches, uint64_t *sort_passes);

const char *ccld_status_str(ccld_status s);

#ifdef __cplusplus
}
#endif
#endif /* CCLD_H */

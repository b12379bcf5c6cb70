/*
 * ftred - round-synchronous execution of the correction-based fault-tolerant
 * reduce and allreduce over P virtual processes and a batch of S failure
 * scenarios on one MI355X (gfx950).
 *
 * Method: Kuettler & Haertig, "Fault-tolerant Reduce and Allreduce operations
 * based on correction".  Citations below name that paper's sections,
 * algorithms and theorems.
 *
 * Conventions of every entry point
 *   - returns an int code (FTRED_OK = 0); never throws, never aborts.  On an
 *     error the message is available from ftred_last_error() (thread-local).
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host"
 *     pointers are host memory.  The library owns only the plan.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work on that stream and return without waiting, except
 *     where stated.
 *   - ranks in arguments and results are PHYSICAL ranks 0..P-1; the relabelling
 *     that makes the root number 0 (section "Reduce", first paragraph) is
 *     internal.
 *   - a scenario = one independent execution of the operation with its own
 *     failure set (and payload, root).  Argument errors give FTRED_EINVAL;
 *     errors in the DATA of one scenario give a per-scenario status and the run
 *     goes on for the others.
 *
 * Failure model (sections "Failures", "Reduce / Semantics"; rounds are this
 * library's execution model): per scenario f slots (fail_rank, fail_round).
 * fail_rank = FTRED_NO_RANK marks an unused slot.  fail_round = 0: the process
 * failed before the operation.  fail_round = r >= 1: the process performs all
 * sends of global rounds < r and nothing from round r on (fail-stop).  Global
 * rounds count from 1; in an allreduce they keep counting over the attempts.
 * A message that is missing in the round it has in the failure-free run tells
 * the receiver that the sender failed.
 */
#ifndef FTRED_H
#define FTRED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ftred_plan_s ftred_plan_t;   /* opaque; created by ftred_plan, freed by ftred_plan_destroy */

enum { FTRED_OK = 0, FTRED_EINVAL = 1, FTRED_ENOMEM = 2, FTRED_EDEVICE = 3, FTRED_EUNSUPPORTED = 4 };

/* element type of the payload */
enum { FTRED_I64 = 0, FTRED_U32 = 1, FTRED_F64 = 2 };

/* reduction function (section "Reduce": associative and commutative).
   SUM wraps for the integer types; BOR (bitwise or) is for integer types only. */
enum { FTRED_SUM = 0, FTRED_BOR = 1 };

/* per-scenario status */
enum {
    FTRED_ST_OK = 0,
    FTRED_ST_ROOT_FAILED = 1,        /* reduce only: the root failed, the operation is a no-op
                                        (section "Reduce / Algorithm") */
    FTRED_ST_NO_CLEAN_SUBTREE = 2,   /* the root found no child reporting "no failure" (Algorithm
                                        "reduce, root"); impossible with <= f failures (third theorem) */
    FTRED_ST_BAD_FAILURE_SET = 3     /* a rank >= P, a rank listed twice, a root >= P, or (allreduce) a
                                        root candidate 0..f listed with fail_round != 0; nothing is
                                        simulated, outputs of the scenario are zero */
};

#define FTRED_NO_RANK 0xFFFFFFFFu
#define FTRED_MAX_F 15u

/* ftred_validate verdict bits (0 = valid) */
enum {
    FTRED_BAD_VALUE = 1,      /* result is not the reduction over the never-failed processes plus one
                                 subset of the processes that failed during the operation */
    FTRED_BAD_HOLDER = 2,     /* allreduce: a never-failed process does not hold the result, or holds
                                 another value; or a process failed beforehand is marked as holder */
    FTRED_BAD_STATUS = 4,     /* status does not match the failure set (e.g. OK with a failed root) */
    FTRED_BAD_COUNT = 8       /* message counters outside what the message-count theorems allow */
};

typedef struct ftred_info {
    uint32_t P, f, elems, dtype, op;
    uint32_t groups_full;        /* floor((P-1)/(f+1)) up-correction groups of f+1 processes */
    uint32_t a;                  /* ((P-1) mod (f+1)) + 1; the root is in a group iff a > 1 */
    uint32_t D;                  /* height of the tree (rounds of the tree phase) */
    uint32_t rounds_reduce;      /* f + D */
    uint32_t rounds_attempt;     /* 2 (f + D): reduce, broadcast down the tree, f correction rounds */
    uint32_t tiers;              /* kernel launches of one tree phase */
    uint32_t deep_kernel;        /* deepest tier: 0 = LDS tiles, 1 = registers, one lane per subtree,
                                    2 = registers, eight lanes per subtree (elems == 1) */
    uint64_t msgs_uc_ff;         /* failure-free up-correction messages (message-count theorem) */
    uint64_t msgs_tree_ff;       /* failure-free tree messages = P - 1 */
    uint64_t msgs_bcast_tree_ff; /* failure-free broadcast tree messages = P - 1 */
    uint64_t msgs_bcast_corr_ff; /* failure-free broadcast correction messages (= msgs_uc_ff) */
    uint32_t fused;              /* 1: with deep_kernel 1, one workgroup folds the deepest tier and the levels above
                                    it in a single launch: a whole scenario down to the root's choice, or, where the
                                    top rows of a scenario's subtrees do not fit its LDS tile, the part of the tree
                                    below one row (the few levels above those rows then take one more launch) */
    uint32_t shape;              /* tree inside a subtree of the root: 2, k, or 1 = binomial (ftred_plan, flags) */
    /* message steps of one failure-free attempt, one port per process: per kind of message (up-correction, tree,
       broadcast down the tree, broadcast correction) the sum over its rounds of the number of messages the
       busiest process sends or receives in the round (see ftred_detect); all 0 for trees of more than 2^22
       processes per subtree, for which they are not worked out */
    uint32_t steps_uc, steps_tree, steps_bcast_tree, steps_bcast_corr;
    uint32_t reserved;
} ftred_info_t;

/* Create a plan for P processes, failure bound f, `elems` values of `dtype` per
   process and reduction `op`.  Requires P >= f + 2 (the root needs f+1 children:
   definition of the I(f)-tree), f <= FTRED_MAX_F, elems >= 1, P * elems * size
   < 2^31 bytes, no BOR on FTRED_F64.  Payloads of more than 64 values per process
   run as blocks of value indices with one failure pattern; a payload whose
   up-correction group fits no LDS tile where the tree is too shallow for the
   register kernels runs on the plain per-depth kernels of the other tree shapes
   (below).  flags: 0 for the defaults; tuning knobs of
   the tree kernels otherwise: bits 0..7 = LDS budget in KiB of the deepest tier's
   tiles (4..24), bits 8..11 = 1 + log2 of the tiles one workgroup walks through,
   bit 12 = LDS-tile kernel also for the deepest tier (the default there is a
   register kernel when the tree is deep enough: one lane per subtree, or eight
   lanes per subtree when elems == 1; for f + 1 >= 10 only while 31 up-correction
   groups of f + 1 payloads fit 24 KiB),
   bits 13..15 = 1 + log2 of the groups of subtrees one wavefront of the register
   kernel walks through, bit 16 = the deepest tier and the levels above it always in
   launches of their own (the default folds a whole scenario in one workgroup and
   one launch where the levels above the deepest tier fit its LDS tile),
   bits 17..19 = 1 + log2(KiB / 4) of the receive buffers one workgroup of the
   broadcast writes (4 .. 64 KiB).
   bits 20..26 = the shape of the tree inside each subtree of the root, which the
   definition of the I(f)-tree leaves free: 0 or 2 = two children per process,
   filled breadth-first (the default: the tree of the paper's second tree figure);
   k = 3..64 = k children per process, filled breadth-first; 1 = the binomial tree
   built by doubling (the j-th process of a subtree, j >= 1, is a child of process
   j - 2^floor(log2 j)).  Values under failures before the operation and all
   message counts of the reduce do not depend on the shape; the number of rounds
   (ftred_info.D) and what a failure during the operation does do.  Other shapes
   than the default run on plain kernels (one launch per depth of the tree, a
   workspace as large as the payload) and do not carry the lists of failed
   processes (the _info entry points return FTRED_EUNSUPPORTED).
   Host call; no device work. */
int ftred_plan(ftred_plan_t **out, uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, uint32_t flags);
int ftred_plan_info(const ftred_plan_t *plan, ftred_info_t *info /* host, written */);
void ftred_plan_destroy(ftred_plan_t *plan);
const char *ftred_last_error(void);      /* never NULL; valid until the thread's next failing call */

/* The hash of the sources this library was built from (hex sha256 over the HIP
   sources and headers, computed by the build); never NULL, "unknown" for a build
   that did not pass one.  Lets a binding refuse a library that is older than the
   sources beside it. */
const char *ftred_source_hash(void);

/* Bytes of device workspace a run or validation of S scenarios needs. */
uint64_t ftred_workspace_bytes(const ftred_plan_t *plan, uint32_t S);

/* Index arithmetic of one process (host call, no device work): the tree of
   section "Reduce / Properties" (definition of the I(f)-tree; subtree rule of
   the replication theorem's proof) and the up-correction group of section
   "Up-Correction", for operation root `root`.  All ranks physical.
   parent = FTRED_NO_RANK for the root; children: up to f+1 entries for the root,
   two otherwise (k in a k-ary tree, up to 32 in a binomial tree); group[0..group_size) in group order (empty if the process is in
   no group), group_pos = own index in it; subtree = 0 for the root else 1..f+1;
   send_round = round of the tree message inside one reduce (0 for the root). */
typedef struct ftred_partners {
    uint32_t parent;
    uint32_t n_children;
    uint32_t children[32];
    uint32_t group_size, group_pos;
    uint32_t group[FTRED_MAX_F + 1];
    uint32_t subtree, depth, height, send_round;
} ftred_partners_t;
int ftred_partners(const ftred_plan_t *plan, uint32_t root, uint32_t rank, ftred_partners_t *out /* host */);

/* The same arithmetic evaluated on the GPU for every rank (device index functions
   as used by the kernels): each output is dev [P] uint32 or NULL. */
int ftred_structure(const ftred_plan_t *plan, uint32_t root,
                    uint32_t *parent, uint32_t *subtree, uint32_t *group_id, uint32_t *group_pos,
                    uint32_t *group_size, uint32_t *depth, uint32_t *send_round, void *hip_stream);

/* S fault-tolerant reduces (Algorithms "Up-correction", "reduce at non-roots",
   "reduce at the root"; failure information = the single failed bit of section
   "Failure information").
     root        dev [S] root of each scenario, or NULL = 0
     payload     dev [S][P][elems] input of every process; scen_stride_elems =
                 distance between scenarios in elements (P*elems when packed,
                 0 = one payload shared by all scenarios)
     fail_rank, fail_round  dev [S][max(f,1)]
     result      dev [S][elems] value returned at the root (zeros unless status OK)
     status      dev [S]
     msgs        dev [S][2] uint64 {up-correction, tree} messages sent, or NULL
     workspace   dev, ftred_workspace_bytes(plan, S) bytes, 256-byte aligned
   The root delivers iff it is alive in the last round f + D.  Among several
   children reporting "no failure" the root takes the lowest-numbered one. */
int ftred_run_reduce(const ftred_plan_t *plan, uint32_t S, const uint32_t *root,
                     const void *payload, uint64_t scen_stride_elems,
                     const uint32_t *fail_rank, const uint32_t *fail_round,
                     void *result, uint32_t *status, uint64_t *msgs,
                     void *workspace, uint64_t workspace_bytes, void *hip_stream);

/* S fault-tolerant allreduces (Algorithm "Allreduce"): reduce to root r, broadcast
   from r, retry with r+1 while r had failed; roots tried are ranks 0,1,..,f and
   may fail only before the operation (section "Allreduce / Description").  The
   broadcast sends the value down the same tree (D rounds) and then runs f
   correction rounds in the up-correction groups (every holder sends to one group
   mate per round).
     result          dev [S][elems] the value every surviving process holds
     has_bitmap      dev [S][ceil(P/32)] bit p%32 of word p/32 = process p holds it; or NULL
     per_process_out dev [S][P][elems] receive buffer of every process (zeros for
                     processes that hold nothing); or NULL
     attempts        dev [S] roots tried; msgs dev [S][4] uint64 {up-correction, tree,
                     broadcast tree, broadcast correction} over all attempts, or NULL */
int ftred_run_allreduce(const ftred_plan_t *plan, uint32_t S,
                        const void *payload, uint64_t scen_stride_elems,
                        const uint32_t *fail_rank, const uint32_t *fail_round,
                        void *result, uint32_t *has_bitmap, void *per_process_out,
                        uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                        void *workspace, uint64_t workspace_bytes, void *hip_stream);

/* ftred_run_allreduce for callers that cannot allocate device memory (code under
   HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
   same operation, arguments and results, but the workspace is a fixed array of
   FTRED_NOALLOC_WORKSPACE_BYTES in device memory that belongs to the library
   (every GPU the library runs on holds its own copy until the process ends).
   The call allocates and frees nothing; it enqueues kernels on the caller's
   stream like ftred_run_allreduce.  Returns FTRED_EUNSUPPORTED, with nothing
   enqueued, when ftred_workspace_bytes(plan, S) exceeds the array: use fewer
   scenarios per call.  All calls on one GPU share that GPU's array, which keeps
   what the last call left (the run clears what it needs to find zero): calls
   whose kernels may overlap on one GPU, on different streams or from different
   threads, race on it and must be ordered by the caller. */
#define FTRED_NOALLOC_WORKSPACE_BYTES (32u * 1024u * 1024u)
int ftred_run_allreduce_noalloc(const ftred_plan_t *plan, uint32_t S,
                                const void *payload, uint64_t scen_stride_elems,
                                const uint32_t *fail_rank, const uint32_t *fail_round,
                                void *result, uint32_t *has_bitmap, void *per_process_out,
                                uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                                void *hip_stream);

/* The same operations with the two richer failure descriptions of section
   "Failure information" carried by the tree messages beside the failed bit: the
   list of the processes a sender and its descendants could not receive a value
   from, in the up-correction phase and in the tree phase (first scheme), and the
   length of that list (second scheme).  The value, the status and the counters
   are those of ftred_run_reduce / ftred_run_allreduce: which child the root
   selects depends on the failed bit alone.  Extra outputs (each may be NULL, not
   all three); for the allreduce they describe the reduce of the last attempt:
     info_count  dev [S] length of the list carried by the message the root selected
     info_ids    dev [S][max(f,1)] that list: ranks in the order of the scenario's
                 failure list, padded with FTRED_NO_RANK
     info_child  dev [S][f+1] what the root holds from child k+1 (the top of subtree
                 k+1) at the end: bits 16..17 = 0 no message, 1 message without the
                 failed bit, 2 message with it; bits 0..15 = its list as a set of
                 slots of the scenario's failure list (bit q = fail_rank[s][q])
   All three are zero / FTRED_NO_RANK for a scenario without a result. */
int ftred_run_reduce_info(const ftred_plan_t *plan, uint32_t S, const uint32_t *root,
                          const void *payload, uint64_t scen_stride_elems,
                          const uint32_t *fail_rank, const uint32_t *fail_round,
                          void *result, uint32_t *status, uint64_t *msgs,
                          uint32_t *info_count, uint32_t *info_ids, uint32_t *info_child,
                          void *workspace, uint64_t workspace_bytes, void *hip_stream);
int ftred_run_allreduce_info(const ftred_plan_t *plan, uint32_t S,
                             const void *payload, uint64_t scen_stride_elems,
                             const uint32_t *fail_rank, const uint32_t *fail_round,
                             void *result, uint32_t *has_bitmap, void *per_process_out,
                             uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                             uint32_t *info_count, uint32_t *info_ids, uint32_t *info_child,
                             void *workspace, uint64_t workspace_bytes, void *hip_stream);

/* Latency bookkeeping.  The paper names no cost model; its setting is latency-critical
   small messages (Introduction), and a receiver that waits for a failed sender times
   out and asks the failure monitor (section "Up-Correction", last paragraph).  This
   library's reading: an attempt of S scenarios' operation costs
       t_message * (steps of the plan, ftred_info.steps_*: a round takes as many message
                    steps as its busiest process sends or receives messages, failure-free)
     + t_timeout * (number of DETECTED processes),
   where a listed process is detected when some process that is alive finds, in the round
   in which it acts on it, that a message of the failure-free schedule has not come, and
   the process has indeed failed by then.  ftred_detect works that out from the failure
   lists alone (kind 0 = reduce with `root` (dev [S] or NULL), 1 = allreduce over all its
   attempts): detected dev [S], bit q = the process in slot q of the scenario's failure
   list was detected; 0 for a scenario whose failure set is not valid.  The number of
   attempts, and with it the total of message steps, is what ftred_run_allreduce returns
   in `attempts`. */
int ftred_detect(const ftred_plan_t *plan, int kind, uint32_t S, const uint32_t *root,
                 const uint32_t *fail_rank, const uint32_t *fail_round,
                 uint32_t *detected, void *hip_stream);

/* Event-driven times of the reduce.  In the paper a process runs its phases one after
   the other without regard to the progress of the others (section "Related work", last
   paragraph), and a receive from a failed sender ends by a time-out and the failure
   monitor's confirmation, and is retried while the monitor says the sender lives
   (section "Up-Correction", last paragraph; liveness part of the proof in "Reduce /
   Properties").  This library's model of that: every process starts at time 0 with a
   clock of its own; it exchanges with its up-correction group (round t: send to its
   target, then receive from its source), receives from its children in ascending
   order, sends to its parent; the root receives from its children in order until a
   message without the failed bit is there.  A send takes t_msg of the sender's time
   and the message is at the receiver when the send ends; a receive ends at once if
   the message is there, at its arrival otherwise; if the sender has stopped without
   sending it, the receiver asks the monitor after every t_timeout of waiting and
   gives up at the first such moment that lies AFTER the moment the sender stopped.
   A process with fail_round r stops when it reaches the first step of a round >= r
   (rounds as in ftred_run_reduce).  What is sent and received is what the round model
   sends and receives, so results, statuses and counters are ftred_run_reduce's; this
   call works out the clocks, from the failure lists alone (no payload):
     t_done dev [S]     the moment the root delivers (status NO_CLEAN_SUBTREE: the moment
                        it has gone through all its children); FTRED_NEVER for a root that
                        has failed and for a failure set that is not valid
     t_proc dev [S][P]  required, also the working storage: the moment each process has
                        done its part (sent to its parent; the root: t_done), by physical
                        rank; FTRED_NEVER for a process that stops before
   root dev [S] or NULL (process 0).  t_msg, t_timeout in 1 .. 2^32 - 1.  One launch per
   depth of the tree and one for the roots, on hip_stream. */
#define FTRED_NEVER 0xFFFFFFFFFFFFFFFFull
int ftred_reduce_times(const ftred_plan_t *plan, uint32_t S, const uint32_t *root,
                       const uint32_t *fail_rank, const uint32_t *fail_round,
                       uint64_t t_msg, uint64_t t_timeout,
                       uint64_t *t_done, uint64_t *t_proc, void *hip_stream);

/* Check results against the semantics (sections "Reduce / Semantics", items 3
   and 4, and "Allreduce / Semantics", items 4 and 5; message-count theorems),
   independently of the protocol: per scenario the reduction over the never-failed
   processes is recomputed from the payload, and the result must equal it combined
   with one subset of the processes that failed during the operation (integers:
   exactly; FTRED_F64: within 1e-12 * sum of |x| per element).  kind 0 = reduce,
   1 = allreduce.  has_bitmap / per_process_out / msgs may be NULL (not checked).
   verdict dev [S] gets FTRED_BAD_* bits; *n_invalid (host, may be NULL) gets the
   number of scenarios with verdict != 0: when it is not NULL the call waits for
   the stream. */
int ftred_validate(const ftred_plan_t *plan, int kind, uint32_t S, const uint32_t *root,
                   const void *payload, uint64_t scen_stride_elems,
                   const uint32_t *fail_rank, const uint32_t *fail_round,
                   const void *result, const uint32_t *has_bitmap, const void *per_process_out,
                   const uint32_t *status, const uint32_t *attempts, const uint64_t *msgs,
                   uint32_t *verdict, uint64_t *n_invalid,
                   void *workspace, uint64_t workspace_bytes, void *hip_stream);

/* Counter-based failure scenarios on the device (Philox4x32-10, counter =
   (scenario, slot, draw, stream), key = seed): k uniform in 0..f failed ranks per
   scenario, uniform without replacement; each failure happens during the operation
   with probability inop_permille/1000 at a round uniform in 1..A*rounds_per_attempt
   (A = 1 + number of leading ranks 0,1,.. below `protected_ranks` in the set), else
   before the operation; ranks below protected_ranks always fail before it.
   root_out (dev [S] or NULL) gets a uniform root per scenario.
   fail_rank, fail_round: dev [S][max(f,1)], written.  Scenario ids scen0..scen0+S-1. */
int ftred_gen_failures(const ftred_plan_t *plan, uint64_t seed, uint32_t S, uint32_t scen0,
                       uint32_t inop_permille, uint32_t rounds_per_attempt, uint32_t protected_ranks,
                       uint32_t *root_out, uint32_t *fail_rank, uint32_t *fail_round, void *hip_stream);

/* Counter-based integer payloads on the device, same generator: payload dev
   [S][P][elems] of the plan's integer dtype, each value `bits` random bits
   (FTRED_I64: minus 2^(bits-1), i.e. uniform in [-2^(bits-1), 2^(bits-1))). */
int ftred_gen_payload_int(const ftred_plan_t *plan, uint64_t seed, uint32_t S, uint32_t scen0,
                          uint32_t bits, void *payload, void *hip_stream);

/* Per-kernel timing with HIP events, for benchmarks: between ftred_timing_begin and
   ftred_timing_end every kernel the library launches is bracketed by two events
   recorded on the stream it is launched on (up to max_records launches; later ones
   are not timed).  ftred_timing_end waits for the recorded events, adds up the
   elapsed milliseconds and the number of launches per phase (arrays of
   FTRED_PH_COUNT entries, host, either may be NULL), frees the events and switches
   timing off.  For benchmarks only: the state is process-wide and not
   thread-safe, so while timing is on (and during the two calls themselves) no
   other thread may call into the library; callers that time several streams get
   the sum over them. */
enum {
    FTRED_PH_CHECK = 0,        /* scenario check */
    FTRED_PH_RETRY = 1,        /* attempts with a failed root */
    FTRED_PH_TREE_DEEP = 2,    /* up-correction + deepest tier of the tree phase (reads the payload) */
    FTRED_PH_TREE_UPPER = 3,   /* upper tiers and the root's choice */
    FTRED_PH_BCAST = 4,        /* broadcast: holders and receive buffers */
    FTRED_PH_VAL_PARTIAL = 5,  /* validation pass 1 */
    FTRED_PH_VAL_FINAL = 6,    /* validation pass 2 */
    FTRED_PH_GEN = 7,          /* scenario / payload generation */
    FTRED_PH_COUNT = 8
};
int ftred_timing_begin(uint32_t max_records);
int ftred_timing_end(double *ms, uint64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* FTRED_H */
